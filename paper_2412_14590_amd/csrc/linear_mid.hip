// Path for a few dozen tokens (17 <= M <= 64): still bound by the weight stream, but with too
// many tokens for the decode kernels (whose LDS stage holds the whole activation matrix) and too
// few for the tiled kernel (its 128 x 128 block tiles leave most CUs idle and its K loop is
// serial per block: ~25 us on any layer of K = 4096).
//  * Work is dealt as in the evenly split decode variant: a block takes an equal share of the
//    quarter tiles (4 channels x all of K) of one precision; 4 consecutive quarter tiles form
//    the 16-column virtual tile of one wave (the last one of a share may be partly filled), and a wave owns its virtual tile for all of K: its accumulators (MT token tiles of
//    16 x 16) stay in registers, nothing is reduced between waves.  A block with more than 8
//    virtual tiles walks K once per round of 8.
//  * The loop runs over K in steps of 4 groups (512 k).  The int8 activations of a step, M x 512
//    bytes, are staged in LDS straight from global memory (`global_load_lds_dwordx4`, rows of
//    128 bytes per group with the 16-byte chunks swizzled so that a fragment read is free of
//    bank conflicts), three buffers; every wave streams the 4 groups of
//    its own virtual tile (4 KB of 4-bit or 8 KB of 8-bit weights) into a ring of register slots.
//  * All loads of the loop are issued and awaited by hand (async_loads.h): stage and weights of
//    a step form one packet, requested two steps before the step that uses it; a step waits for its own packet only, the younger ones stay in flight.  A step of
//    a small layer is far shorter than a memory round trip, so the depth of this pipeline is
//    what decides the time (8 steps of K = 4096: 25 us one step ahead).
//  * Per group: unpack with the zero point subtracted (step 1 of the two-step dequantization,
//    Sec. 3.3), MT x 2 `v_mfma_i32_16x16x64_i8`, int32 partial per group, fp32 rescale (step 2).
//    Token scale, fp16 conversion and scatter (Sec. 3.4) at the end of a round.
// Both scale granularities: with one activation scale per (token, group) the scales of the whole
// batch sit in LDS next to the stages (converted to fp32 once per block) and every group's partial
// is multiplied by its token's scale of that group; with one 8-bit weight scale per group the 8-bit
// tiles fetch four fp16 scales per K step like the 4-bit ones.
#include <algorithm>
#include <type_traits>

#include "async_loads.h"
#include "internal.h"

namespace mixllm {

namespace {

constexpr int NW = 8;
constexpr int NT = NW * 64;
constexpr size_t LDS_LIMIT = 150 * 1024;

// 3 activation stages of up to 64 tokens (96 KB of LDS) and 3 weight slots per wave.  (128 tokens would leave room for 2
// stages, one step of lookahead, and the kernel with 8 token tiles per wave does not fit the
// register file next to its weight ring: those sizes take the tiled kernel.)
constexpr int stage_buffers(int) { return 3; }

struct MidArgs {
    int nblk8, nblk4;   // blocks of the 8-bit and of the 4-bit part
    int qv8, qv4;       // quarter tiles per virtual tile
};

template <int I, int N, typename F>
__device__ inline void sfor(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        sfor<I + 1, N>(f);
    }
}

__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <bool PART8>
struct Slot {   // the 4 groups of one K step
    v4i w[4][PART8 ? 2 : 1];
    uint2 s;       // 4 fp16 group scales (4-bit)
    uint32_t z;    // 4 zero points (4-bit)
};

// ties the registers of a slot to the wait that precedes it
__device__ inline void tie_slot(Slot<false> &k)
{
    asm volatile("" : "+v"(k.w[0][0]), "+v"(k.w[1][0]), "+v"(k.w[2][0]), "+v"(k.w[3][0]), "+v"(k.s), "+v"(k.z)::"memory");
}
__device__ inline void tie_slot(Slot<true> &k)
{
    asm volatile(""
                 : "+v"(k.w[0][0]), "+v"(k.w[0][1]), "+v"(k.w[1][0]), "+v"(k.w[1][1]), "+v"(k.w[2][0]), "+v"(k.w[2][1]),
                   "+v"(k.w[3][0]), "+v"(k.w[3][1]), "+v"(k.s)::"memory");
}

// ACT_PT: one activation scale per token (else per token and group); W8PC: one scale per 8-bit
// channel (else per channel and group)
template <int MT, bool DUMP, bool PART8, bool ACT_PT, bool W8PC>
__device__ inline void mid_block(const LinearParams &p, const MidArgs &a, uint8_t *smem)
{
    constexpr int GB = PART8 ? 2048 : 1024;    // bytes of one group of one tile
    constexpr bool PG8 = PART8 && !W8PC && !DUMP;   // 8-bit tile that fetches group scales
    constexpr int NL = PART8 ? (PG8 ? 9 : 8) : 6;   // loads of one K step of weights
    constexpr int MP = MT * 16;                // staged token rows
    constexpr int GROUP_STAGE = MP * G;        // bytes of one group of the activation stage
    constexpr int STAGE = 4 * GROUP_STAGE;
    constexpr int NBUF = stage_buffers(MT);    // activation stages and weight slots: NBUF - 1 steps in flight
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, ks = lane >> 4;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;
    const int joff = PART8 ? 0 : p.n8;
    const int ng = p.ng, ngp = p.ngp;
    const int nquads = (ng + 3) / 4;

    // ---- the block's share of quarter tiles, its virtual tiles ----
    const int nblk = PART8 ? a.nblk8 : a.nblk4;
    const int b = (int)blockIdx.x - (PART8 ? 0 : a.nblk8);
    const int qv = PART8 ? a.qv8 : a.qv4;
    const unsigned nunits = 4u * (unsigned)ntiles;
    const int Q_lo = (int)(nunits * (unsigned)b / (unsigned)nblk), Q_hi = (int)(nunits * (unsigned)(b + 1) / (unsigned)nblk);
    const int nvt = (Q_hi - Q_lo + qv - 1) / qv;   // >= 1: never more blocks than quarter tiles
    const int rounds = (nvt + NW - 1) / NW;

    // ---- activation stage: instruction i of this wave fills 8 rows of one group ----
    // lane l writes chunk position l & 7 of row +(l >> 3), which holds the global chunk
    // (l & 7) ^ ((row >> 1) & 7); rows past M re-read row M - 1 (their outputs are never stored)
    uint32_t a_voff[MT];
    int a_group[MT];
    uint32_t a_lds[MT];
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(lds_address(smem));
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int li = wave * MT + i;          // 0 .. MP/2 - 1: (group, set of 8 rows)
        const int u = li / (MP / 8), rs = li % (MP / 8);
        const int row = rs * 8 + (lane >> 3);
        const int cs = (lane & 7) ^ ((row >> 1) & 7);
        a_voff[i] = (uint32_t)min(row, p.M - 1) * (uint32_t)p.K + cs * 16;
        a_group[i] = u;
        a_lds[i] = (uint32_t)(u * GROUP_STAGE + rs * 1024);
    }
    auto load_a = [&](int q, int buf) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
            load_lds16(lds_base + buf * STAGE + a_lds[i], a_voff[i], p.xq + (size_t)min(4 * q + a_group[i], ng - 1) * G);
    };
    // fragment reads: token row 16 mt + c, 16-byte chunk ks (k 0..63 of the group) and 4 + ks
    const int sw = (c >> 1) & 7;
    const int a_rd0 = c * G + ((ks ^ sw) << 4), a_rd1 = c * G + (((4 + ks) ^ sw) << 4);
    // activation scales per (token, group): the whole batch, as fp32, behind the stages (visible
    // after the barrier that opens the first round)
    float *xsg = (float *)(smem + NBUF * STAGE);
    if (!ACT_PT && !DUMP)
        for (int i = tid; i < p.M * ng; i += NT) xsg[i] = (float)p.xscale[i];

    const uint8_t *wpart = PART8 ? (const uint8_t *)p.w8 : p.w4;
    for (int r = 0; r < rounds; ++r) {
        // ---- this wave's virtual tile of the round: lane (c, ks) holds channel (c & 3) of the
        //      tile's quarter number c >> 2; a wave without a tile only stages and synchronizes ----
        const int vt = r * NW + wave;
        const bool has = vt < nvt;
        const int u0 = Q_lo + qv * min(vt, nvt - 1);
        const int cnt = min(qv, Q_hi - u0);
        const bool lane_valid = has && (c >> 2) < cnt;
        const int uc = u0 + min(c >> 2, cnt - 1);
        const int base_tile = u0 >> 2;
        const int row = (uc >> 2) * TILE_N + 4 * (uc & 3) + (c & 3);
        const int rel = row - base_tile * TILE_N;   // 0..31
        const uint32_t w_voff = has ? (uint32_t)((rel >> 4) * ng * GB + ((rel & 15) + 16 * ks) * 16) : 0u;
        const uint32_t s_voff = has ? (uint32_t)(rel * ngp * 2) : 0u, z_voff = has ? (uint32_t)(rel * (ngp / 2)) : 0u;
        const int ch = (lane_valid && row < nrows) ? p.perm[joff + row] : -1;
        const float sw_row = (PART8 && W8PC && !DUMP) ? (float)p.s8[row] : 0.0f;
        auto issue = [&](int q, Slot<PART8> &k) {
            const int g0 = 4 * q;
            const int last = ng - 1 - g0;   // at the ragged end of K the last group is re-read (its scale is forced to zero)
            const uint8_t *wb = wpart + ((size_t)base_tile * ng + g0) * GB;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint8_t *wu = wb + (size_t)min(u, last) * GB;
                load_reg16_nt<0>(k.w[u][0], w_voff, wu);
                if (PART8) load_reg16_nt<1024>(k.w[u][PART8 ? 1 : 0], w_voff, wu);
            }
            k.s = make_uint2(0, 0);
            k.z = 0;
            if (!PART8) {
                // (the debug entry point passes no scales: the same number of loads, from a valid address)
                if (!DUMP) load_reg8(k.s, s_voff, p.s4 + ((size_t)base_tile * TILE_N * ngp + g0));
                else load_reg8(k.s, 0u, p.z4);
                load_reg_u16(k.z, z_voff, p.z4 + ((size_t)base_tile * TILE_N * (ngp / 2) + g0 / 2));
            } else if (PG8) {
                load_reg8(k.s, s_voff, p.s8 + ((size_t)base_tile * TILE_N * ngp + g0));
            }
        };
        float acc[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[mt][i] = 0.0f;
        // One K step.  Written out as a software pipeline, because left to itself the compiler
        // emits read, wait, two dependent MFMAs, rescale for one token tile after the other (the
        // LDS and MFMA latencies of all 4 x MT tiles in a row: 3 us per step): the fragments of
        // group u + 1 are requested before the MFMAs of group u, the MT first-half MFMAs of a group
        // are issued back to back, then the MT second halves, then the rescales.
        auto compute = [&](int q, const Slot<PART8> &k, int buf) {
            // The four fp16 scales are taken out of the two loaded dwords with integer operations
            // only: a reinterpreting copy of k.s makes the compiler keep k.s as 16-bit pieces, and
            // it then splits the dwords right after the load is issued, before the data is there.
            const float sh[4] = {half_bits_to_float(k.s.x & 0xffffu), half_bits_to_float(k.s.x >> 16),
                                 half_bits_to_float(k.s.y & 0xffffu), half_bits_to_float(k.s.y >> 16)};
            const uint8_t *stage = smem + buf * STAGE;
            v4i fa[2][MT][2];
            auto read_frags = [&](int u, v4i (&f)[MT][2]) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const uint8_t *t = stage + u * GROUP_STAGE + mt * 16 * G;
                    f[mt][0] = *(const v4i *)(t + a_rd0);
                    f[mt][1] = *(const v4i *)(t + a_rd1);
                }
            };
            read_frags(0, fa[0]);
            sfor<0, 4>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                const int g = 4 * q + u;
                const bool gvalid = g < ng;
                if constexpr (u + 1 < 4) read_frags(u + 1, fa[(u + 1) & 1]);
                v4i b0, b1;
                float swg;
                if (PART8) {
                    b0 = k.w[u][0];
                    b1 = k.w[u][PART8 ? 1 : 0];
                    swg = PG8 ? sh[u] : sw_row;
                } else {
                    const uint32_t zb = zbias((int)((k.z >> (4 * u)) & 15));
                    const v4i w = k.w[u][0];
                    b0 = unpack16((uint32_t)w[0], (uint32_t)w[1], zb);
                    b1 = unpack16((uint32_t)w[2], (uint32_t)w[3], zb);
                    swg = sh[u];
                }
                if (!gvalid) swg = 0.0f;
                __builtin_amdgcn_sched_barrier(0);
                v4i P[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) P[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[u & 1][mt][0], b0, v4i{0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) P[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[u & 1][mt][1], b1, P[mt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if (DUMP) {
                        if (gvalid && ch >= 0) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int m = mt * 16 + 4 * ks + i;
                                if (m < p.M) p.P[((size_t)m * p.N + ch) * ng + g] = P[mt][i];
                            }
                        }
                    } else if (ACT_PT) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[mt][i] = __builtin_fmaf((float)P[mt][i], swg, acc[mt][i]);
                    } else {
                        const int gc = min(g, ng - 1);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float sa = xsg[min(mt * 16 + 4 * ks + i, p.M - 1) * ng + gc];
                            acc[mt][i] = __builtin_fmaf((float)P[mt][i], swg * sa, acc[mt][i]);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        };

        // ---- the K loop: packets (activation stage + weights of one step) NBUF - 1 steps ahead ----
        constexpr int PK = MT + NL;   // loads of one packet
        Slot<PART8> ring[NBUF];
        lds_barrier();   // the readers of the previous round are done with every buffer
        sfor<0, NBUF - 1>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if (j < nquads) {
                load_a(j, j);
                issue(j, ring[j]);
            }
        });
        for (int q0 = 0; q0 < nquads; q0 += NBUF) {
            sfor<0, NBUF>([&](auto dc) {
                constexpr int d = decltype(dc)::value;
                const int q = q0 + d;
                if (q < nquads) {
                    // packet q: all but the packets requested after it have landed
                    const int younger = min(NBUF - 2, nquads - 1 - q);
                    sfor<0, NBUF - 1>([&](auto yc) {
                        constexpr int y = decltype(yc)::value;
                        if (younger == y) await_loads<y * PK>();
                    });
                    tie_slot(ring[d]);
                    lds_barrier();   // every wave's part of stage q has landed; the buffer of step q - 1 is free
                    if (q + NBUF - 1 < nquads) {
                        load_a(q + NBUF - 1, (d + NBUF - 1) % NBUF);
                        issue(q + NBUF - 1, ring[(d + NBUF - 1) % NBUF]);
                    }
                    if (has) compute(q, ring[d], d);   // a wave without a tile only stages and synchronizes
                }
            });
        }
        sfor<0, NBUF>([&](auto dc) { tie_slot(ring[decltype(dc)::value]); });

        // ---- token scale, fp16, scatter (Sec. 3.4) ----
        if (!DUMP && ch >= 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = mt * 16 + 4 * ks + i;
                    if (m < p.M) p.y[(size_t)m * p.N + ch] = (half_t)(ACT_PT ? acc[mt][i] * (float)p.xscale[m] : acc[mt][i]);
                }
        }
    }
}

template <int MT, bool DUMP, bool ACT_PT, bool W8PC>
__global__ __launch_bounds__(NT) void linear_mid_kernel(LinearParams p, MidArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    if ((int)blockIdx.x < a.nblk8)
        mid_block<MT, DUMP, true, ACT_PT, W8PC>(p, a, smem);
    else
        mid_block<MT, DUMP, false, ACT_PT, W8PC>(p, a, smem);
}

// ---- host side ------------------------------------------------------------------------------

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Quarter tiles per virtual tile.  A wave's time per K step does not depend on how many of its 16
// columns are in use, and two waves on one SIMD take turns, so fewer, fuller virtual tiles are
// never slower: always 4.
int pick_qv(int) { return 4; }

// rounds of 8 virtual tiles a block of this share walks K for
int rounds_of(int share) { return ceil_div(ceil_div(share, pick_qv(share)), NW); }

// Blocks for the 8-bit and the 4-bit quarter tiles (an 8-bit one has twice the bytes): the split
// with the fewest rounds, then the smallest largest share in bytes.
void split_blocks(int units8, int units4, int nb, int &nblk8, int &nblk4)
{
    if (units8 == 0 || units4 == 0) {
        nblk8 = std::min(units8, nb);
        nblk4 = std::min(units4, nb);
        return;
    }
    long best = -1;
    for (int b8 = 1; b8 < nb; ++b8) {
        const int n8 = std::min(b8, units8), n4 = std::min(nb - b8, units4);
        const int s8 = ceil_div(units8, n8), s4 = ceil_div(units4, n4);
        const long cost = 1000000L * std::max(rounds_of(s8), rounds_of(s4)) + std::max(2L * s8, (long)s4);
        if (best < 0 || cost < best) {
            best = cost;
            nblk8 = n8;
            nblk4 = n4;
        }
    }
}

int token_tiles(int M) { return M <= 16 ? 1 : M <= 32 ? 2 : 4; }

// the activation stages, then the activation scales of the batch where there is one per (token, group)
size_t lds_bytes_of(const LinearParams &p)
{
    const int mt = token_tiles(p.M);
    const size_t xsg = (p.act_per_token || p.P) ? 0 : ((size_t)p.M * p.ng * sizeof(float) + 15) / 16 * 16;
    return (size_t)stage_buffers(mt) * mt * 8 * 1024 + xsg;
}

}  // namespace

bool mid_covers(const LinearParams &p)
{
    if (p.M < 1 || p.M > 64 || p.ng < 1 || p.x) return false;
    // one activation scale per (token, group): up to 32 tokens (with four token tiles per wave the extra
    // scale reads do not fit the register file next to the weight ring: the tiled kernel takes those)
    if (!p.act_per_token && !p.P && p.M > 32) return false;
    if (lds_bytes_of(p) > LDS_LIMIT) return false;
    // 32-bit lane offsets inside the activation, weight and metadata arrays
    const size_t two_tiles = 2 * (size_t)p.ng * 2048 + 2048;
    if ((size_t)p.M * p.K >= (1ull << 31) || two_tiles >= (1ull << 31)) return false;
    if (4ll * std::max(p.ntiles8, p.ntiles4) * 4096 >= (1ll << 31)) return false;
    return p.ntiles8 + p.ntiles4 > 0;
}

static void mid_args(const LinearParams &p, MidArgs &a, size_t &lds_bytes)
{
    a.nblk8 = a.nblk4 = 0;
    split_blocks(4 * p.ntiles8, 4 * p.ntiles4, cu_count(), a.nblk8, a.nblk4);
    a.qv8 = a.nblk8 ? pick_qv(ceil_div(4 * p.ntiles8, a.nblk8)) : 4;
    a.qv4 = a.nblk4 ? pick_qv(ceil_div(4 * p.ntiles4, a.nblk4)) : 4;
    lds_bytes = lds_bytes_of(p);
}

// the launch plan as five integers (blocks of the 8-bit part, of the 4-bit part, quarter tiles per
// virtual tile of either part, bytes of LDS), for the host-side test of the work split
bool mid_plan(const LinearParams &p, int out[5])
{
    if (!mid_covers(p)) return false;
    MidArgs a;
    size_t lds_bytes;
    mid_args(p, a, lds_bytes);
    out[0] = a.nblk8;
    out[1] = a.nblk4;
    out[2] = a.qv8;
    out[3] = a.qv4;
    out[4] = (int)lds_bytes;
    return true;
}

int launch_linear_mid(const LinearParams &p, hipStream_t st)
{
    if (!mid_covers(p)) return (int)hipErrorInvalidValue;
    MidArgs a;
    size_t lds_bytes;
    mid_args(p, a, lds_bytes);
    const int mt = token_tiles(p.M);
    dim3 grid(a.nblk8 + a.nblk4), block(NT);
    auto go = [&](auto kernel) {
        if (lds_bytes > 48 * 1024)
            if (int e = ensure_dynamic_lds((const void *)kernel, lds_bytes)) return e;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, p, a);
        return (int)hipGetLastError();
    };
    if (p.P) {
        switch (mt) {
        case 1: return go(linear_mid_kernel<1, true, true, true>);
        case 2: return go(linear_mid_kernel<2, true, true, true>);
        default: return go(linear_mid_kernel<4, true, true, true>);
        }
    }
    auto pick = [&](auto mtc) {
        constexpr int MT = decltype(mtc)::value;
        if (p.act_per_token) return p.w8_per_channel ? go(linear_mid_kernel<MT, false, true, true>) : go(linear_mid_kernel<MT, false, true, false>);
        if constexpr (MT <= 2)
            return p.w8_per_channel ? go(linear_mid_kernel<MT, false, false, true>) : go(linear_mid_kernel<MT, false, false, false>);
        return (int)hipErrorInvalidValue;   // (mid_covers refuses these)
    };
    switch (mt) {
    case 1: return pick(std::integral_constant<int, 1>{});
    case 2: return pick(std::integral_constant<int, 2>{});
    default: return pick(std::integral_constant<int, 4>{});
    }
}

}  // namespace mixllm
