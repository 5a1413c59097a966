// Decode path of the quantized linear (M <= 16 tokens): HBM-bandwidth bound, so the design
// goal is one coalesced pass over the packed weights with many independent 16-byte loads
// in flight per lane.
//
//  * A wave owns TPW weight tiles (16 output channels each) and a contiguous range of
//    quantization groups; the WPB waves of a block split K between them and reduce their
//    fp32 partial outputs through LDS (no global atomics, no workspace).
//  * Packed weights go HBM -> registers directly: a wave-wide 16-byte load is one
//    contiguous 1 KB block that already is the B operand of v_mfma_i32_16x16x64_i8
//    (after the in-register uint4 -> int8 unpack with zero-point subtraction, step 1 of
//    the two-step dequantization, Sec. 3.3).
//  * The stream is software pipelined in chunks of 4 groups over two register sets: the
//    loads of chunk i+1 (weights, activation fragments, scales, zero points) are issued
//    before chunk i is computed.  (A deeper ring of 4 sets, and staging the activations in
//    LDS to free registers for it, were both measured and were slower.)
//  * Activations are the A operand: row = token; rows >= M carry whatever token M-1 holds,
//    and their outputs are never stored.
//  * One int32 MFMA accumulator per group (2 MFMAs = 128 k), then float rescale by the
//    group scale (step 2, Sec. 3.3); the token scale is applied once at the end when it
//    does not depend on the group.
//  * Epilogue scatters fp16 results to their original channel (Sec. 3.4).
// 8-bit tiles and 4-bit tiles are different block ranges of the same launch.
#include <type_traits>

#include "internal.h"

namespace mixllm {

// compile-time loop: f(std::integral_constant<int, I>) for I in [I, N)
template <int I, int N, typename F>
static __device__ inline void static_for_dec(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for_dec<I + 1, N>(f);
    }
}

template <int TPW, bool PART8>
struct WChunk {   // weights and group metadata of 4 consecutive groups
    v4i w[TPW][4][PART8 ? 2 : 1];    // [tile][group][64-k half (8-bit only)]
    uint2 s[TPW];                    // 4 fp16 group scales
    uint32_t z[TPW];                 // 4 uint4 zero points in the low 16 bits
};
struct AChunk {   // activation fragments of 4 consecutive groups: [group][64-k half]
    v4i a[4][2];
};

template <int TPW, int WPB, bool DUMP, bool ACT_PT, bool PART8>
static __device__ inline void decode_block(const LinearParams &p, int tile0, float (*red)[TPW][4][64])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, ks = lane >> 4;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;          // real rows of this part
    const int joff = PART8 ? 0 : p.n8;              // position of the part in the concatenation
    const int nsteps = p.K / 64;
    const int ng = p.ng;
    const int nquads = (ng + 3) / 4;
    // chunk (= quad of groups) range of this wave
    const int q_lo = nquads * wave / WPB, q_hi = nquads * (wave + 1) / WPB;
    const int nch = q_hi - q_lo;
    const bool per_group_s8 = PART8 && !p.w8_per_channel;

    // A operand: lane (c, ks) supplies token min(c, M-1), k = 16*ks..+15 of each 64-k step
    const int8_t *xrow = p.xq + (size_t)min(c, p.M - 1) * p.K + ks * 16;

    int tile[TPW], row[TPW];
    const uint8_t *wbase[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        tile[t] = min(tile0 + t, ntiles - 1);
        row[t] = tile[t] * TILE_N + c;
        wbase[t] = PART8 ? (const uint8_t *)p.w8 + ((size_t)tile[t] * nsteps * 64 + lane) * 16
                         : p.w4 + ((size_t)tile[t] * ng * 64 + lane) * 16;
    }

    auto load_w = [&](int i, WChunk<TPW, PART8> &k) {
        const int q = min(q_lo + i, max(q_hi - 1, q_lo));   // past the range: re-read its last chunk
        const int g0 = 4 * min(q, nquads - 1);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int gc = min(g0 + u, ng - 1);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if (PART8) {
                    k.w[t][u][0] = __builtin_nontemporal_load((const v4i *)(wbase[t] + (size_t)gc * 2048));
                    k.w[t][u][PART8 ? 1 : 0] = __builtin_nontemporal_load((const v4i *)(wbase[t] + (size_t)gc * 2048 + 1024));
                } else {
                    k.w[t][u][0] = __builtin_nontemporal_load((const v4i *)(wbase[t] + (size_t)gc * 1024));
                }
            }
        }
        // metadata arrays are zero padded to a multiple of 8 groups: reading 4 at a quad start is in bounds
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            k.s[t] = make_uint2(0, 0);
            k.z[t] = 0;
            if (!PART8) {
                if (!DUMP) k.s[t] = *(const uint2 *)(p.s4 + (size_t)row[t] * p.ngp + g0);
                k.z[t] = *(const uint16_t *)(p.z4 + (size_t)row[t] * (p.ngp / 2) + g0 / 2);
            } else if (!DUMP && per_group_s8) {
                k.s[t] = *(const uint2 *)(p.s8 + (size_t)row[t] * p.ngp + g0);
            }
        }
    };
    auto load_a = [&](int i, AChunk &k) {
        const int q = min(q_lo + i, max(q_hi - 1, q_lo));
        const int g0 = 4 * min(q, nquads - 1);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int gc = min(g0 + u, ng - 1);
            k.a[u][0] = *(const v4i *)(xrow + (size_t)gc * G);
            k.a[u][1] = *(const v4i *)(xrow + (size_t)gc * G + 64);
        }
    };

    int ch[TPW];   // output channel of this lane's column (debug dump only)
    if (DUMP) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) ch[t] = (tile0 + t < ntiles && row[t] < nrows) ? p.perm[joff + row[t]] : -1;
    }
    float sw_row[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) sw_row[t] = (PART8 && !DUMP && p.w8_per_channel) ? (float)p.s8[row[t]] : 0.0f;

    float acc[TPW][4];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = 0.0f;

    auto compute = [&](int i, const WChunk<TPW, PART8> &k, const AChunk &ka) {
        const int q = q_lo + i;
        const bool qvalid = q < q_hi;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = 4 * q + u;
            const bool gvalid = qvalid && g < ng;
            float sa[4] = {1.0f, 1.0f, 1.0f, 1.0f};
            if (!ACT_PT && !DUMP) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    sa[r] = (float)p.xscale[(size_t)min(4 * ks + r, p.M - 1) * ng + min(g, ng - 1)];
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                v4i b0, b1;
                float sw = 0.0f;
                half_t s4h[4];
                __builtin_memcpy(s4h, &k.s[t], 8);
                if (PART8) {
                    b0 = k.w[t][u][0];
                    b1 = k.w[t][u][PART8 ? 1 : 0];
                    if (!DUMP) sw = per_group_s8 ? (float)s4h[u] : sw_row[t];
                } else {
                    const v4i w = k.w[t][u][0];
                    const uint32_t zb = zbias((k.z[t] >> (4 * u)) & 15);
                    b0 = unpack16((uint32_t)w[0], (uint32_t)w[1], zb);
                    b1 = unpack16((uint32_t)w[2], (uint32_t)w[3], zb);
                    if (!DUMP) sw = (float)s4h[u];
                }
                if (!gvalid) sw = 0.0f;   // a clamped re-read past the range contributes nothing
                v4i P = __builtin_amdgcn_mfma_i32_16x16x64_i8(ka.a[u][0], b0, v4i{0, 0, 0, 0}, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(ka.a[u][1], b1, P, 0, 0, 0);
                if (DUMP) {
                    if (gvalid && ch[t] >= 0) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int m = 4 * ks + r;
                            if (m < p.M) p.P[((size_t)m * p.N + ch[t]) * ng + g] = P[r];
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        acc[t][r] = __builtin_fmaf((float)P[r], ACT_PT ? sw : sw * sa[r], acc[t][r]);
                }
            }
        }
    };

    // two register sets: chunk i+1 is in flight while chunk i is computed
    WChunk<TPW, PART8> kw[2];
    AChunk ka[2];
    if (nch > 0) {
        load_w(0, kw[0]);
        load_a(0, ka[0]);
    }
    for (int i = 0; i < nch; i += 2) {
        if (i + 1 < nch) {
            load_w(i + 1, kw[1]);
            load_a(i + 1, ka[1]);
        }
        compute(i, kw[0], ka[0]);
        if (i + 1 < nch) {
            if (i + 2 < nch) {
                load_w(i + 2, kw[0]);
                load_a(i + 2, ka[0]);
            }
            compute(i + 1, kw[1], ka[1]);
        }
    }
    if (DUMP) return;

    // reduce the K-split partial outputs of the WPB waves through LDS
    if (WPB > 1) {
#pragma unroll
        for (int t = 0; t < TPW; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][t][r][lane] = acc[t][r];
        __syncthreads();
    }
    for (int idx = threadIdx.x; idx < TPW * 256; idx += WPB * 64) {
        const int t = idx >> 8, r = (idx >> 6) & 3, l = idx & 63;
        float v = 0.0f;
        if (WPB > 1) {
#pragma unroll
            for (int w = 0; w < WPB; ++w) v += red[w][t][r][l];
        } else {
            // a single wave: idx walks (t, r) for this lane, l == lane
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    if (tt == t && rr == r) v = acc[tt][rr];
        }
        const int m = 4 * (l >> 4) + r;
        const int rw = (tile0 + t) * TILE_N + (l & 15);
        if (tile0 + t < ntiles && rw < nrows && m < p.M) {
            if (ACT_PT) v *= (float)p.xscale[m];
            p.y[(size_t)m * p.N + p.perm[joff + rw]] = (half_t)v;   // scatter, Sec. 3.4
        }
    }
}

template <int TPW, int WPB, bool DUMP, bool ACT_PT>
__global__ __launch_bounds__(WPB * 64) void linear_decode_kernel(LinearParams p, int nblk8)
{
    __shared__ float red[(DUMP || WPB == 1) ? 1 : WPB][TPW][4][64];
    if ((int)blockIdx.x < nblk8)
        decode_block<TPW, WPB, DUMP, ACT_PT, true>(p, blockIdx.x * TPW, red);
    else
        decode_block<TPW, WPB, DUMP, ACT_PT, false>(p, (blockIdx.x - nblk8) * TPW, red);
}

template <int TPW, int WPB>
static int launch_cfg(const LinearParams &p, hipStream_t st)
{
    const int nblk8 = (p.ntiles8 + TPW - 1) / TPW, nblk4 = (p.ntiles4 + TPW - 1) / TPW;
    dim3 grid(nblk8 + nblk4), block(WPB * 64);
    if (p.P) {
        hipLaunchKernelGGL((linear_decode_kernel<TPW, WPB, true, true>), grid, block, 0, st, p, nblk8);
    } else {
        if (p.act_per_token)
            hipLaunchKernelGGL((linear_decode_kernel<TPW, WPB, false, true>), grid, block, 0, st, p, nblk8);
        else
            hipLaunchKernelGGL((linear_decode_kernel<TPW, WPB, false, false>), grid, block, 0, st, p, nblk8);
    }
    return (int)hipGetLastError();
}

template <int TPW>
static int launch_wpb(const LinearParams &p, int wpb, hipStream_t st)
{
    switch (wpb) {
    case 1: return launch_cfg<TPW, 1>(p, st);
    case 2: return launch_cfg<TPW, 2>(p, st);
    case 4: return launch_cfg<TPW, 4>(p, st);
    default: return launch_cfg<TPW, 8>(p, st);
    }
}

// ---- resident-activation variant -------------------------------------------------------------
// The streaming variant above re-reads the activation fragments for every tile: at M = 16 that
// is twice the L1 traffic of the weights themselves, and at any M most of its vector-memory
// instructions.  Here a block of WPB waves walks a contiguous range of tiles, slab by slab: a
// slab is WPB * 4 quantization groups of K, wave w owns groups 4w..4w+3 of it, and keeps the A
// fragments of those groups in registers for all tiles of the block.  Per (slab, tile) item a
// wave issues only the weight, metadata and channel-index loads, D - 1 items ahead of the one
// it computes (a ring of D register sets), and the K-split partial outputs meet in LDS once
// per item (double buffered: one barrier per item).  With several slabs the finishing wave of
// a tile carries the tile's running sum in LDS.
//
// Integer pipeline of a 4-bit group, with the zero point hoisted out of the unpack:
//   sum_k a (q - z) = sum_k a q  -  z * sum_k a
// The nibbles go to the MFMA as they are (two mask/shift instructions per 8 weights instead of
// seven), and sum_k a per (token, group) comes from one more MFMA pair per group against an
// all-ones operand, computed once per slab because the activations are resident.  Everything
// is int32 and exact, so the group partial sums are bit-identical to the plain definition.
// NR = number of accumulator registers that matter (1 when M = 1: token 0 is register 0).
// The barrier is written out: __syncthreads() would also wait for the prefetched loads.
constexpr int RES_MAX_TILES = 16;   // tiles per block the LDS running sums provide for

static __device__ inline void tile_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <bool PART8>
struct ResItem {   // one (slab, tile) item of one wave: 4 groups of one tile
    v4i w[4][PART8 ? 2 : 1];
    uint2 s;        // 4 fp16 group scales
    uint32_t z;     // 4 uint4 zero points in the low 16 bits
    int ch;         // original channel of this lane's column, -1 for a padding row
    half_t sw_row;  // per-channel scale of an 8-bit row
};

// FUSED: the activations arrive as fp16 (p.x) and every block quantizes them itself while its
// first weight loads are in flight (Sec. 2 formula, z = 0; the same arithmetic as the stand-alone
// quantizer, so the codes are identical): wave w quantizes its own 512 k of every token row
// (the row maxima of the waves meet in LDS), leaves the codes in LDS and picks its A fragments
// up from there.  The work per block is that of the whole stand-alone quantizer: measured, it
// wins for one token, ties at two and loses from three on, so it is built for one token; and it
// requires a single slab (K <= WPB * 512).
typedef half_t h8v __attribute__((ext_vector_type(8)));
constexpr int FUSED_MAX_M = 1;

template <int WPB>
struct QuantScratch {
    float part[WPB][FUSED_MAX_M];         // per-wave row maxima
    float scale[WPB][FUSED_MAX_M][4];     // per wave: row scale ([0]) or the 4 group scales of its share
    __attribute__((aligned(16))) uint8_t code[WPB][FUSED_MAX_M][512];   // int8 codes of each wave's share of K
};

template <int WPB, int D, int NR, bool DUMP, bool ACT_PT, bool PART8, bool FUSED>
static __device__ inline void decode_resident(const LinearParams &p, int tile_begin, int tile_end,
                                              float (*red)[WPB][NR][64], float (*tacc)[NR][64],
                                              QuantScratch<WPB> *qs)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, ks = lane >> 4;
    const int nrows = PART8 ? p.n8 : p.n4;
    const int joff = PART8 ? 0 : p.n8;
    const int nsteps = p.K / 64;
    const int ng = p.ng;
    const int nquads = (ng + 3) / 4;
    const int nslab = (nquads + WPB - 1) / WPB;
    const int ntl = tile_end - tile_begin;
    const int total = nslab * ntl;   // items, slab-major: f -> slab f / ntl, tile tile_begin + f % ntl
    const bool per_group_s8 = PART8 && !p.w8_per_channel;

    const int8_t *xrow = FUSED ? nullptr : p.xq + (size_t)min(c, p.M - 1) * p.K + ks * 16;
    float xs[NR];   // per-token activation scales of rows 4ks..
#pragma unroll
    for (int r = 0; r < NR; ++r) xs[r] = (!FUSED && ACT_PT && !DUMP) ? (float)p.xscale[min(4 * ks + r, p.M - 1)] : 1.0f;

    // resident state of the current slab
    v4i a[4][2];
    int S[4][NR];        // sum_k a per (group, row) (4-bit tiles only)
    float sa[4][NR];     // per-(token, group) activation scales (unused when per token)
    auto load_slab = [&](int slab) {
        const int g0 = 4 * min(slab * WPB + wave, nquads - 1);
        if (FUSED) {
            // This wave's share of K is k in [512 wave, 512 wave + 512): lane l quantizes the 8
            // values at 512 wave + 8 l of each token row (values past K count as zero), so every
            // code is computed once per block, not once per lane that later uses it.
            const int k0 = 512 * wave + 8 * lane;
            const bool kvalid = k0 < p.K;
            for (int r = 0; r < p.M; ++r) {
                h8v xv;
#pragma unroll
                for (int i = 0; i < 8; ++i) xv[i] = (half_t)0.0f;
                if (kvalid) xv = *(const h8v *)(p.x + (size_t)r * p.K + k0);
                float amax = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)xv[i]));
                // 16 lanes cover one group of 128
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
                float sc;
                if (ACT_PT) {
                    amax = fmaxf(amax, __shfl_xor(amax, 16, 64));
                    amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
                    if (lane == 0) qs->part[wave][r] = amax;
                    tile_barrier();   // every wave runs this loop the same number of times
                    float row = 0.0f;
#pragma unroll
                    for (int w = 0; w < WPB; ++w) row = fmaxf(row, qs->part[w][r]);
                    sc = (float)store_scale(row / 127.0f);
                    if (lane == 0) qs->scale[wave][r][0] = sc;
                } else {
                    sc = (float)store_scale(amax / 127.0f);
                    if ((lane & 15) == 0) qs->scale[wave][r][lane >> 4] = sc;
                }
                const float rc = recip(sc);
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    w0 |= quant_code(xv[i], sc, rc) << (8 * i);
                    w1 |= quant_code(xv[4 + i], sc, rc) << (8 * i);
                }
                *(uint2 *)&qs->code[wave][r][8 * lane] = make_uint2(w0, w1);
            }
            // the fragments and scales this lane needs come from other lanes of the same wave
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            const int rc = min(c, p.M - 1);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a[u][0] = *(const v4i *)&qs->code[wave][rc][u * 128 + ks * 16];
                a[u][1] = *(const v4i *)&qs->code[wave][rc][u * 128 + 64 + ks * 16];
#pragma unroll
                for (int r = 0; r < NR; ++r) sa[u][r] = ACT_PT ? 1.0f : qs->scale[wave][min(4 * ks + r, p.M - 1)][u];
            }
#pragma unroll
            for (int r = 0; r < NR; ++r) xs[r] = ACT_PT ? qs->scale[wave][min(4 * ks + r, p.M - 1)][0] : 1.0f;
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int gc = min(g0 + u, ng - 1);
                a[u][0] = *(const v4i *)(xrow + (size_t)gc * G);
                a[u][1] = *(const v4i *)(xrow + (size_t)gc * G + 64);
#pragma unroll
                for (int r = 0; r < NR; ++r)
                    sa[u][r] = (!ACT_PT && !DUMP) ? (float)p.xscale[(size_t)min(4 * ks + r, p.M - 1) * ng + gc] : 1.0f;
            }
        }
        if (!PART8) {
            const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v4i t = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][0], ones, v4i{0, 0, 0, 0}, 0, 0, 0);
                t = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][1], ones, t, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < NR; ++r) S[u][r] = t[r];
            }
        }
    };

    // byte offsets that do not change from item to item
    constexpr int GB = PART8 ? 2048 : 1024;                       // bytes of one group of one tile
    const size_t tile_bytes = (size_t)ng * GB;
    const uint8_t *wlane = (PART8 ? (const uint8_t *)p.w8 : p.w4) + (size_t)tile_begin * tile_bytes + lane * 16;
    auto load = [&](int slab, int tl, ResItem<PART8> &t) {
        const int row = (tile_begin + tl) * TILE_N + c;
        const int g0 = 4 * min(slab * WPB + wave, nquads - 1);
        const uint8_t *wb = wlane + (size_t)tl * tile_bytes + (size_t)g0 * GB;
        const int last = ng - 1 - g0;   // at the ragged end of K the last group is re-read (its scale is forced to zero)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int du = min(u, last);
            t.w[u][0] = __builtin_nontemporal_load((const v4i *)(wb + du * GB));
            if (PART8) t.w[u][PART8 ? 1 : 0] = __builtin_nontemporal_load((const v4i *)(wb + du * GB + 1024));
        }
        t.s = make_uint2(0, 0);
        t.z = 0;
        t.sw_row = (half_t)0.0f;
        if (!PART8) {
            if (!DUMP) t.s = *(const uint2 *)(p.s4 + (size_t)row * p.ngp + g0);
            t.z = *(const uint16_t *)(p.z4 + (size_t)row * (p.ngp / 2) + g0 / 2);
        } else if (!DUMP) {
            if (per_group_s8) t.s = *(const uint2 *)(p.s8 + (size_t)row * p.ngp + g0);
            else t.sw_row = p.s8[row];
        }
        const int ch = p.perm[min(joff + row, p.N - 1)];
        t.ch = row < nrows ? ch : -1;
    };

    float acc[NR];
    auto compute = [&](int slab, const ResItem<PART8> &t) {
        const int q = slab * WPB + wave;
        half_t sh[4];
        __builtin_memcpy(sh, &t.s, 8);
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = 4 * q + u;
            const bool gvalid = q < nquads && g < ng;
            v4i P;
            float sw;
            if (PART8) {
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][0], t.w[u][0], v4i{0, 0, 0, 0}, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][1], t.w[u][PART8 ? 1 : 0], P, 0, 0, 0);
                sw = per_group_s8 ? (float)sh[u] : (float)t.sw_row;
            } else {
                const v4i w = t.w[u][0];
                const int m4 = 0x0F0F0F0F;
                const v4i b0 = {w[0] & m4, (int)((uint32_t)w[0] >> 4) & m4, w[1] & m4, (int)((uint32_t)w[1] >> 4) & m4};
                const v4i b1 = {w[2] & m4, (int)((uint32_t)w[2] >> 4) & m4, w[3] & m4, (int)((uint32_t)w[3] >> 4) & m4};
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][0], b0, v4i{0, 0, 0, 0}, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[u][1], b1, P, 0, 0, 0);
                const int z = (int)((t.z >> (4 * u)) & 15);
#pragma unroll
                for (int r = 0; r < NR; ++r) P[r] -= z * S[u][r];
                sw = (float)sh[u];
            }
            if (!gvalid) sw = 0.0f;   // a clamped re-read past the end of K contributes nothing
            if (DUMP) {
                if (gvalid && t.ch >= 0) {
#pragma unroll
                    for (int r = 0; r < NR; ++r) {
                        const int m = 4 * ks + r;
                        if (m < p.M) p.P[((size_t)m * p.N + t.ch) * ng + g] = P[r];
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < NR; ++r) acc[r] = __builtin_fmaf((float)P[r], ACT_PT ? sw : sw * sa[u][r], acc[r]);
            }
        }
    };
    // partial outputs of the item to LDS, one barrier, one wave sums them up
    auto finish = [&](int slab, int tl, int par, const ResItem<PART8> &t) {
        if (DUMP) return;
        if (WPB > 1) {
#pragma unroll
            for (int r = 0; r < NR; ++r) red[par][wave][r][lane] = acc[r];
            tile_barrier();
        }
        if (WPB == 1 || wave == tl % WPB) {
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                float v = acc[r];
                if (WPB > 1) {
                    v = 0.0f;
#pragma unroll
                    for (int w = 0; w < WPB; ++w) v += red[par][w][r][lane];
                }
                if (slab > 0) v += tacc[tl][r][lane];
                if (slab + 1 < nslab) {
                    tacc[tl][r][lane] = v;   // the same wave finishes this tile in every slab
                } else {
                    const int m = 4 * ks + r;
                    if (m < p.M && t.ch >= 0) p.y[(size_t)m * p.N + t.ch] = (half_t)(v * xs[r]);   // scatter, Sec. 3.4
                }
            }
        }
    };

    static_assert(D % 2 == 0, "the LDS double buffer alternates with the ring position");
    ResItem<PART8> ring[D];
    int lslab = 0, ltl = 0;   // position of the next item to request
    auto request = [&](ResItem<PART8> &t) {
        load(lslab, ltl, t);
        if (++ltl == ntl) {
            ltl = 0;
            ++lslab;
        }
    };
    static_for_dec<0, D - 1>([&](auto dc) {
        constexpr int d = decltype(dc)::value;
        if (d < total) request(ring[d]);
    });
    int slab = 0, tl = 0;     // position of the item being computed
    for (int f0 = 0; f0 < total; f0 += D) {
        static_for_dec<0, D>([&](auto dc) {
            constexpr int d = decltype(dc)::value;
            const int f = f0 + d;
            if (f < total) {
                if (f + D - 1 < total) request(ring[(d + D - 1) % D]);
                if (tl == 0) load_slab(slab);
                compute(slab, ring[d]);
                finish(slab, tl, d & 1, ring[d]);
                if (++tl == ntl) {
                    tl = 0;
                    ++slab;
                }
            }
        });
    }
}

template <int WPB, int NR, bool DUMP, bool ACT_PT, bool FUSED>
__global__ __launch_bounds__(WPB * 64) void linear_decode_resident_kernel(LinearParams p, int nblk8, int per8, int per4)
{
    __shared__ float red[(DUMP || WPB == 1) ? 1 : 2][WPB][NR][64];
    __shared__ float tacc[DUMP ? 1 : RES_MAX_TILES][NR][64];
    __shared__ QuantScratch<FUSED ? WPB : 1> qscratch;
    QuantScratch<WPB> *qlds = (QuantScratch<WPB> *)&qscratch;   // only dereferenced when FUSED
    const int b = blockIdx.x;
    if (b < nblk8) {
        const int t0 = b * per8;
        decode_resident<WPB, 2, NR, DUMP, ACT_PT, true, FUSED>(p, t0, min(t0 + per8, p.ntiles8), red, tacc, qlds);
    } else {
        const int t0 = (b - nblk8) * per4;
        decode_resident<WPB, 4, NR, DUMP, ACT_PT, false, FUSED>(p, t0, min(t0 + per4, p.ntiles4), red, tacc, qlds);
    }
}

template <int WPB, int NR>
static int launch_resident(const LinearParams &p, int nblk8, int per8, int nblk4, int per4, hipStream_t st)
{
    dim3 grid(nblk8 + nblk4), block(WPB * 64);
    if (p.P)
        hipLaunchKernelGGL((linear_decode_resident_kernel<WPB, NR, true, true, false>), grid, block, 0, st, p, nblk8, per8, per4);
    else if (p.x) {
        if constexpr (NR == 1) {   // fp16 activations: one token only (resident_can_fuse)
            if (p.act_per_token)
                hipLaunchKernelGGL((linear_decode_resident_kernel<WPB, 1, false, true, true>), grid, block, 0, st, p, nblk8, per8, per4);
            else
                hipLaunchKernelGGL((linear_decode_resident_kernel<WPB, 1, false, false, true>), grid, block, 0, st, p, nblk8, per8, per4);
        } else {
            return (int)hipErrorInvalidValue;
        }
    }
    else if (p.act_per_token)
        hipLaunchKernelGGL((linear_decode_resident_kernel<WPB, NR, false, true, false>), grid, block, 0, st, p, nblk8, per8, per4);
    else
        hipLaunchKernelGGL((linear_decode_resident_kernel<WPB, NR, false, false, false>), grid, block, 0, st, p, nblk8, per8, per4);
    return (int)hipGetLastError();
}

// Resident variant: blocks walk contiguous tile ranges.  8-bit tiles hold twice the bytes of
// 4-bit tiles, so an 8-bit block gets half as many tiles as a 4-bit block, and the tile counts
// per block are the smallest for which all blocks are resident at once.
// Returns -1 when the shape is not covered (then the streaming variant runs).
template <int WPB>
static int try_launch_resident(const LinearParams &p, int blocks_per_cu, hipStream_t st)
{
    const int slots = cu_count() * blocks_per_cu;   // blocks resident at once
    auto blocks = [&](int i4) {
        const int i8 = i4 >= 2 ? i4 / 2 : 1;
        return (p.ntiles4 + i4 - 1) / i4 + (p.ntiles8 + i8 - 1) / i8;
    };
    int per4 = 1;
    while (blocks(per4) > slots && per4 < RES_MAX_TILES) ++per4;
    if (blocks(per4) > slots) return -1;
    const int per8 = per4 >= 2 ? per4 / 2 : 1;
    const int nblk8 = (p.ntiles8 + per8 - 1) / per8, nblk4 = (p.ntiles4 + per4 - 1) / per4;
    return p.M == 1 ? launch_resident<WPB, 1>(p, nblk8, per8, nblk4, per4, st)
                    : launch_resident<WPB, 4>(p, nblk8, per8, nblk4, per4, st);
}

// Launch shape (from sweeps on the Llama-shaped layers): at most 8 waves per CU in total; K
// is split WPB ways inside a block when there are too few tiles for that, and a wave takes
// two tiles when M is large enough for the activation traffic to matter.
// The resident variant takes fp16 activations when K is a single slab of 8 waves (K <= 4096).
static bool resident_can_fuse(const LinearParams &p)
{
    return p.M >= 1 && p.M <= FUSED_MAX_M && p.ng <= 32 && !p.P;
}

// The evenly split variant is taken wherever it can run: it streams large layers faster than
// the two older variants (67 MB of weights, one token: 13.9 us against 16.2; 34 MB with
// K = 14336: 11.1 against 13.0; 16 tokens: 15.7 against 19.6) and is within 0.3 us of the
// resident variant on the smallest (8 MB, one token: 6.0 against 5.8; faster from two tokens
// on).  A caller that names another variant gets that one.
static bool prefer_split(const LinearParams &p)
{
    return p.variant == DECODE_ANY || p.variant == DECODE_SPLIT;
}

// fp16 activations (p.x set on the copy that is tested) can be taken by one of the variants
bool decode_can_fuse_quantizer(const LinearParams &p)
{
    LinearParams q = p;
    q.x = (const half_t *)(uintptr_t)16;   // only tested against null
    return resident_can_fuse(p) || (!p.P && decode_split_covers(q));
}

int launch_linear_decode(const LinearParams &p, hipStream_t st)
{
    if (p.M == 0 || p.N == 0) return hipSuccess;
    if (decode_split_covers(p) && (prefer_split(p) || (p.x && !resident_can_fuse(p)))) return launch_linear_decode_split(p, st);
    // Shapes the split variant does not take (one to four tokens of K > 32768): the kernel for a few
    // dozen tokens stages the activations per K step and measured 10-25 % faster than the streaming
    // variant on layers of at least two tiles per CU, slower on smaller ones (one tile per CU: 30 vs 20 us).
    if (p.variant == DECODE_ANY && !p.x && p.ntiles8 + p.ntiles4 >= 512 && mid_covers(p)) return launch_linear_mid(p, st);
    if (p.x) {   // fused quantizer
        if (!resident_can_fuse(p)) return (int)hipErrorInvalidValue;
        const int rc = try_launch_resident<8>(p, 1, st);
        return rc >= 0 ? rc : (int)hipErrorInvalidValue;
    }
    const int tiles = p.ntiles8 + p.ntiles4;
    // Resident variant where it measured faster on the Llama-shaped layers: K of one slab
    // (K <= 4096) and either few tiles or a single token.
    const bool resident = p.variant == DECODE_STREAM ? false
                        : p.variant == DECODE_RESIDENT ? true : (p.ng <= 32 && (tiles <= 1024 || p.M == 1));
    if (resident) {
        const int rc = try_launch_resident<8>(p, 1, st);
        if (rc >= 0) return rc;
    }
    const int nquads = (p.ng + 3) / 4;
    const int tpw = (tiles >= 300 && p.M > 4) ? 2 : 1;
    int wpb = 1;
    while (wpb < 8 && wpb * 2 <= nquads && tiles * wpb * 2 <= 8 * cu_count()) wpb *= 2;
    return tpw == 2 ? launch_wpb<2>(p, wpb, st) : launch_wpb<1>(p, wpb, st);
}

}  // namespace mixllm
