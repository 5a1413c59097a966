// Prefill path of the quantized linear (M > 16 tokens): int8-MFMA bound.
//
// A block of WM x WN waves computes a (WM*TM*32) x (WN*TN*32) tile of y with
// v_mfma_i32_32x32x32_i8; a wave owns TM x TN MFMA tiles of 32 tokens x 32 channels.
//  * Activations (A operand, rows = tokens) are staged per quantization group through LDS,
//    double buffered, one barrier per group; rows are padded to 144 bytes so that the
//    16-byte fragment reads of 32 lanes fall in distinct banks.
//  * Packed weights (B operand, columns = channels) go HBM/L2 -> registers directly, in the
//    same packed layout the decode path streams: two 16-byte loads per lane fetch one group
//    of one 32-channel tile.  No weight byte passes through LDS.
//  * uint4 -> int8 unpack with zero-point subtraction in registers (step 1 of the two-step
//    dequantization, Sec. 3.3), once per group, reused by the TM token tiles of the wave.
//  * Per group and tile: 4 chained MFMAs (K = 128) into an int32 accumulator, then
//    int->float and one FMA per element with the group scale (step 2, Sec. 3.3).  The
//    channel a lane owns is the MFMA column, so the group scale is one register per lane.
//  * Issue order.  On this hardware a vector instruction only overlaps an MFMA that does
//    not feed the next MFMA in program order, and a dependent MFMA issued right behind its
//    predecessor stalls the port.  So tiles are processed in pairs (two independent
//    accumulation chains, alternating), and the float rescale of the PREVIOUS pair (and the
//    LDS reads of the next fragments) is placed in the shadow of each MFMA; the pipeline
//    runs across group boundaries.  Two waves per SIMD cover the remaining bubbles.
//  * Epilogue: token scale, fp16 conversion, scatter to the original channel (Sec. 3.4).
// 8-bit and 4-bit channel tiles are different block ranges of one launch.
#include <type_traits>

#include "internal.h"

namespace mixllm {

constexpr int A_STRIDE = G + 16;   // bytes per LDS row of the activation tile

// compile-time loop: f(std::integral_constant<int, I>) for I in [I, N)
template <int I, int N, typename F>
static __device__ inline void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int WM_, int WN_, int TM_, int TN_>
struct Shape {
    static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
    static constexpr int THREADS = 64 * WM * WN;
    static constexpr int BM = WM * TM * 32;       // tokens per block
    static constexpr int BN = WN * TN * 32;       // channels per block
    static constexpr int A_STAGE = BM * A_STRIDE;
    static constexpr int A_CHUNKS = BM * 8 / THREADS;   // 16-byte chunks of the A tile per thread
    static_assert(BM * 8 % THREADS == 0, "A tile must split evenly over the threads");
    static_assert(TN == 1 || TN == 2, "a wave owns one or two 32-channel tiles");
    static_assert((TM * TN) % 4 == 0, "tiles are processed in an even number of pairs");
};

template <typename C, bool DUMP, bool ACT_PT, bool PART8>
static __device__ inline void prefill_block(const LinearParams &p, int m0, int t16_0, uint8_t *lds_a,
                                            float *lds_sa)
{
    constexpr int TM = C::TM, TN = C::TN, WN = C::WN;
    constexpr int THREADS = C::THREADS, BM = C::BM, A_STAGE = C::A_STAGE, A_CHUNKS = C::A_CHUNKS;
    constexpr int NP = TM * TN / 2;          // tile pairs per group
    constexpr int NA = TN == 1 ? 2 : 1;      // distinct token tiles in a pair
    constexpr int NSTEP = NP * 4;            // (pair, 32-k step) steps per group
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int n32 = lane & 31, h = lane >> 5;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;
    const int joff = PART8 ? 0 : p.n8;
    const int nsteps = p.K / 64;
    const int ng = p.ng;
    const int mw0 = wm * TM * 32;   // first row of this wave inside the block tile

    // this lane's channel in each of the wave's 32-channel tiles
    int tile16[TN], rw[TN], ch[TN];
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
        const int t = t16_0 + (wn * TN + nt) * 2 + (n32 >> 4);
        tile16[nt] = min(t, ntiles - 1);
        rw[nt] = tile16[nt] * TILE_N + (n32 & 15);
        ch[nt] = (t < ntiles && rw[nt] < nrows) ? p.perm[joff + rw[nt]] : -1;
    }

    // ---- loaders -------------------------------------------------------------------
    // Activation tile of one group: BM rows x 128 bytes.  Rows past M re-read row M-1: token
    // rows are independent, and outputs of rows >= M are never stored.
    const int8_t *a_src[A_CHUNKS];
    int a_dst[A_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        const int id = tid + THREADS * i, row = id >> 3, c16 = id & 7;
        a_src[i] = p.xq + (size_t)min(m0 + row, p.M - 1) * p.K + c16 * 16;
        a_dst[i] = row * A_STRIDE + c16 * 16;
    }
    // weights of one group for the wave's TN tiles.
    //  4-bit: wq[nt][0] = 16-k chunks h and 4+h, wq[nt][1] = chunks 2+h and 6+h (packed)
    //  8-bit: wq[nt][j] = chunk 2j+h (int8)
    constexpr int NBQ = PART8 ? 4 : 2;
    const uint8_t *b_src[TN];
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
        if (PART8)
            b_src[nt] = (const uint8_t *)p.w8 + ((size_t)tile16[nt] * nsteps * 64 + (n32 & 15)) * 16;
        else
            b_src[nt] = p.w4 + ((size_t)tile16[nt] * ng * 64 + (n32 & 15) + 16 * h) * 16;
    }
    auto load_b = [&](int g, v4i (&wq)[TN][NBQ]) {
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
            if (PART8) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = 2 * j + h;   // 16-k chunk: 64-k step 2g + c/4, k-slot c%4
                    wq[nt][j] = *(const v4i *)(b_src[nt] + ((size_t)(2 * g + (c >> 2)) * 64 + 16 * (c & 3)) * 16);
                }
            } else {
                const uint8_t *base = b_src[nt] + (size_t)g * 1024;
                wq[nt][0] = *(const v4i *)base;
                wq[nt][1] = *(const v4i *)(base + 512);
            }
        }
    };
    // Group metadata is kept as loaded (fp16 scale bits, zero-point byte) and only converted
    // when its group is computed, so that nothing waits on a load in the iteration that
    // issued it.
    struct Meta {
        half_t sw[TN];
        uint8_t zraw[TN];
    };
    auto load_meta = [&](int g, Meta &mt) {
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
            mt.sw[nt] = (half_t)0.0f;
            mt.zraw[nt] = 0;
            if (PART8) {
                if (!DUMP) mt.sw[nt] = p.w8_per_channel ? p.s8[rw[nt]] : p.s8[(size_t)rw[nt] * p.ngp + g];
            } else {
                if (!DUMP) mt.sw[nt] = p.s4[(size_t)rw[nt] * p.ngp + g];
                mt.zraw[nt] = p.z4[(size_t)rw[nt] * (p.ngp / 2) + (g >> 1)];
            }
        }
    };

    v16i zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0;

    float acc[TM][TN][16];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int nt = 0; nt < TN; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    // Rescale (or, for the debug entry point, dump) registers 4j..4j+3 of one finished tile:
    // rows m0 + mw0 + 32 mt + 8 j + 4 h + {0..3}, column = this lane's channel of tile nt.
    auto finish4 = [&](const v16i &P, auto mtc, auto ntc, auto jc, float sw, int gp) {
        constexpr int mt = decltype(mtc)::value, nt = decltype(ntc)::value, j = decltype(jc)::value;
        if (DUMP) {
            if (gp >= 0 && gp < ng && ch[nt] >= 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = m0 + mw0 + mt * 32 + 8 * j + 4 * h + i;
                    if (m < p.M) p.P[((size_t)m * p.N + ch[nt]) * ng + gp] = P[4 * j + i];
                }
            }
        } else if (ACT_PT) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[mt][nt][4 * j + i] = __builtin_fmaf((float)P[4 * j + i], sw, acc[mt][nt][4 * j + i]);
        } else {
            // per-(token, group) activation scales of the tile's group, staged in LDS (3 stages)
            const v4f sa = *(const v4f *)(lds_sa + ((gp + 3) % 3) * BM + mw0 + mt * 32 + 8 * j + 4 * h);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[mt][nt][4 * j + i] = __builtin_fmaf((float)P[4 * j + i], sw * sa[i], acc[mt][nt][4 * j + i]);
        }
    };

    // ---- prologue ------------------------------------------------------------------
    // Global loads run two groups ahead of the MFMAs (one group of compute is shorter than a
    // loaded memory round trip): register sets [parity of the group].  Group g+2 is requested
    // at the top of iteration g into the set group g just vacated; activations of group g+1
    // move from registers to the other LDS stage at the bottom of iteration g.
    v4i areg[2][A_CHUNKS];
    v4i wq[2][TN][NBQ];
    Meta meta[2];
    float sa_reg[2] = {0.0f, 0.0f};
    const int g1 = min(1, ng - 1);
    load_b(0, wq[0]);
    load_meta(0, meta[0]);
    load_b(g1, wq[1]);
    load_meta(g1, meta[1]);
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) areg[0][i] = *(const v4i *)a_src[i];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) areg[1][i] = *(const v4i *)(a_src[i] + (size_t)g1 * G);
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) *(v4i *)(lds_a + a_dst[i]) = areg[0][i];
    if (!ACT_PT && !DUMP && tid < BM) {
        lds_sa[tid] = (float)p.xscale[(size_t)min(m0 + tid, p.M - 1) * ng];
        sa_reg[1] = (float)p.xscale[(size_t)min(m0 + tid, p.M - 1) * ng + g1];
    }
    __builtin_amdgcn_s_waitcnt(0);   // nothing in flight at loop entry
    __syncthreads();

    // int32 accumulators of the pair in flight (P[s]) and of the pair being rescaled (P[s^1])
    v16i P[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 2; ++i) P[s][i] = zero16;
    float sw_prev[TN];   // group scale of the pair left over from the previous group
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) sw_prev[nt] = 0.0f;

    // one group; PAR = g & 1 selects the register sets and the LDS stage at compile time
    auto group_step = [&](int g, auto parc) {
        constexpr int PAR = decltype(parc)::value;
        // B fragments of this group: b[nt][j] = the 16 k of chunk 2j+h as int8.  A group past
        // the end (odd group count) gets scale 0 and contributes nothing.
        float sw_cur[TN];
        v4i b[TN][4];
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
            sw_cur[nt] = g < ng ? (float)meta[PAR].sw[nt] : 0.0f;
            if (PART8) {
#pragma unroll
                for (int j = 0; j < 4; ++j) b[nt][j] = wq[PAR][nt][j];
            } else {
                const uint32_t zb = zbias(PAR ? (meta[PAR].zraw[nt] >> 4) : (meta[PAR].zraw[nt] & 15));
                b[nt][0] = unpack16((uint32_t)wq[PAR][nt][0][0], (uint32_t)wq[PAR][nt][0][1], zb);
                b[nt][1] = unpack16((uint32_t)wq[PAR][nt][1][0], (uint32_t)wq[PAR][nt][1][1], zb);
                b[nt][2] = unpack16((uint32_t)wq[PAR][nt][0][2], (uint32_t)wq[PAR][nt][0][3], zb);
                b[nt][3] = unpack16((uint32_t)wq[PAR][nt][1][2], (uint32_t)wq[PAR][nt][1][3], zb);
            }
        }
        // request group g+2 (clamped at the end: a harmless re-read keeps the body branch-free)
        const int gn = min(g + 2, ng - 1);
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) areg[PAR][i] = *(const v4i *)(a_src[i] + (size_t)gn * G);
        load_b(gn, wq[PAR]);
        load_meta(gn, meta[PAR]);
        if (!ACT_PT && !DUMP && tid < BM) sa_reg[PAR] = (float)p.xscale[(size_t)min(m0 + tid, p.M - 1) * ng + gn];

        // activation fragments: af[step % 3][tile of the pair], fetched two steps ahead
        const uint8_t *a_base = lds_a + PAR * A_STAGE + (mw0 + n32) * A_STRIDE + h * 16;
        v4i af[3][NA];
        auto load_af = [&](auto stc) {
            constexpr int st = decltype(stc)::value, q = st / 4, j = st % 4;
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int mt = (2 * q + i) / TN;
                af[st % 3][i] = *(const v4i *)(a_base + mt * 32 * A_STRIDE + j * 32);
            }
        };
        load_af(std::integral_constant<int, 0>{});
        load_af(std::integral_constant<int, 1>{});
        __builtin_amdgcn_sched_barrier(0);

        static_for<0, NSTEP>([&](auto stc) {
            constexpr int st = decltype(stc)::value, q = st / 4, j = st % 4, s = q & 1;
            constexpr int t0 = 2 * q, t1 = 2 * q + 1;                 // tiles of the pair in flight
            constexpr int qp = (q + NP - 1) % NP;                     // pair being rescaled
            constexpr int u0 = 2 * qp, u1 = 2 * qp + 1;
            const int gp = q == 0 ? g - 1 : g;                        // ... and its group
            if constexpr (st + 2 < NSTEP) load_af(std::integral_constant<int, st + 2>{});
            // slot 1: first tile of the pair
            P[s][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[st % 3][0], b[t0 % TN][j], j == 0 ? zero16 : P[s][0], 0, 0, 0);
            finish4(P[s ^ 1][0], std::integral_constant<int, u0 / TN>{}, std::integral_constant<int, u0 % TN>{},
                    std::integral_constant<int, j>{}, q == 0 ? sw_prev[u0 % TN] : sw_cur[u0 % TN], gp);
            // slot 2: second tile of the pair
            P[s][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[st % 3][NA - 1], b[t1 % TN][j], j == 0 ? zero16 : P[s][1], 0, 0, 0);
            finish4(P[s ^ 1][1], std::integral_constant<int, u1 / TN>{}, std::integral_constant<int, u1 % TN>{},
                    std::integral_constant<int, j>{}, q == 0 ? sw_prev[u1 % TN] : sw_cur[u1 % TN], gp);
            if (!DUMP) {
                // issue order: MFMA, the LDS reads and 8 vector instructions in its shadow, twice
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, ACT_PT ? 1 : 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, ACT_PT ? 8 : 12, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, ACT_PT ? 1 : 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, ACT_PT ? 8 : 12, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        });

        // activations of group g+1 (requested one iteration ago) go to the other LDS stage
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) *(v4i *)(lds_a + (PAR ^ 1) * A_STAGE + a_dst[i]) = areg[PAR ^ 1][i];
        if (!ACT_PT && !DUMP && tid < BM) lds_sa[((g + 1) % 3) * BM + tid] = sa_reg[PAR ^ 1];
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) sw_prev[nt] = sw_cur[nt];
        __syncthreads();
    };
    for (int g = 0; g < ng; g += 2) {
        group_step(g, std::integral_constant<int, 0>{});
        group_step(g + 1, std::integral_constant<int, 1>{});
    }
    const int g_last = ((ng + 1) & ~1) - 1;   // group index the pending pair belongs to (may be the phantom one)
    // the last pair of the last group is still waiting for its rescale
    static_for<0, 4>([&](auto jc) {
        constexpr int u0 = 2 * (NP - 1), u1 = u0 + 1, sp = (NP - 1) & 1;
        finish4(P[sp][0], std::integral_constant<int, u0 / TN>{}, std::integral_constant<int, u0 % TN>{}, jc,
                sw_prev[u0 % TN], g_last);
        finish4(P[sp][1], std::integral_constant<int, u1 / TN>{}, std::integral_constant<int, u1 % TN>{}, jc,
                sw_prev[u1 % TN], g_last);
    });
    if (DUMP) return;

    // ---- epilogue: token scale, fp16, scatter (Sec. 3.4) ------------------------------
    // per token tile: the 16 token scales of the lane's rows are fetched together (clamped,
    // unconditional) so that the loads overlap instead of costing one round trip per row
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        float sa[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            sa[r] = ACT_PT ? (float)p.xscale[min(m, p.M - 1)] : 1.0f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
            for (int nt = 0; nt < TN; ++nt)
                if (m < p.M && ch[nt] >= 0)
                    p.y[(size_t)m * p.N + ch[nt]] = (half_t)(acc[mt][nt][r] * sa[r]);
        }
    }
}

template <typename C, int MINW, bool DUMP, bool ACT_PT>
__global__ __launch_bounds__(C::THREADS, MINW) void linear_prefill_kernel(LinearParams p, int nbm, int nb8,
                                                                         int nb4, int per_xcd)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[2 * C::A_STAGE];
    __shared__ __attribute__((aligned(16))) float lds_sa[(ACT_PT || DUMP) ? 4 : 3 * C::BM];
    // Consecutive logical ids share a weight tile (same bn, successive bm); give each XCD
    // (blocks are dealt round-robin to the 8 XCDs) a contiguous range of logical ids so that
    // its L2 sees each weight tile and each activation tile from as few places as possible.
    const int total = nbm * (nb8 + nb4);
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= total) return;
    const int bn = L / nbm, bm = L % nbm;
    constexpr int T16 = C::BN / TILE_N;
    if (bn < nb8)
        prefill_block<C, DUMP, ACT_PT, true>(p, bm * C::BM, bn * T16, lds_a, lds_sa);
    else
        prefill_block<C, DUMP, ACT_PT, false>(p, bm * C::BM, (bn - nb8) * T16, lds_a, lds_sa);
}

template <typename C, int MINW>
static int launch_shape(const LinearParams &p, hipStream_t st)
{
    constexpr int BM = C::BM, BN = C::BN;
    const int nbm = (p.M + BM - 1) / BM;
    const int nb8 = (p.ntiles8 * TILE_N + BN - 1) / BN, nb4 = (p.ntiles4 * TILE_N + BN - 1) / BN;
    const int total = nbm * (nb8 + nb4);
    const int per_xcd = (total + 7) / 8;
    dim3 grid(per_xcd * 8), block(C::THREADS);
    if (p.P)
        hipLaunchKernelGGL((linear_prefill_kernel<C, MINW, true, true>), grid, block, 0, st, p, nbm, nb8, nb4, per_xcd);
    else if (p.act_per_token)
        hipLaunchKernelGGL((linear_prefill_kernel<C, MINW, false, true>), grid, block, 0, st, p, nbm, nb8, nb4, per_xcd);
    else
        hipLaunchKernelGGL((linear_prefill_kernel<C, MINW, false, false>), grid, block, 0, st, p, nbm, nb8, nb4, per_xcd);
    return (int)hipGetLastError();
}

int launch_linear_prefill(const LinearParams &p, hipStream_t st)
{
    if (p.M == 0 || p.N == 0) return hipSuccess;
    switch (p.tune) {
    case 1: return launch_shape<Shape<1, 4, 4, 2>, 1>(p, st);    // 128 x 256, one wave per SIMD
    case 2: return launch_shape<Shape<2, 2, 2, 2>, 2>(p, st);    // 128 x 128, wave tile 64 x 64
    case 3: return launch_shape<Shape<2, 4, 4, 1>, 2>(p, st);    // 256 x 128, 8 waves, wave tile 128 x 32
    case 4: return launch_shape<Shape<2, 4, 2, 2>, 2>(p, st);    // 128 x 256, 8 waves, wave tile 64 x 64
    default: return launch_shape<Shape<1, 4, 4, 1>, 2>(p, st);   // 128 x 128, wave tile 128 x 32
    }
}

}  // namespace mixllm
