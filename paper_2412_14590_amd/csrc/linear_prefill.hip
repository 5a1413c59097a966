// Prefill path of the quantized linear (M > 16 tokens): int8-MFMA bound.
//
// Block = 4 waves, block tile 128 tokens x 256 output channels, waves side by side along N
// (wave tile 128 x 64 = 4 x 2 MFMA tiles of 32x32, v_mfma_i32_32x32x32_i8).
//  * Activations (A operand, rows = tokens) are staged per quantization group through LDS,
//    double buffered, one barrier per group; rows are padded to 144 bytes so that the
//    16-byte fragment reads of 32 lanes fall in distinct banks.
//  * Packed weights (B operand, columns = channels) go HBM/L2 -> registers directly: each
//    wave owns its 64 channels, so no weight byte is shared between waves and none passes
//    through LDS.  Two 16-byte loads per lane fetch one group of one 32-channel tile.
//  * uint4 -> int8 unpack with zero-point subtraction in registers (step 1 of the two-step
//    dequantization, Sec. 3.3), reused by the 4 token tiles of the wave.
//  * Per group: 4 chained MFMAs (K = 128) into an int32 accumulator, then int->float and
//    one FMA per element with the group scale (step 2, Sec. 3.3).  The channel a lane owns
//    is the MFMA column, so the group scale is one register per lane.
//  * Epilogue: token scale, fp16 conversion, scatter to the original channel (Sec. 3.4).
// 8-bit and 4-bit channel tiles are different block ranges of one launch.
#include "internal.h"

namespace mixllm {

constexpr int BM = 128;            // tokens per block
constexpr int BN = 256;            // channels per block (16 packed tiles of 16)
constexpr int A_STRIDE = G + 16;   // bytes per LDS row of the activation tile
constexpr int A_STAGE = BM * A_STRIDE;

template <bool DUMP, bool ACT_PT, bool PART8>
static __device__ inline void prefill_block(const LinearParams &p, int m0, int t16_0, uint8_t *lds_a,
                                            float *lds_sa)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n32 = lane & 31, h = lane >> 5;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;
    const int joff = PART8 ? 0 : p.n8;
    const int nsteps = p.K / 64;
    const int ng = p.ng;

    // this lane's channel in each of the wave's two 32-channel tiles
    int tile16[2], rw[2];
    bool cvalid[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int t = t16_0 + 4 * wave + 2 * nt + (n32 >> 4);
        tile16[nt] = min(t, ntiles - 1);
        rw[nt] = tile16[nt] * TILE_N + (n32 & 15);
        cvalid[nt] = t < ntiles && rw[nt] < nrows;
    }

    // ---- loaders -------------------------------------------------------------------
    // activation tile of one group: 128 rows x 128 bytes = 1024 chunks of 16 bytes, 4 per thread
    auto load_a = [&](int g, v4i (&areg)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + 256 * i, row = id >> 3, c16 = id & 7;
            const int m = m0 + row;
            areg[i] = *(const v4i *)(p.xq + (size_t)min(m, p.M - 1) * p.K + (size_t)g * G + c16 * 16);
            if (m >= p.M) areg[i] = v4i{0, 0, 0, 0};
        }
    };
    auto store_a = [&](int stage, const v4i (&areg)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + 256 * i, row = id >> 3, c16 = id & 7;
            *(v4i *)(lds_a + stage * A_STAGE + row * A_STRIDE + c16 * 16) = areg[i];
        }
    };
    // weights of one group for the wave's two 32-channel tiles.
    //  4-bit: wq[nt][0] = 16-k chunks h and 4+h, wq[nt][1] = chunks 2+h and 6+h (packed)
    //  8-bit: wq[nt][j] = chunk 2j+h (int8)
    auto load_b = [&](int g, v4i (&wq)[2][4]) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (PART8) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ch = 2 * j + h;
                    wq[nt][j] = *(const v4i *)((const uint8_t *)p.w8 +
                                               (((size_t)tile16[nt] * nsteps + 2 * g + (ch >> 2)) * 64 +
                                                (n32 & 15) + 16 * (ch & 3)) * 16);
                }
            } else {
                const uint8_t *base = p.w4 + (((size_t)tile16[nt] * ng + g) * 64 + (n32 & 15)) * 16;
                wq[nt][0] = *(const v4i *)(base + 16 * h * 16);
                wq[nt][1] = *(const v4i *)(base + 16 * (2 + h) * 16);
            }
        }
    };
    struct Meta {
        float sw[2];
        uint32_t zb[2];
    };
    auto load_meta = [&](int g, Meta &mt) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            mt.sw[nt] = 0.0f;
            mt.zb[nt] = 0;
            if (PART8) {
                if (!DUMP)
                    mt.sw[nt] = (float)(p.w8_per_channel ? p.s8[rw[nt]] : p.s8[(size_t)rw[nt] * p.ngp + g]);
            } else {
                if (!DUMP) mt.sw[nt] = (float)p.s4[(size_t)rw[nt] * p.ngp + g];
                mt.zb[nt] = zbias(z4_load(p.z4, rw[nt], g, p.ngp));
            }
        }
    };

    int ch[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) ch[nt] = cvalid[nt] ? p.perm[joff + rw[nt]] : -1;

    v16i zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0;

    float acc[4][2][16];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    // ---- prologue ------------------------------------------------------------------
    v4i areg[4];
    v4i wq_cur[2][4], wq_nxt[2][4];
    Meta meta_cur, meta_nxt;
    load_a(0, areg);
    load_b(0, wq_cur);
    load_meta(0, meta_cur);
    store_a(0, areg);
    if (!ACT_PT && !DUMP && tid < BM) lds_sa[tid] = (float)p.xscale[(size_t)min(m0 + tid, p.M - 1) * ng];
    __syncthreads();

    for (int g = 0; g < ng; ++g) {
        const int cur = g & 1;
        const bool more = g + 1 < ng;
        float sa_nxt = 0.0f;
        if (more) {
            load_a(g + 1, areg);
            load_b(g + 1, wq_nxt);
            load_meta(g + 1, meta_nxt);
            if (!ACT_PT && !DUMP && tid < BM)
                sa_nxt = (float)p.xscale[(size_t)min(m0 + tid, p.M - 1) * ng + g + 1];
        }
        // B fragments of this group: b[nt][j] = the 16 k of chunk 2j+h as int8
        v4i b[2][4];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (PART8) {
#pragma unroll
                for (int j = 0; j < 4; ++j) b[nt][j] = wq_cur[nt][j];
            } else {
                const uint32_t zb = meta_cur.zb[nt];
                b[nt][0] = unpack16((uint32_t)wq_cur[nt][0][0], (uint32_t)wq_cur[nt][0][1], zb);
                b[nt][2] = unpack16((uint32_t)wq_cur[nt][0][2], (uint32_t)wq_cur[nt][0][3], zb);
                b[nt][1] = unpack16((uint32_t)wq_cur[nt][1][0], (uint32_t)wq_cur[nt][1][1], zb);
                b[nt][3] = unpack16((uint32_t)wq_cur[nt][1][2], (uint32_t)wq_cur[nt][1][3], zb);
            }
        }
        const uint8_t *a_base = lds_a + cur * A_STAGE + n32 * A_STRIDE + h * 16;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            v4i a[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] = *(const v4i *)(a_base + mt * 32 * A_STRIDE + j * 32);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                v16i P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[0], b[nt][0], zero16, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[1], b[nt][1], P, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[2], b[nt][2], P, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[3], b[nt][3], P, 0, 0, 0);
                if (DUMP) {
                    if (ch[nt] >= 0) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int m = m0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                            if (m < p.M) p.P[((size_t)m * p.N + ch[nt]) * ng + g] = P[r];
                        }
                    }
                } else if (ACT_PT) {
                    const float sw = meta_cur.sw[nt];
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mt][nt][r] += (float)P[r] * sw;
                } else {
                    const float sw = meta_cur.sw[nt];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float sa = lds_sa[cur * BM + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3)];
                        acc[mt][nt][r] += (float)P[r] * (sw * sa);
                    }
                }
            }
        }
        if (more) {
            store_a(cur ^ 1, areg);
            if (!ACT_PT && !DUMP && tid < BM) lds_sa[(cur ^ 1) * BM + tid] = sa_nxt;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) wq_cur[nt][j] = wq_nxt[nt][j];
            meta_cur = meta_nxt;
        }
        __syncthreads();
    }
    if (DUMP) return;

    // ---- epilogue: token scale, fp16, scatter (Sec. 3.4) ------------------------------
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            if (m < p.M) {
                const float sa = ACT_PT ? (float)p.xscale[m] : 1.0f;
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    if (ch[nt] >= 0) p.y[(size_t)m * p.N + ch[nt]] = (half_t)(acc[mt][nt][r] * sa);
            }
        }
}

template <bool DUMP, bool ACT_PT>
__global__ __launch_bounds__(256) void linear_prefill_kernel(LinearParams p, int nbm, int nb8, int nb4,
                                                             int per_xcd)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[2 * A_STAGE];
    __shared__ float lds_sa[2 * BM];
    // Consecutive logical ids share a weight tile (same bn, successive bm); give each XCD
    // (blocks are dealt round-robin to the 8 XCDs) a contiguous range of logical ids so that
    // its L2 sees each weight tile and each activation tile from as few places as possible.
    const int total = nbm * (nb8 + nb4);
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || L >= total) return;
    const int bn = L / nbm, bm = L % nbm;
    if (bn < nb8)
        prefill_block<DUMP, ACT_PT, true>(p, bm * BM, bn * (BN / TILE_N), lds_a, lds_sa);
    else
        prefill_block<DUMP, ACT_PT, false>(p, bm * BM, (bn - nb8) * (BN / TILE_N), lds_a, lds_sa);
}

int launch_linear_prefill(const LinearParams &p, hipStream_t st)
{
    if (p.M == 0 || p.N == 0) return hipSuccess;
    const int nbm = (p.M + BM - 1) / BM;
    const int nb8 = (p.ntiles8 * TILE_N + BN - 1) / BN, nb4 = (p.ntiles4 * TILE_N + BN - 1) / BN;
    const int total = nbm * (nb8 + nb4);
    const int per_xcd = (total + 7) / 8;
    dim3 grid(per_xcd * 8), block(256);
    if (p.P)
        hipLaunchKernelGGL((linear_prefill_kernel<true, true>), grid, block, 0, st, p, nbm, nb8, nb4, per_xcd);
    else if (p.act_per_token)
        hipLaunchKernelGGL((linear_prefill_kernel<false, true>), grid, block, 0, st, p, nbm, nb8, nb4, per_xcd);
    else
        hipLaunchKernelGGL((linear_prefill_kernel<false, false>), grid, block, 0, st, p, nbm, nb8, nb4, per_xcd);
    return (int)hipGetLastError();
}

}  // namespace mixllm
