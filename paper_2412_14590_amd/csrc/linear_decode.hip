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
//  * Activations are the A operand: row = token (padded to 16 with zeros), read from the
//    L2-resident xq; M only changes how many rows are non-zero.
//  * One int32 MFMA accumulator per group (2 MFMAs = 128 k), then float rescale by the
//    group scale (step 2, Sec. 3.3); the token scale is applied once at the end when it
//    does not depend on the group.
//  * Epilogue scatters fp16 results to their original channel (Sec. 3.4).
// 8-bit tiles and 4-bit tiles are different block ranges of the same launch.
#include "internal.h"

namespace mixllm {

template <int TPW, int WPB, bool DUMP, bool ACT_PT, bool PART8>
static __device__ inline void decode_block(const LinearParams &p, int tile0, float (*red)[TPW][4][64])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, ks = lane >> 4;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;          // real rows of this part
    const int joff = PART8 ? 0 : p.n8;              // position of the part in the concatenation
    const int nsteps = p.K / 64;
    const int nquads = (p.ng + 3) / 4;
    const int q_lo = nquads * wave / WPB, q_hi = nquads * (wave + 1) / WPB;

    // A operand: lane (c, ks) supplies token c, k = 16*ks..+15 of each 64-k step
    const bool mvalid = c < p.M;
    const int8_t *xrow = p.xq + (size_t)min(c, p.M - 1) * p.K + ks * 16;

    int tile[TPW], row[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        tile[t] = min(tile0 + t, ntiles - 1);
        row[t] = tile[t] * TILE_N + c;
    }
    // output rows held by this lane: tokens 4*ks + r
    int ch[TPW];
    if (DUMP) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) ch[t] = row[t] < nrows ? p.perm[joff + row[t]] : -1;
    }

    float acc[TPW][4];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = 0.0f;

    float sw_row[TPW];
    if (PART8 && !DUMP && p.w8_per_channel) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) sw_row[t] = (float)p.s8[row[t]];
    }

    for (int q = q_lo; q < q_hi; ++q) {
        const int g0 = 4 * q;
        // group metadata of 4 groups at once (arrays are zero padded to a multiple of 8 groups)
        half_t sw4[TPW][4];
        uint32_t zq[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            if (!PART8) {
                if (!DUMP) {
                    const uint2 s = *(const uint2 *)(p.s4 + (size_t)row[t] * p.ngp + g0);
                    __builtin_memcpy(sw4[t], &s, 8);
                }
                zq[t] = *(const uint16_t *)(p.z4 + (size_t)row[t] * (p.ngp / 2) + g0 / 2);
            } else if (!DUMP && !p.w8_per_channel) {
                const uint2 s = *(const uint2 *)(p.s8 + (size_t)row[t] * p.ngp + g0);
                __builtin_memcpy(sw4[t], &s, 8);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = g0 + u;
            const bool gvalid = g < p.ng;
            const int gc = min(g, p.ng - 1);
            v4i a0 = *(const v4i *)(xrow + (size_t)gc * G);
            v4i a1 = *(const v4i *)(xrow + (size_t)gc * G + 64);
            if (!(mvalid && gvalid)) {
                a0 = v4i{0, 0, 0, 0};
                a1 = v4i{0, 0, 0, 0};
            }
            float sa[4];
            if (!ACT_PT && !DUMP) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    sa[r] = (float)p.xscale[(size_t)min(4 * ks + r, p.M - 1) * p.ng + gc];
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                v4i b0, b1;
                float sw = 0.0f;
                if (PART8) {
                    const uint8_t *base =
                        (const uint8_t *)p.w8 + (((size_t)tile[t] * nsteps + 2 * gc) * 64 + lane) * 16;
                    b0 = *(const v4i *)base;
                    b1 = *(const v4i *)(base + 1024);
                    if (!DUMP) sw = p.w8_per_channel ? sw_row[t] : (float)sw4[t][u];
                } else {
                    const v4i w = *(const v4i *)(p.w4 + (((size_t)tile[t] * p.ng + gc) * 64 + lane) * 16);
                    const uint32_t zb = zbias((zq[t] >> (4 * u)) & 15);
                    b0 = unpack16((uint32_t)w[0], (uint32_t)w[1], zb);
                    b1 = unpack16((uint32_t)w[2], (uint32_t)w[3], zb);
                    if (!DUMP) sw = (float)sw4[t][u];
                }
                v4i P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, v4i{0, 0, 0, 0}, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, P, 0, 0, 0);
                if (DUMP) {
                    if (gvalid && ch[t] >= 0) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int m = 4 * ks + r;
                            if (m < p.M && tile0 + t < ntiles)
                                p.P[((size_t)m * p.N + ch[t]) * p.ng + g] = P[r];
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (ACT_PT)
                            acc[t][r] += (float)P[r] * sw;
                        else
                            acc[t][r] += (float)P[r] * (sw * sa[r]);
                    }
                }
            }
        }
    }
    if (DUMP) return;

    // reduce the K-split partial outputs of the WPB waves through LDS
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][t][r][lane] = acc[t][r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < TPW * 256; idx += WPB * 64) {
        const int t = idx >> 8, r = (idx >> 6) & 3, l = idx & 63;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < WPB; ++w) v += red[w][t][r][l];
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
    __shared__ float red[DUMP ? 1 : WPB][TPW][4][64];
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

// Launch shape: enough waves to keep >= 8 per CU busy on the small layers (K split 8 or 16
// ways inside the block), two tiles per wave once there are plenty of tiles so that the
// activation fragments are fetched half as often.
int launch_linear_decode(const LinearParams &p, hipStream_t st)
{
    if (p.M == 0 || p.N == 0) return hipSuccess;
    const int tiles = p.ntiles8 + p.ntiles4;
    const int nquads = (p.ng + 3) / 4;
    if (nquads >= 16 && tiles < 2048) return launch_cfg<1, 16>(p, st);
    if (tiles >= 1024 && p.M > 4) return launch_cfg<2, 8>(p, st);
    if (nquads >= 8) return launch_cfg<1, 8>(p, st);
    return launch_cfg<1, 4>(p, st);
}

}  // namespace mixllm
