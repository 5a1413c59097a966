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
#include "internal.h"

namespace mixllm {

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

// Launch shape (from sweeps on the Llama-shaped layers): at most 8 waves per CU in total; K
// is split WPB ways inside a block when there are too few tiles for that, and a wave takes
// two tiles when M is large enough for the activation traffic to matter.
int launch_linear_decode(const LinearParams &p, hipStream_t st)
{
    if (p.M == 0 || p.N == 0) return hipSuccess;
    const int tiles = p.ntiles8 + p.ntiles4;
    const int nquads = (p.ng + 3) / 4;
    int tpw = (tiles >= 300 && p.M > 4) ? 2 : 1;
    int wpb = 1;
    while (wpb < 8 && wpb * 2 <= nquads && tiles * wpb * 2 <= 2048) wpb *= 2;
    if (p.tune > 0) {   // experiments: tune = 100 * tpw + wpb
        tpw = p.tune / 100;
        wpb = p.tune % 100;
    }
    return tpw == 2 ? launch_wpb<2>(p, wpb, st) : launch_wpb<1>(p, wpb, st);
}

}  // namespace mixllm
