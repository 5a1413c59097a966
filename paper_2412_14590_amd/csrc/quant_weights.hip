// Offline weight path: quantize fp16 weights straight into the packed layouts, and convert
// between canonical (one code per byte, row-major) and packed arrays.
// Quantizer: Sec. 2 formula; 8-bit symmetric / 4-bit asymmetric group-wise, Sec. 3.1.2 and 4.1.
// The packed layouts are the ahead-of-time prepacking of Sec. 3.3, chosen for gfx950:
// every 16-byte slot is exactly what one lane feeds to an int8 MFMA as its B operand.
#include "internal.h"

namespace mixllm {

typedef half_t h8 __attribute__((ext_vector_type(8)));

static __device__ inline float block_max_256(float v, float *red)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    v = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return v;
}

// ------------------------------------------------- order of the concatenated rows --
// feature_perm from a DEVICE list of the 8-bit channels (Sec. 3.4: the two parts own different
// channel indices; Alg. 1's per-layer slice arrives on the device from mixllm_select_salient):
// the listed channels ascending, then all others ascending.  No scratch memory: while the order
// is being built, bit 31 of perm[c] says "channel c is in the list" and the low 31 bits are the
// entry under construction (channel numbers are below 2^24).

__global__ __launch_bounds__(256) void perm_clear_kernel(int32_t *__restrict__ perm, int N)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < N) perm[c] = 0;
}

// An index outside [0, N) is ignored; a channel listed twice is marked once.
__global__ __launch_bounds__(256) void perm_mark_kernel(const int32_t *__restrict__ idx, int n8, int32_t *__restrict__ perm,
                                                        int N)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n8) {
        const int c = idx[i];
        if (c >= 0 && c < N) perm[c] = (int32_t)0x80000000u;
    }
}

// One block walks the channels in order, 1024 at a time: a marked channel goes to the next free
// position of the first part, an unmarked one to the next free position of the second part.
// Position and channel of a write differ, so a write keeps the mark bit of the word it lands in
// (only the thread that owns a position writes its low bits; the mark bit is only ever read).
// With fewer than n8 distinct valid indices in the list the second part would run past N: those
// writes are dropped (the call's contract is a list of n8 distinct channels; a bad list gives an
// unspecified order, never an access out of bounds).
__global__ __launch_bounds__(1024) void perm_scan_kernel(int32_t *__restrict__ perm, int N, int n8)
{
    __shared__ int wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int marked_before = 0;   // marked channels in the chunks already walked
    for (int c0 = 0; c0 < N; c0 += 1024) {
        const int c = c0 + tid;
        const int flag = (c < N && perm[c] < 0) ? 1 : 0;
        int inc = flag;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o, 64);
            if (lane >= o) inc += t;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();   // every flag of the chunk has been read; wave totals are visible
        int base = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            if (w < wave) base += wave_tot[w];
            total += wave_tot[w];
        }
        const int a = marked_before + base + inc - flag;   // marked channels before c
        if (c < N) {
            const int pos = flag ? a : n8 + (c - a);
            if (pos < N) perm[pos] = (perm[pos] & (int32_t)0x80000000u) | c;
        }
        marked_before += total;
        __syncthreads();   // wave_tot is rewritten by the next chunk; this chunk's writes are done
    }
    for (int c = tid; c < N; c += 1024) perm[c] &= 0x7fffffff;
}

int launch_build_feature_perm(int N, int n8, const int32_t *salient_idx_dev, int32_t *perm, hipStream_t st)
{
    if (N <= 0) return (int)hipSuccess;
    hipLaunchKernelGGL(perm_clear_kernel, dim3((N + 255) / 256), dim3(256), 0, st, perm, N);
    if (n8 > 0)
        hipLaunchKernelGGL(perm_mark_kernel, dim3((n8 + 255) / 256), dim3(256), 0, st, salient_idx_dev, n8, perm, N);
    hipLaunchKernelGGL(perm_scan_kernel, dim3(1), dim3(1024), 0, st, perm, N, n8);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------ quantize + pack --

// blocks [0, n8p): one 8-bit row each; blocks [n8p, n8p + n4p): one 4-bit row each.
__global__ __launch_bounds__(256) void quantize_pack_kernel(
    const half_t *__restrict__ W, const int32_t *__restrict__ perm, int K, int n8, int n4, int n8p,
    int ng, int ngp, int w8_per_channel, int8_t *__restrict__ w8, uint8_t *__restrict__ w4,
    half_t *__restrict__ s8, half_t *__restrict__ s4, uint8_t *__restrict__ z4)
{
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const int nsteps = K / 64;
    if ((int)blockIdx.x < n8p) {
        // ---- 8-bit row: thread handles 16 consecutive k (one packed slot) per iteration
        const int r = blockIdx.x;
        const bool real = r < n8;
        const half_t *row = real ? W + (size_t)perm[r] * K : nullptr;
        const int nchunk = K / 16;
        float s_row = 1.0f;
        if (w8_per_channel) {
            float amax = 0.0f;
            if (real)
                for (int c = tid; c < nchunk; c += 256) {
                    h8 a = *(const h8 *)(row + c * 16), b = *(const h8 *)(row + c * 16 + 8);
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        amax = fmaxf(amax, fmaxf(fabsf((float)a[i]), fabsf((float)b[i])));
                }
            amax = block_max_256(amax, red);
            half_t s16 = real ? store_scale(amax / 127.0f) : (half_t)0.0f;
            if (tid == 0) s8[r] = s16;
            s_row = (float)s16;
        } else {
            // zero the metadata padding of this row (groups ng..ngp-1)
            for (int g = ng + tid; g < ngp; g += 256) s8[(size_t)r * ngp + g] = (half_t)0.0f;
        }
        // nchunk is a multiple of 8, so the 8 lanes of one group are always active together
        for (int c = tid; c < nchunk; c += 256) {
            uint4 out = make_uint4(0, 0, 0, 0);
            float s = s_row;
            if (real) {
                h8 a = *(const h8 *)(row + c * 16), b = *(const h8 *)(row + c * 16 + 8);
                if (!w8_per_channel) {
                    float amax = 0.0f;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        amax = fmaxf(amax, fmaxf(fabsf((float)a[i]), fabsf((float)b[i])));
#pragma unroll
                    for (int o = 4; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 8));
                    half_t s16 = store_scale(amax / 127.0f);
                    if ((c & 7) == 0) s8[(size_t)r * ngp + (c >> 3)] = s16;
                    s = (float)s16;
                }
                uint32_t w[4] = {0, 0, 0, 0};
                const float rs = recip(s);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float v = (i < 8) ? (float)a[i] : (float)b[i - 8];
                    float t = fminf(fmaxf(__builtin_rintf(quotient(v, s, rs)), -127.0f), 127.0f);
                    w[i >> 2] |= ((uint32_t)(int)t & 0xffu) << (8 * (i & 3));
                }
                out = make_uint4(w[0], w[1], w[2], w[3]);
            } else if (!w8_per_channel && (c & 7) == 0) {
                s8[(size_t)r * ngp + (c >> 3)] = (half_t)0.0f;
            }
            *(uint4 *)((uint8_t *)w8 + w8_slot_offset(r, c >> 2, c & 3, nsteps)) = out;
        }
    } else {
        // ---- 4-bit row: 16 lanes per group, 8 consecutive k (one packed dword) per lane
        const int r = blockIdx.x - n8p;
        const bool real = r < n4;
        const half_t *row = real ? W + (size_t)perm[n8 + r] * K : nullptr;
        const int sub = tid >> 4, i16 = tid & 15;
        for (int g0 = 0; g0 < ngp; g0 += 16) {
            const int g = g0 + sub;
            float sc = 0.0f, zf = 0.0f;
            half_t s16 = (half_t)0.0f;
            uint32_t packed = 0;
            if (real && g < ng) {
                h8 v = *(const h8 *)(row + (size_t)g * G + i16 * 8);
                float mn = 0.0f, mx = 0.0f;   // the range always contains 0
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    mn = fminf(mn, (float)v[i]);
                    mx = fmaxf(mx, (float)v[i]);
                }
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) {
                    mn = fminf(mn, __shfl_xor(mn, o, 16));
                    mx = fmaxf(mx, __shfl_xor(mx, o, 16));
                }
                s16 = store_scale((mx - mn) / 15.0f);
                sc = (float)s16;
                const float rsc = recip(sc);
                zf = fminf(fmaxf(__builtin_rintf(quotient(-mn, sc, rsc)), 0.0f), 15.0f);
                uint32_t code[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float t = __builtin_rintf(quotient((float)v[i], sc, rsc)) + zf;
                    code[i] = (uint32_t)(int)fminf(fmaxf(t, 0.0f), 15.0f);
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) packed |= (code[b] | (code[b + 4] << 4)) << (8 * b);
            }
            if (g < ng) {
                // lane i16 holds k-local 8*i16..+7: 16-k chunk c = i16/2, dword i16%2
                const int c = i16 >> 1, ks = c & 3, half = c >> 2;
                *(uint32_t *)(w4 + w4_slot_offset(r, g, ks, ng) + half * 8 + (i16 & 1) * 4) = packed;
            }
            // metadata, including the zero padding up to ngp
            int z = (int)zf;
            int z_next = __shfl_down(z, 16, 64);   // zero point of group g+1 (next 16-lane set)
            if (i16 == 0 && g < ngp) {
                s4[(size_t)r * ngp + g] = s16;
                if ((sub & 1) == 0) z4[(size_t)r * (ngp / 2) + (g >> 1)] = (uint8_t)(z | (z_next << 4));
            }
        }
    }
}

int launch_quantize_weights(const mixllm_desc &d, const void *W, void *w8, void *w4, void *s8,
                            void *s4, void *z4, const int32_t *perm, hipStream_t st)
{
    const int n4 = d.N - d.n8, n8p = round_up(d.n8, TILE_N), n4p = round_up(n4, TILE_N);
    const int ng = d.K / G, ngp = round_up(ng, 8);
    if (n8p + n4p == 0) return hipSuccess;
    hipLaunchKernelGGL(quantize_pack_kernel, dim3(n8p + n4p), dim3(256), 0, st, (const half_t *)W,
                       perm, d.K, d.n8, n4, n8p, ng, ngp, d.w8_group == d.K ? 1 : 0, (int8_t *)w8,
                       (uint8_t *)w4, (half_t *)s8, (half_t *)s4, (uint8_t *)z4);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------ canonical -> packed --

__global__ __launch_bounds__(256) void pack_w4_kernel(const uint8_t *__restrict__ q4, int n4, int n4p,
                                                      int K, int ng, uint32_t *__restrict__ w4)
{
    const size_t total = (size_t)n4p * K / 8;   // packed dwords
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
        const int dw = o & 3, l = (o >> 2) & 63;
        const size_t tg = o >> 8;                // tile * ng + g
        const int g = (int)(tg % ng), tile = (int)(tg / ng);
        const int r = tile * TILE_N + (l & 15), ks = l >> 4;
        const int k0 = g * G + (dw >> 1) * 64 + ks * 16 + (dw & 1) * 8;
        uint32_t packed = 0;
        if (r < n4) {
            const uint8_t *src = q4 + (size_t)r * K + k0;
#pragma unroll
            for (int b = 0; b < 4; ++b)
                packed |= ((uint32_t)(src[b] & 15) | ((uint32_t)(src[b + 4] & 15) << 4)) << (8 * b);
        }
        w4[o] = packed;
    }
}

__global__ __launch_bounds__(256) void pack_w8_kernel(const int8_t *__restrict__ q8, int n8, int n8p,
                                                      int K, uint4 *__restrict__ w8)
{
    const int nsteps = K / 64;
    const size_t total = (size_t)n8p * K / 16;   // 16-byte slots
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
        const int l = o & 63;
        const size_t ts = o >> 6;
        const int step = (int)(ts % nsteps), tile = (int)(ts / nsteps);
        const int r = tile * TILE_N + (l & 15), ks = l >> 4;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < n8) v = *(const uint4 *)(q8 + (size_t)r * K + step * 64 + ks * 16);
        w8[o] = v;
    }
}

// scales (fp16 [rows][ncan] -> [rowsp][nstride], zero padded); also used with ncan = nstride = 1
__global__ __launch_bounds__(256) void pack_scales_kernel(const half_t *__restrict__ src, int rows,
                                                          int rowsp, int ncan, int nstride,
                                                          half_t *__restrict__ dst)
{
    const size_t total = (size_t)rowsp * nstride;
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
        const int r = (int)(o / nstride), g = (int)(o % nstride);
        dst[o] = (r < rows && g < ncan) ? src[(size_t)r * ncan + g] : (half_t)0.0f;
    }
}

__global__ __launch_bounds__(256) void pack_zeros_kernel(const uint8_t *__restrict__ z4c, int n4,
                                                         int n4p, int ng, int ngp,
                                                         uint8_t *__restrict__ z4)
{
    const size_t total = (size_t)n4p * (ngp / 2);
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
        const int r = (int)(o / (ngp / 2)), g = 2 * (int)(o % (ngp / 2));
        uint32_t lo = 0, hi = 0;
        if (r < n4) {
            if (g < ng) lo = z4c[(size_t)r * ng + g] & 15;
            if (g + 1 < ng) hi = z4c[(size_t)r * ng + g + 1] & 15;
        }
        z4[o] = (uint8_t)(lo | (hi << 4));
    }
}

static inline int grid_for(size_t total)
{
    size_t b = (total + 255) / 256;
    return (int)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

int launch_pack_weights(const mixllm_desc &d, const int8_t *q8, const void *s8c, const uint8_t *q4,
                        const void *s4c, const uint8_t *z4c, void *w8, void *w4, void *s8, void *s4,
                        void *z4, hipStream_t st)
{
    const int n4 = d.N - d.n8, n8p = round_up(d.n8, TILE_N), n4p = round_up(n4, TILE_N);
    const int ng = d.K / G, ngp = round_up(ng, 8);
    if (n4p) {
        hipLaunchKernelGGL(pack_w4_kernel, dim3(grid_for((size_t)n4p * d.K / 8)), dim3(256), 0, st, q4,
                           n4, n4p, d.K, ng, (uint32_t *)w4);
        hipLaunchKernelGGL(pack_scales_kernel, dim3(grid_for((size_t)n4p * ngp)), dim3(256), 0, st,
                           (const half_t *)s4c, n4, n4p, ng, ngp, (half_t *)s4);
        hipLaunchKernelGGL(pack_zeros_kernel, dim3(grid_for((size_t)n4p * ngp / 2)), dim3(256), 0, st,
                           z4c, n4, n4p, ng, ngp, (uint8_t *)z4);
    }
    if (n8p) {
        hipLaunchKernelGGL(pack_w8_kernel, dim3(grid_for((size_t)n8p * d.K / 16)), dim3(256), 0, st, q8,
                           d.n8, n8p, d.K, (uint4 *)w8);
        const int ncan = d.w8_group == d.K ? 1 : ng, nstride = d.w8_group == d.K ? 1 : ngp;
        hipLaunchKernelGGL(pack_scales_kernel, dim3(grid_for((size_t)n8p * nstride)), dim3(256), 0, st,
                           (const half_t *)s8c, d.n8, n8p, ncan, nstride, (half_t *)s8);
    }
    return (int)hipGetLastError();
}

// ------------------------------------------------------------ packed -> canonical --

__global__ __launch_bounds__(256) void unpack_w4_kernel(const uint32_t *__restrict__ w4, int n4, int K,
                                                        int ng, uint8_t *__restrict__ q4)
{
    const size_t total = (size_t)n4 * K / 8;   // one packed dword (8 codes) per thread
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int r = (int)(i / (K / 8));
        const int k0 = (int)(i % (K / 8)) * 8;           // canonical k of the first code
        const int g = k0 / G, kl = k0 % G;
        const int half = kl / 64, ks = (kl % 64) / 16, d = (kl % 16) / 8;
        const uint32_t w = *(const uint32_t *)((const uint8_t *)w4 + w4_slot_offset(r, g, ks, ng) +
                                               half * 8 + d * 4);
        uint8_t *dst = q4 + (size_t)r * K + k0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            dst[b] = (uint8_t)((w >> (8 * b)) & 15);
            dst[b + 4] = (uint8_t)((w >> (8 * b + 4)) & 15);
        }
    }
}

__global__ __launch_bounds__(256) void unpack_w8_kernel(const uint4 *__restrict__ w8, int n8, int K,
                                                        int8_t *__restrict__ q8)
{
    const int nsteps = K / 64;
    const size_t total = (size_t)n8 * K / 16;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int r = (int)(i / (K / 16)), c = (int)(i % (K / 16));
        *(uint4 *)(q8 + (size_t)r * K + c * 16) =
            *(const uint4 *)((const uint8_t *)w8 + w8_slot_offset(r, c >> 2, c & 3, nsteps));
    }
}

__global__ __launch_bounds__(256) void unpack_scales_kernel(const half_t *__restrict__ src, int rows,
                                                            int ncan, int nstride,
                                                            half_t *__restrict__ dst)
{
    const size_t total = (size_t)rows * ncan;
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256)
        dst[o] = src[(o / ncan) * nstride + (o % ncan)];
}

__global__ __launch_bounds__(256) void unpack_zeros_kernel(const uint8_t *__restrict__ z4, int n4, int ng,
                                                           int ngp, uint8_t *__restrict__ z4c)
{
    const size_t total = (size_t)n4 * ng;
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
        const int r = (int)(o / ng), g = (int)(o % ng);
        const uint8_t b = z4[(size_t)r * (ngp / 2) + (g >> 1)];
        z4c[o] = (g & 1) ? (b >> 4) : (b & 15);
    }
}

int launch_unpack_weights(const mixllm_desc &d, const void *w8, const void *w4, const void *s8,
                          const void *s4, const void *z4, int8_t *q8, void *s8c, uint8_t *q4,
                          void *s4c, uint8_t *z4c, hipStream_t st)
{
    const int n4 = d.N - d.n8;
    const int ng = d.K / G, ngp = round_up(ng, 8);
    if (n4) {
        hipLaunchKernelGGL(unpack_w4_kernel, dim3(grid_for((size_t)n4 * d.K / 8)), dim3(256), 0, st,
                           (const uint32_t *)w4, n4, d.K, ng, q4);
        hipLaunchKernelGGL(unpack_scales_kernel, dim3(grid_for((size_t)n4 * ng)), dim3(256), 0, st,
                           (const half_t *)s4, n4, ng, ngp, (half_t *)s4c);
        hipLaunchKernelGGL(unpack_zeros_kernel, dim3(grid_for((size_t)n4 * ng)), dim3(256), 0, st,
                           (const uint8_t *)z4, n4, ng, ngp, z4c);
    }
    if (d.n8) {
        hipLaunchKernelGGL(unpack_w8_kernel, dim3(grid_for((size_t)d.n8 * d.K / 16)), dim3(256), 0, st,
                           (const uint4 *)w8, d.n8, d.K, q8);
        const int ncan = d.w8_group == d.K ? 1 : ng, nstride = d.w8_group == d.K ? 1 : ngp;
        hipLaunchKernelGGL(unpack_scales_kernel, dim3(grid_for((size_t)d.n8 * ncan)), dim3(256), 0, st,
                           (const half_t *)s8, d.n8, ncan, nstride, (half_t *)s8c);
    }
    return (int)hipGetLastError();
}

}  // namespace mixllm
