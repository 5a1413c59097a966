// Generic path of the quantized linear: one thread per output element, scalar integer dot
// products straight from the packed layouts, no MFMA, no LDS.  Covers every shape and
// variant; it exists as the simple in-library cross-check of the two fast paths and as the
// fallback for shapes they do not take.  Same definition as the fast paths:
// per-group int32 partial sum, then float rescale (Sec. 3.3), then scatter (Sec. 3.4).
#include "internal.h"

namespace mixllm {

static __device__ inline int dot4(uint32_t a, uint32_t b, int acc)
{
    // four int8 x int8 products
#pragma unroll
    for (int i = 0; i < 4; ++i)
        acc += (int)(int8_t)(a >> (8 * i)) * (int)(int8_t)(b >> (8 * i));
    return acc;
}

// DUMP: 0 = the linear, 1 = the per-group partial sums, 2 = their integer sums over the groups
template <int DUMP>
__global__ __launch_bounds__(256) void linear_generic_kernel(LinearParams p)
{
    const int j = blockIdx.x * 256 + threadIdx.x;   // row of the concatenation [8-bit ; 4-bit]
    const int m = blockIdx.y;
    if (j >= p.N) return;
    const int c = p.perm[j];
    const int8_t *xrow = p.xq + (size_t)m * p.K;
    const int nsteps = p.K / 64;
    float acc = 0.0f;
    int isum = 0;
    for (int g = 0; g < p.ng; ++g) {
        int P = 0;
        float sw = 0.0f;
        if (j < p.n8) {
            const int r = j;
#pragma unroll
            for (int half = 0; half < 2; ++half)
                for (int ks = 0; ks < 4; ++ks) {
                    const uint4 w = *(const uint4 *)((const uint8_t *)p.w8 +
                                                     w8_slot_offset(r, 2 * g + half, ks, nsteps));
                    const uint4 a = *(const uint4 *)(xrow + g * G + half * 64 + ks * 16);
                    P = dot4(a.x, w.x, P);
                    P = dot4(a.y, w.y, P);
                    P = dot4(a.z, w.z, P);
                    P = dot4(a.w, w.w, P);
                }
            if (DUMP == 0) sw = (float)(p.w8_per_channel ? p.s8[r] : p.s8[(size_t)r * p.ngp + g]);
        } else {
            const int r = j - p.n8;
            const uint32_t zb = zbias(z4_load(p.z4, r, g, p.ngp));
            for (int ks = 0; ks < 4; ++ks) {
                const uint4 w = *(const uint4 *)(p.w4 + w4_slot_offset(r, g, ks, p.ng));
                const uint32_t wd[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const uint4 a = *(const uint4 *)(xrow + g * G + half * 64 + ks * 16);
                    int b0, b1, b2, b3;
                    unpack_sub(wd[2 * half], zb, b0, b1);       // k-local 0..3, 4..7
                    unpack_sub(wd[2 * half + 1], zb, b2, b3);   // k-local 8..11, 12..15
                    P = dot4(a.x, (uint32_t)b0, P);
                    P = dot4(a.y, (uint32_t)b1, P);
                    P = dot4(a.z, (uint32_t)b2, P);
                    P = dot4(a.w, (uint32_t)b3, P);
                }
            }
            if (DUMP == 0) sw = (float)p.s4[(size_t)r * p.ngp + g];
        }
        if (DUMP == 1) {
            p.P[((size_t)m * p.N + c) * p.ng + g] = P;
        } else if (DUMP == 2) {
            isum += P;
        } else {
            const float sa = (float)(p.act_per_token ? p.xscale[m] : p.xscale[(size_t)m * p.ng + g]);
            acc += (float)P * sw * sa;
        }
    }
    if (DUMP == 2) p.S[(size_t)m * p.N + c] = isum;
    if (!DUMP) p.y[(size_t)m * p.N + c] = (half_t)acc;
}

int launch_linear_generic(const LinearParams &p, hipStream_t st)
{
    if (p.M == 0 || p.N == 0) return hipSuccess;
    dim3 grid((p.N + 255) / 256, p.M);
    if (p.P)
        hipLaunchKernelGGL(linear_generic_kernel<1>, grid, dim3(256), 0, st, p);
    else if (p.S)
        hipLaunchKernelGGL(linear_generic_kernel<2>, grid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(linear_generic_kernel<0>, grid, dim3(256), 0, st, p);
    return (int)hipGetLastError();
}

}  // namespace mixllm
