// Activation quantizer: fp16 -> int8 symmetric, one scale per token or per (token, group).
// Sec. 2 quantizer formula with z = 0; 8-bit symmetric activations, Sec. 3.1.2.
// HBM-streaming kernel: 2 B read + 1 B written per element.
#include "internal.h"

namespace mixllm {

typedef half_t h8 __attribute__((ext_vector_type(8)));

static __device__ inline float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

static __device__ inline uint2 quant8(const h8 &v, float s)
{
    const float r = recip(s);
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        w[i >> 2] |= quant_code(v[i], s, r) << (8 * (i & 3));
    }
    return make_uint2(w[0], w[1]);
}

// Exhaustive check of quotient(): for every positive finite fp16 scale (one block each) and every
// finite fp16 value the int8 code from quotient() against the code from the IEEE division.
__global__ __launch_bounds__(256) void check_fast_division_kernel(unsigned long long *mismatches)
{
    const uint16_t sb = (uint16_t)(blockIdx.x + 1);   // 0x0001 .. 0x7BFF
    const float s = (float)__builtin_bit_cast(half_t, sb);
    const float r = recip(s);
    unsigned long long bad = 0;
    for (int xb = threadIdx.x; xb < 65536; xb += 256) {
        if ((xb & 0x7C00) == 0x7C00) continue;   // infinities and NaNs
        const half_t x = __builtin_bit_cast(half_t, (uint16_t)xb);
        bad += quant_code(x, s, r) != quant_code_ieee(x, s);
        // the 4-bit weight quantizer rounds the same quotient without the int8 clamp
        bad += __builtin_rintf(quotient((float)x, s, r)) != __builtin_rintf((float)x / s);
    }
    if (bad) atomicAdd(mismatches, bad);
}

// One block per token, the row held in registers between the absmax pass and the quantizing
// pass (up to NV vectors of 8 per thread: K <= 2048 * NV): one trip to memory instead of two,
// which is most of the duration of this kernel when M is small.
template <int NV>
__global__ __launch_bounds__(256) void act_quant_per_token_regs(const half_t *__restrict__ x,
                                                                int8_t *__restrict__ xq,
                                                                half_t *__restrict__ xs, int K)
{
    __shared__ float red[4];
    const int m = blockIdx.x;
    const h8 *row = (const h8 *)(x + (size_t)m * K);
    const int nvec = K / 8;
    h8 d[NV];
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int v = threadIdx.x + 256 * j;
        if (v < nvec) {
            d[j] = row[v];
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)d[j][i]));
        }
    }
    amax = wave_max(amax);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    half_t s16 = store_scale(amax / 127.0f);
    float s = (float)s16;
    if (threadIdx.x == 0) xs[m] = s16;
    uint2 *out = (uint2 *)(xq + (size_t)m * K);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int v = threadIdx.x + 256 * j;
        if (v < nvec) out[v] = quant8(d[j], s);
    }
}

// One block per token, any K; the row is read twice (the second read hits L2).
__global__ __launch_bounds__(256) void act_quant_per_token(const half_t *__restrict__ x,
                                                           int8_t *__restrict__ xq,
                                                           half_t *__restrict__ xs, int K)
{
    __shared__ float red[4];
    const int m = blockIdx.x;
    const h8 *row = (const h8 *)(x + (size_t)m * K);
    const int nvec = K / 8;
    float amax = 0.0f;
    for (int v = threadIdx.x; v < nvec; v += 256) {
        h8 d = row[v];
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)d[i]));
    }
    amax = wave_max(amax);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    half_t s16 = store_scale(amax / 127.0f);
    float s = (float)s16;
    if (threadIdx.x == 0) xs[m] = s16;
    uint2 *out = (uint2 *)(xq + (size_t)m * K);
    for (int v = threadIdx.x; v < nvec; v += 256) out[v] = quant8(row[v], s);
}

// 16 lanes per quantization group of 128; a block covers 16 groups of one token.
__global__ __launch_bounds__(256) void act_quant_per_group(const half_t *__restrict__ x,
                                                           int8_t *__restrict__ xq,
                                                           half_t *__restrict__ xs, int K, int ng)
{
    const int m = blockIdx.x;
    const int g = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (g >= ng) return;   // whole 16-lane groups leave together; no block barrier below
    const size_t off = (size_t)m * K + (size_t)g * G + (threadIdx.x & 15) * 8;
    h8 d = *(const h8 *)(x + off);
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)d[i]));
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 16));
    half_t s16 = store_scale(amax / 127.0f);
    if ((threadIdx.x & 15) == 0) xs[(size_t)m * ng + g] = s16;
    *(uint2 *)(xq + off) = quant8(d, (float)s16);
}

int launch_check_fast_division(unsigned long long *mismatches, hipStream_t st)
{
    hipLaunchKernelGGL(check_fast_division_kernel, dim3(0x7BFF), dim3(256), 0, st, mismatches);
    return (int)hipGetLastError();
}

int launch_quantize_activations(const mixllm_desc &d, const void *x, int8_t *xq, void *xs,
                                hipStream_t st)
{
    if (d.M == 0) return hipSuccess;
    if (d.act_group == d.K) {
        if (d.K <= 2048 * 2)
            hipLaunchKernelGGL(act_quant_per_token_regs<2>, dim3(d.M), dim3(256), 0, st, (const half_t *)x, xq,
                               (half_t *)xs, d.K);
        else if (d.K <= 2048 * 8)
            hipLaunchKernelGGL(act_quant_per_token_regs<8>, dim3(d.M), dim3(256), 0, st, (const half_t *)x, xq,
                               (half_t *)xs, d.K);
        else
            hipLaunchKernelGGL(act_quant_per_token, dim3(d.M), dim3(256), 0, st, (const half_t *)x, xq,
                               (half_t *)xs, d.K);
    } else {
        const int ng = d.K / G;
        hipLaunchKernelGGL(act_quant_per_group, dim3(d.M, (ng + 15) / 16), dim3(256), 0, st,
                           (const half_t *)x, xq, (half_t *)xs, d.K, ng);
    }
    return (int)hipGetLastError();
}

}  // namespace mixllm
