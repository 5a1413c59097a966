// Global precision search (Sec. 3.2): the salience of every output channel of a layer
// (Eq. 4) and the choice of the T most salient channels over all layers (Alg. 1).
// Offline, off the timed path of the linear; the salience kernel is a plain streaming
// reduction over W and G (4 bytes per weight), the selection a radix select over the
// saliences' bit patterns followed by an ordered compaction per layer.
#include <algorithm>

#include "internal.h"

namespace mixllm {

namespace {

typedef half_t h8 __attribute__((ext_vector_type(8)));

// ---- channel salience -------------------------------------------------------------------
// One block of 4 waves per output channel.  A wave-wide 16-byte load covers 4 quantization
// groups (16 lanes x 8 values each); the group's range, scale and zero point are found inside
// the 16-lane segment exactly as the weight quantizer finds them, so the codes are the ones
// mixllm_quantize_weights would store for this row as a 4-bit row.
__global__ __launch_bounds__(256) void channel_salience_kernel(const half_t *__restrict__ W, const half_t *__restrict__ Gr,
                                                               int K, float weight, int accumulate,
                                                               float *__restrict__ salience)
{
    __shared__ float part[4];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const half_t *w_row = W + (size_t)n * K, *g_row = Gr + (size_t)n * K;
    float acc = 0.0f;
    // 512 values per wave and iteration, 2048 per block
    for (int k0 = wave * 512 + lane * 8; k0 < K; k0 += 2048) {
        const h8 w = *(const h8 *)(w_row + k0);
        const h8 g = *(const h8 *)(g_row + k0);
        float mn = 0.0f, mx = 0.0f;   // the range always contains 0
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            mn = fminf(mn, (float)w[i]);
            mx = fmaxf(mx, (float)w[i]);
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, o, 16));
            mx = fmaxf(mx, __shfl_xor(mx, o, 16));
        }
        const float sc = (float)store_scale((mx - mn) / 15.0f);
        const float rsc = recip(sc);
        const float zf = fminf(fmaxf(__builtin_rintf(quotient(-mn, sc, rsc)), 0.0f), 15.0f);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float wf = (float)w[i];
            const float code = fminf(fmaxf(__builtin_rintf(quotient(wf, sc, rsc)) + zf, 0.0f), 15.0f);
            const float delta = (code - zf) * sc - wf;   // quantize(W) - W
            acc = __builtin_fmaf((float)g[i], delta, acc);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (tid == 0) {
        const float s1 = (part[0] + part[1]) + (part[2] + part[3]);
        const float s = fabsf(s1 + 0.5f * s1 * s1);
        salience[n] = (accumulate ? salience[n] : 0.0f) + weight * s;
    }
}

// ---- global selection -------------------------------------------------------------------
// Saliences are non-negative floats, so their bit patterns order like the values.  Four
// passes of 256-bin histograms (most significant byte first) find the bit pattern of the
// T-th largest salience and how many channels with exactly that value still belong to the
// chosen set; equal values are taken in the order of the concatenation (earlier layer, then
// lower channel).

struct SelectState {
    uint32_t prefix;      // bytes of the threshold found so far
    uint32_t remaining;   // rank still to be found inside the current prefix; after the last pass:
                          // number of channels equal to the threshold that are chosen
    uint32_t hist[256];
};

__global__ void select_init_kernel(SelectState *st, uint32_t T)
{
    const int t = threadIdx.x;
    if (t < 256) st->hist[t] = 0;
    if (t == 0) {
        st->prefix = 0;
        st->remaining = T;
    }
}

// histogram of byte `pass` over the keys whose higher bytes equal the prefix
__global__ __launch_bounds__(256) void select_hist_kernel(const uint32_t *__restrict__ keys, int64_t total, int pass, SelectState *st)
{
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t prefix = st->prefix;
    const int hi_shift = 8 * (pass + 1);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const uint32_t k = keys[i];
        const bool match = pass == 3 || (k >> hi_shift) == (prefix >> hi_shift);
        if (match) atomicAdd(&h[(k >> (8 * pass)) & 255u], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&st->hist[threadIdx.x], h[threadIdx.x]);
}

// walk the bins from the largest byte value down to the one that holds the wanted rank
__global__ void select_pick_kernel(SelectState *st, int pass)
{
    if (threadIdx.x == 0) {
        uint32_t remaining = st->remaining;
        int d = 255;
        if (remaining > 0) {
            while (d > 0 && st->hist[d] < remaining) {
                remaining -= st->hist[d];
                --d;
            }
            st->prefix |= (uint32_t)d << (8 * pass);
            st->remaining = remaining;
        } else {
            st->prefix = 0xFFFFFFFFu;   // T = 0: nothing reaches the threshold
        }
    }
    __syncthreads();
    if (threadIdx.x < 256) st->hist[threadIdx.x] = 0;
}

// per layer: channels above the threshold, channels equal to it
__global__ __launch_bounds__(256) void select_count_kernel(const uint32_t *__restrict__ keys, const int64_t *__restrict__ offsets,
                                                           const SelectState *st, uint32_t *gt, uint32_t *eq)
{
    __shared__ uint32_t s_gt, s_eq;
    if (threadIdx.x == 0) s_gt = s_eq = 0;
    __syncthreads();
    const int l = blockIdx.x;
    const uint32_t thr = st->prefix;
    uint32_t a = 0, b = 0;
    for (int64_t i = offsets[l] + threadIdx.x; i < offsets[l + 1]; i += 256) {
        const uint32_t k = keys[i];
        a += k > thr;
        b += k == thr;
    }
    atomicAdd(&s_gt, a);
    atomicAdd(&s_eq, b);
    __syncthreads();
    if (threadIdx.x == 0) {
        gt[l] = s_gt;
        eq[l] = s_eq;
    }
}

// in layer order: how many of a layer's threshold-valued channels are chosen, where its list starts
__global__ void select_scan_kernel(const SelectState *st, int L, const uint32_t *gt, const uint32_t *eq, uint32_t *eq_take,
                                   uint32_t *out_off, int32_t *layer_counts)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    uint32_t left = st->prefix == 0xFFFFFFFFu ? 0u : st->remaining, run = 0;
    for (int l = 0; l < L; ++l) {
        const uint32_t take = eq[l] < left ? eq[l] : left;
        left -= take;
        eq_take[l] = take;
        out_off[l] = run;
        layer_counts[l] = (int32_t)(gt[l] + take);
        run += gt[l] + take;
    }
}

// exclusive prefix sum of one value per thread over the block of 256 (wave scans, then the 4 wave totals)
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t &block_total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();   // wave_tot may still be read from the previous call
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
    for (int w = 0; w < wave; ++w) base += wave_tot[w];
    block_total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    return base + inc - v;
}

// one block per layer walks its channels in order and writes the chosen indices, ascending
__global__ __launch_bounds__(256) void select_emit_kernel(const uint32_t *__restrict__ keys, const int64_t *__restrict__ offsets,
                                                          const SelectState *st, const uint32_t *eq_take, const uint32_t *out_off,
                                                          int32_t *selected)
{
    __shared__ uint32_t wave_tot[4];
    const int l = blockIdx.x;
    const uint32_t thr = st->prefix, take = eq_take[l];
    const int64_t lo = offsets[l], n = offsets[l + 1] - lo;
    uint32_t eq_seen = 0, written = 0;
    for (int64_t c0 = 0; c0 < n; c0 += 256) {
        const int64_t c = c0 + threadIdx.x;
        const uint32_t k = c < n ? keys[lo + c] : 0u;
        const uint32_t is_eq = (c < n && k == thr) ? 1u : 0u;
        uint32_t eq_total, sel_total;
        const uint32_t eq_rank = eq_seen + block_exclusive_scan(is_eq, wave_tot, eq_total);
        const uint32_t sel = (c < n && (k > thr || (is_eq && eq_rank < take))) ? 1u : 0u;
        const uint32_t pos = written + block_exclusive_scan(sel, wave_tot, sel_total);
        if (sel) selected[out_off[l] + pos] = (int32_t)c;
        eq_seen += eq_total;
        written += sel_total;
    }
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The layer offsets come from a host array that may be gone when the call returns, and the call
// must neither block nor stage a copy: they travel as kernel arguments, 128 at a time.
struct OffsetChunk {
    int64_t v[128];
};
__global__ void select_offsets_kernel(int64_t *dst, int n, OffsetChunk c)
{
    const int t = threadIdx.x;
    if (t < n) dst[t] = c.v[t];
}

}  // namespace

int launch_channel_salience(const void *W, const void *Gr, int N, int K, float weight, int accumulate, float *salience,
                            hipStream_t st)
{
    if (N == 0) return (int)hipSuccess;
    hipLaunchKernelGGL(channel_salience_kernel, dim3(N), dim3(256), 0, st, (const half_t *)W, (const half_t *)Gr, K, weight,
                       accumulate, salience);
    return (int)hipGetLastError();
}

size_t select_salient_workspace_bytes(int L)
{
    return align_up(sizeof(SelectState), 256) + align_up(sizeof(int64_t) * (size_t)(L + 1), 256) +
           4 * align_up(sizeof(uint32_t) * (size_t)L, 256);
}

int launch_select_salient(const float *salience, const int64_t *layer_offsets_host, int L, int64_t T, int32_t *selected,
                          int32_t *layer_counts, void *workspace, hipStream_t st)
{
    uint8_t *ws = (uint8_t *)workspace;
    SelectState *state = (SelectState *)ws;
    ws += align_up(sizeof(SelectState), 256);
    int64_t *offsets = (int64_t *)ws;
    ws += align_up(sizeof(int64_t) * (size_t)(L + 1), 256);
    const size_t per = align_up(sizeof(uint32_t) * (size_t)L, 256);
    uint32_t *gt = (uint32_t *)ws, *eq = (uint32_t *)(ws + per), *eq_take = (uint32_t *)(ws + 2 * per),
             *out_off = (uint32_t *)(ws + 3 * per);
    const int64_t total = layer_offsets_host[L];
    for (int o = 0; o <= L; o += 128) {
        OffsetChunk c;
        const int n = std::min(128, L + 1 - o);
        for (int i = 0; i < 128; ++i) c.v[i] = i < n ? layer_offsets_host[o + i] : 0;
        hipLaunchKernelGGL(select_offsets_kernel, dim3(1), dim3(128), 0, st, offsets + o, n, c);
    }
    const uint32_t *keys = (const uint32_t *)salience;
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(256), 0, st, state, (uint32_t)T);
    const int blocks = (int)std::min<int64_t>(2048, (total + 255) / 256);
    for (int pass = 3; pass >= 0; --pass) {
        if (blocks > 0) hipLaunchKernelGGL(select_hist_kernel, dim3(blocks), dim3(256), 0, st, keys, total, pass, state);
        hipLaunchKernelGGL(select_pick_kernel, dim3(1), dim3(256), 0, st, state, pass);
    }
    hipLaunchKernelGGL(select_count_kernel, dim3(L), dim3(256), 0, st, keys, offsets, state, gt, eq);
    hipLaunchKernelGGL(select_scan_kernel, dim3(1), dim3(64), 0, st, state, L, gt, eq, eq_take, out_off, layer_counts);
    hipLaunchKernelGGL(select_emit_kernel, dim3(L), dim3(256), 0, st, keys, offsets, state, eq_take, out_off, selected);
    return (int)hipGetLastError();
}

}  // namespace mixllm
