// C ABI of libmixllm_hip.so: argument validation (host only, before anything is launched),
// size accounting, feature permutation, and dispatch to the kernel launchers.
#include <cstdlib>
#include <mutex>
#include <vector>

#include "internal.h"

using namespace mixllm;

// Scratch of mixllm_mixed_linear_fp16_static (xq, then xscale): one array per GPU, held by the
// loaded code object until the process ends.  In host code the name is only a handle: the device
// address comes from hipGetSymbolAddress, per device (static_scratch_ptr below).
static __device__ __align__(256) uint8_t scratch[MIXLLM_STATIC_SCRATCH_BYTES];

namespace {

inline size_t round_up_sz(size_t a, size_t b) { return (a + b - 1) / b * b; }

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// A buffer argument: must be non-null and 16-byte aligned when its size is non-zero.
inline bool buf_ok(const void *p, size_t bytes) { return bytes == 0 || (p != nullptr && aligned16(p)); }

int check_desc(const mixllm_desc *d)
{
    if (!d) return MIXLLM_EINVAL;
    if (d->M < 0 || d->K <= 0 || d->N <= 0 || d->n8 < 0 || d->n8 > d->N) return MIXLLM_EINVAL;
    if (d->group != G || d->K % G != 0) return MIXLLM_EUNSUPPORTED;
    if (d->act_group != d->K && d->act_group != G) return MIXLLM_EUNSUPPORTED;
    if (d->w8_group != d->K && d->w8_group != G) return MIXLLM_EUNSUPPORTED;
    // K: an 8-bit channel with one scale keeps ONE int32 sum over all of K (K * 127 * 127 < 2^31)
    if (d->K > MIXLLM_MAX_K || d->N > (1 << 24) || d->M > (1 << 24)) return MIXLLM_EUNSUPPORTED;
    return MIXLLM_OK;
}

void sizes_of(const mixllm_desc &d, mixllm_sizes &s)
{
    const size_t n4 = (size_t)(d.N - d.n8);
    const size_t n8p = (size_t)round_up(d.n8, TILE_N), n4p = (size_t)round_up((int)n4, TILE_N);
    const size_t ng = (size_t)d.K / G, ngp = (size_t)round_up((int)ng, 8);
    s.w8_bytes = n8p * (size_t)d.K;
    s.w4_bytes = n4p * (size_t)d.K / 2;
    s.scales8_bytes = (d.w8_group == d.K ? n8p : n8p * ngp) * 2;
    s.scales4_bytes = n4p * ngp * 2;
    s.zeros4_bytes = n4p * ngp / 2;
    s.perm_bytes = (size_t)d.N * 4;
    s.xq_bytes = (size_t)d.M * (size_t)d.K;
    s.xscale_bytes = (size_t)d.M * (size_t)(d.K / d.act_group) * 2;
    s.y_bytes = (size_t)d.M * (size_t)d.N * 2;
    s.linear_workspace_bytes = 0;   // filled in by sizes_with_scratch (needs the launch parameters)
    // scratch of mixllm_mixed_linear_fp16 when it cannot quantize inside the linear kernel: xq, then xscale
    s.workspace_bytes = (size_t)round_up_sz(s.xq_bytes, 256) + (size_t)round_up_sz(s.xscale_bytes, 256);
}

LinearParams make_params(const mixllm_desc &d, const int8_t *xq, const void *xscale, const void *w4,
                         const void *w8, const void *s4, const void *s8, const void *z4,
                         const int32_t *perm)
{
    LinearParams p{};
    p.M = d.M;
    p.K = d.K;
    p.N = d.N;
    p.n8 = d.n8;
    p.n4 = d.N - d.n8;
    p.ng = d.K / G;
    p.ngp = round_up(p.ng, 8);
    p.ntiles8 = round_up(p.n8, TILE_N) / TILE_N;
    p.ntiles4 = round_up(p.n4, TILE_N) / TILE_N;
    p.act_per_token = d.act_group == d.K ? 1 : 0;
    p.w8_per_channel = d.w8_group == d.K ? 1 : 0;
    p.xq = xq;
    p.xscale = (const half_t *)xscale;
    p.w4 = (const uint8_t *)w4;
    p.w8 = (const int8_t *)w8;
    p.s4 = (const half_t *)s4;
    p.s8 = (const half_t *)s8;
    p.z4 = (const uint8_t *)z4;
    p.perm = perm;
    p.variant = DECODE_ANY;
    p.prefill_tm = 0;
    p.kparts = 1;
    p.quads_per_part = (p.ng + 3) / 4;
    p.np = (p.ntiles8 + p.ntiles4) * TILE_N;
    p.partials = nullptr;
    p.partials_cap = 0;
    return p;
}

// scratch the linear would like for this shape: only the tiled kernel uses any (K split over blocks)
size_t linear_scratch_bytes(const mixllm_desc &d)
{
    if (d.M <= 16) return 0;
    LinearParams p = make_params(d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    return prefill_scratch_bytes(p);   // (what the tiled kernel would use if the call reaches it)
}

// sizes_of plus the scratch of the linear; workspace_bytes = xq, xscale, then that scratch
void sizes_with_scratch(const mixllm_desc &d, mixllm_sizes &s)
{
    sizes_of(d, s);
    s.linear_workspace_bytes = linear_scratch_bytes(d);
    s.workspace_bytes += s.linear_workspace_bytes;
}

}  // namespace

namespace mixllm {
int cu_count()
{
    static int n[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (n[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        n[dev] = v;
    }
    return n[dev];
}

int ensure_dynamic_lds(const void *kernel, size_t bytes)
{
    // (kernel, device) pairs already configured with at least this size; a few dozen instantiations exist
    struct Done {
        const void *fn;
        int dev;
        size_t bytes;
    };
    static Done done[256];
    static int ndone = 0;
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < ndone; ++i)
        if (done[i].fn == kernel && done[i].dev == dev) {
            if (done[i].bytes >= bytes) return (int)hipSuccess;
            hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e == hipSuccess) done[i].bytes = bytes;
            return (int)e;
        }
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return (int)e;
    if (ndone < 256) done[ndone++] = Done{kernel, dev, bytes};
    return (int)hipSuccess;
}
}  // namespace mixllm

namespace {

int hip_status(int e) { return e == (int)hipSuccess ? MIXLLM_OK : MIXLLM_EHIP; }

// The library's choice of kernel.  Up to 16 tokens the decode path.  17 to 64 tokens lie between the
// two paths the workload names.  Measured with every launch reading its weights from HBM (copies of
// the layer rotating over 512 MB, as in a step of a model), on the Llama-shaped layers:
//  * up to 32 tokens the weight-streaming kernel for a few dozen tokens (K = N = 4096: 11 against
//    14 us for the tiled kernel), except on layers with a long K when the caller brings the
//    scratch that lets the tiled kernel split K over blocks (K = 14336, N = 4096: 20 against 27 us),
//    and on layers so wide that blocks of 32 x 128 fill the chip (K = 4096, N = 28672: 17 against
//    18 us; K = 8192, N = 57344: 53-57 against 59-62 us);
//  * from 33 tokens the tiled kernel with its small block shapes (K = N = 4096 at 64 tokens: 14.5
//    against 15.4 us; K = 4096, N = 28672: 21 against 25 us; K = 8192, N = 57344: 67 against 81 us),
//    except where its K loop is long, cannot be split for want of scratch, and the grid of 64 x 128
//    tiles leaves CUs empty (K = 14336, N = 4096: 37 us for the streaming kernel, 50 us tiled).
int auto_path(const mixllm_desc &d, const LinearParams &p)
{
    if (d.M <= 16) return MIXLLM_PATH_DECODE;
    if (d.M > 64 || !mid_covers(p)) return MIXLLM_PATH_PREFILL;
    const bool split = prefill_would_split(p);
    const long tiles = (long)(p.ntiles8 * TILE_N + 127) / 128 + (p.ntiles4 * TILE_N + 127) / 128;
    const bool wide = 4 * tiles >= 3L * cu_count();   // column tiles of 128 channels for three quarters of the CUs or more
    if (d.M <= 32) return ((split && p.ng > 64) || wide) ? MIXLLM_PATH_PREFILL : MIXLLM_PATH_MID;
    return (p.ng < 64 || split || wide) ? MIXLLM_PATH_PREFILL : MIXLLM_PATH_MID;
}

// Which kernel a call takes: the caller's path argument with AUTO resolved, or a negative status
// when that path does not cover the shape.  Host arithmetic only; nothing is launched, so that a
// call can refuse before it has enqueued anything.  `q` receives the parameters the launch uses.
int resolve_path(const mixllm_desc &d, const LinearParams &p, int path, LinearParams &q)
{
    q = p;
    if (path == MIXLLM_PATH_AUTO) path = auto_path(d, p);
    const bool sums = p.S != nullptr;   // the sums over the groups come from the generic and the tiled kernel only
    switch (path) {
    case MIXLLM_PATH_GENERIC:
        return d.M > 65535 ? MIXLLM_EUNSUPPORTED : path;
    case MIXLLM_PATH_DECODE:
        return (d.M > 16 || sums) ? MIXLLM_EUNSUPPORTED : path;
    case MIXLLM_PATH_DECODE_STREAM:
    case MIXLLM_PATH_DECODE_RESIDENT:
    case MIXLLM_PATH_DECODE_SPLIT:
        if (d.M > 16 || sums) return MIXLLM_EUNSUPPORTED;
        q.variant = path == MIXLLM_PATH_DECODE_STREAM ? DECODE_STREAM : path == MIXLLM_PATH_DECODE_RESIDENT ? DECODE_RESIDENT : DECODE_SPLIT;
        if (path == MIXLLM_PATH_DECODE_SPLIT && !decode_split_covers(q)) return MIXLLM_EUNSUPPORTED;
        return path;
    case MIXLLM_PATH_MID:
        return (!mid_covers(p) || sums) ? MIXLLM_EUNSUPPORTED : path;
    case MIXLLM_PATH_PREFILL:
    case MIXLLM_PATH_PREFILL_32:
    case MIXLLM_PATH_PREFILL_64:
    case MIXLLM_PATH_PREFILL_128:
        q.prefill_tm = path == MIXLLM_PATH_PREFILL_32 ? 1 : path == MIXLLM_PATH_PREFILL_64 ? 2 : path == MIXLLM_PATH_PREFILL_128 ? 4 : 0;
        return prefill_covers(q) ? MIXLLM_PATH_PREFILL : MIXLLM_EUNSUPPORTED;
    default:
        return MIXLLM_EINVAL;
    }
}

int run_path(const LinearParams &q, int path, hipStream_t st)
{
    switch (path) {
    case MIXLLM_PATH_GENERIC: return hip_status(launch_linear_generic(q, st));
    case MIXLLM_PATH_MID: return hip_status(launch_linear_mid(q, st));
    case MIXLLM_PATH_PREFILL: return hip_status(launch_linear_prefill(q, st));
    default: return hip_status(launch_linear_decode(q, st));   // MIXLLM_PATH_DECODE and its variants
    }
}

int dispatch(const mixllm_desc &d, const LinearParams &p, int path, hipStream_t st)
{
    LinearParams q;
    const int r = resolve_path(d, p, path, q);
    return r < 0 ? r : run_path(q, r, st);
}

}  // namespace

extern "C" {

const char *mixllm_status_string(int status)
{
    switch (status) {
    case MIXLLM_OK: return "ok";
    case MIXLLM_EINVAL: return "invalid argument (null or misaligned pointer, bad size or index)";
    case MIXLLM_EUNSUPPORTED: return "unsupported shape or variant";
    case MIXLLM_EWORKSPACE: return "workspace too small";
    case MIXLLM_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int mixllm_abi_version(void) { return 2; }

int mixllm_query_sizes(const mixllm_desc *d, mixllm_sizes *out)
{
    if (!out) return MIXLLM_EINVAL;
    if (int rc = check_desc(d)) return rc;
    sizes_with_scratch(*d, *out);
    return MIXLLM_OK;
}

int mixllm_build_feature_perm(int32_t N, int32_t n8, const int32_t *salient_idx_host, int32_t *perm_host)
{
    if (N <= 0 || n8 < 0 || n8 > N || !perm_host || (n8 > 0 && !salient_idx_host)) return MIXLLM_EINVAL;
    std::vector<uint8_t> is8((size_t)N, 0);
    for (int32_t i = 0; i < n8; ++i) {
        const int32_t c = salient_idx_host[i];
        if (c < 0 || c >= N || is8[c]) return MIXLLM_EINVAL;
        is8[c] = 1;
    }
    int32_t a = 0, b = n8;
    for (int32_t c = 0; c < N; ++c) perm_host[is8[c] ? a++ : b++] = c;
    return MIXLLM_OK;
}

int mixllm_quantize_weights(const mixllm_desc *d, const void *W, const int32_t *salient_idx,
                            void *packed_w8, void *packed_w4, void *scales8, void *scales4, void *zeros4,
                            int32_t *feature_perm, void *stream)
{
    if (int rc = check_desc(d)) return rc;
    mixllm_sizes s;
    sizes_of(*d, s);
    if (!W || !aligned16(W) || !feature_perm || !aligned16(feature_perm)) return MIXLLM_EINVAL;
    if (d->n8 > 0 && (!salient_idx || ((uintptr_t)salient_idx & 3u))) return MIXLLM_EINVAL;
    if (!buf_ok(packed_w8, s.w8_bytes) || !buf_ok(packed_w4, s.w4_bytes) || !buf_ok(scales8, s.scales8_bytes) ||
        !buf_ok(scales4, s.scales4_bytes) || !buf_ok(zeros4, s.zeros4_bytes))
        return MIXLLM_EINVAL;
    // the order of the rows is built on the device, from the device list: nothing crosses to the host
    hipStream_t st = (hipStream_t)stream;
    if (int rc = hip_status(launch_build_feature_perm(d->N, d->n8, salient_idx, feature_perm, st))) return rc;
    return hip_status(launch_quantize_weights(*d, W, packed_w8, packed_w4, scales8, scales4, zeros4, feature_perm, st));
}

int mixllm_pack_weights(const mixllm_desc *d, const int8_t *q8, const void *s8, const uint8_t *q4,
                        const void *s4, const uint8_t *z4, const int32_t *perm, void *packed_w8,
                        void *packed_w4, void *scales8, void *scales4, void *zeros4, int32_t *feature_perm,
                        void *stream)
{
    if (int rc = check_desc(d)) return rc;
    mixllm_sizes s;
    sizes_of(*d, s);
    const bool has8 = d->n8 > 0, has4 = d->n8 < d->N;
    if (!perm || !feature_perm) return MIXLLM_EINVAL;
    if (has8 && (!q8 || !s8 || !aligned16(q8))) return MIXLLM_EINVAL;
    if (has4 && (!q4 || !s4 || !z4)) return MIXLLM_EINVAL;
    if (!buf_ok(packed_w8, s.w8_bytes) || !buf_ok(packed_w4, s.w4_bytes) || !buf_ok(scales8, s.scales8_bytes) ||
        !buf_ok(scales4, s.scales4_bytes) || !buf_ok(zeros4, s.zeros4_bytes))
        return MIXLLM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (perm != feature_perm &&
        hipMemcpyAsync(feature_perm, perm, s.perm_bytes, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return MIXLLM_EHIP;
    return hip_status(launch_pack_weights(*d, q8, s8, q4, s4, z4, packed_w8, packed_w4, scales8, scales4,
                                          zeros4, st));
}

int mixllm_unpack_weights(const mixllm_desc *d, const void *packed_w8, const void *packed_w4,
                          const void *scales8, const void *scales4, const void *zeros4,
                          const int32_t *feature_perm, int8_t *q8, void *s8, uint8_t *q4, void *s4,
                          uint8_t *z4, int32_t *perm, void *stream)
{
    if (int rc = check_desc(d)) return rc;
    mixllm_sizes s;
    sizes_of(*d, s);
    const bool has8 = d->n8 > 0, has4 = d->n8 < d->N;
    if (!perm || !feature_perm) return MIXLLM_EINVAL;
    if (has8 && (!q8 || !s8 || !aligned16(q8))) return MIXLLM_EINVAL;
    if (has4 && (!q4 || !s4 || !z4)) return MIXLLM_EINVAL;
    if (!buf_ok(packed_w8, s.w8_bytes) || !buf_ok(packed_w4, s.w4_bytes) || !buf_ok(scales8, s.scales8_bytes) ||
        !buf_ok(scales4, s.scales4_bytes) || !buf_ok(zeros4, s.zeros4_bytes))
        return MIXLLM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (perm != feature_perm &&
        hipMemcpyAsync(perm, feature_perm, s.perm_bytes, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return MIXLLM_EHIP;
    return hip_status(launch_unpack_weights(*d, packed_w8, packed_w4, scales8, scales4, zeros4, q8, s8, q4,
                                            s4, z4, st));
}

int mixllm_quantize_activations(const mixllm_desc *d, const void *x, int8_t *xq, void *xscale, void *stream)
{
    if (int rc = check_desc(d)) return rc;
    if (d->M == 0) return MIXLLM_OK;
    if (!x || !xq || !xscale || !aligned16(x) || !aligned16(xq) || !aligned16(xscale)) return MIXLLM_EINVAL;
    return hip_status(launch_quantize_activations(*d, x, xq, xscale, (hipStream_t)stream));
}

// Exactly one of y (the linear), P (per-group partial sums) and S (their sums over the groups) is given.
static int linear_common(const mixllm_desc *d, const int8_t *xq, const void *xscale, const void *packed_w4,
                         const void *packed_w8, const void *scales4, const void *scales8,
                         const void *zeros4, const int32_t *feature_perm, void *y, int32_t *P, int32_t *S,
                         int path, void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_desc(d)) return rc;
    if (path < MIXLLM_PATH_AUTO || path > MIXLLM_PATH_PREFILL_128) return MIXLLM_EINVAL;
    if (d->M == 0) return MIXLLM_OK;
    mixllm_sizes s;
    sizes_of(*d, s);
    if (!xq || !aligned16(xq) || !feature_perm || !aligned16(feature_perm)) return MIXLLM_EINVAL;
    if (!P && (!xscale || !aligned16(xscale))) return MIXLLM_EINVAL;
    if (!P && !S && (!y || !aligned16(y))) return MIXLLM_EINVAL;
    if ((P && !aligned16(P)) || (S && !aligned16(S))) return MIXLLM_EINVAL;
    if (!buf_ok(packed_w8, s.w8_bytes) || !buf_ok(packed_w4, s.w4_bytes) || !buf_ok(zeros4, s.zeros4_bytes))
        return MIXLLM_EINVAL;
    if (!P && (!buf_ok(scales8, s.scales8_bytes) || !buf_ok(scales4, s.scales4_bytes))) return MIXLLM_EINVAL;
    LinearParams p = make_params(*d, xq, xscale, packed_w4, packed_w8, scales4, scales8, zeros4, feature_perm);
    p.y = (half_t *)y;
    p.P = P;
    p.S = S;
    // optional scratch: the tiled kernel splits K over several blocks where the grid is small, if the
    // caller brought room for the parts' sums; without it the same kernel runs unsplit
    if (y && workspace && aligned16(workspace)) {
        p.partials = (float *)workspace;
        p.partials_cap = workspace_bytes;
    }
    return dispatch(*d, p, path, (hipStream_t)stream);
}

int mixllm_mixed_linear_path(const mixllm_desc *d, const int8_t *xq, const void *xscale,
                             const void *packed_w4, const void *packed_w8, const void *scales4,
                             const void *scales8, const void *zeros4, const int32_t *feature_perm, void *y,
                             void *workspace, size_t workspace_bytes, int path, void *stream)
{
    return linear_common(d, xq, xscale, packed_w4, packed_w8, scales4, scales8, zeros4, feature_perm, y,
                         nullptr, nullptr, path, workspace, workspace_bytes, stream);
}

int mixllm_mixed_linear(const mixllm_desc *d, const int8_t *xq, const void *xscale, const void *packed_w4,
                        const void *packed_w8, const void *scales4, const void *scales8, const void *zeros4,
                        const int32_t *feature_perm, void *y, void *workspace, size_t workspace_bytes,
                        void *stream)
{
    return mixllm_mixed_linear_path(d, xq, xscale, packed_w4, packed_w8, scales4, scales8, zeros4,
                                    feature_perm, y, workspace, workspace_bytes, MIXLLM_PATH_AUTO, stream);
}

// fp16 activations in, fp16 outputs out; `scratch` (device, 16-byte aligned, scratch_bytes long) holds xq
// and xscale between the quantizer and the linear where one kernel cannot do both.
static int linear_from_fp16(const mixllm_desc *d, const void *x, const void *packed_w4, const void *packed_w8,
                            const void *scales4, const void *scales8, const void *zeros4, const int32_t *feature_perm,
                            void *y, void *scratch, size_t scratch_bytes, hipStream_t st)
{
    if (int rc = check_desc(d)) return rc;
    if (d->M == 0) return MIXLLM_OK;
    mixllm_sizes s;
    sizes_of(*d, s);
    if (!x || !aligned16(x) || !y || !aligned16(y) || !feature_perm || !aligned16(feature_perm)) return MIXLLM_EINVAL;
    if (!buf_ok(packed_w8, s.w8_bytes) || !buf_ok(packed_w4, s.w4_bytes) || !buf_ok(zeros4, s.zeros4_bytes) ||
        !buf_ok(scales8, s.scales8_bytes) || !buf_ok(scales4, s.scales4_bytes))
        return MIXLLM_EINVAL;
    LinearParams p = make_params(*d, nullptr, nullptr, packed_w4, packed_w8, scales4, scales8, zeros4, feature_perm);
    p.y = (half_t *)y;
    // One kernel when a decode variant can quantize inside the linear: every block then repeats the
    // quantizer, so the variants only offer it where that measured cheaper than the stand-alone
    // kernel's launch and round trips (one token; a few tokens of a short row).
    if (decode_can_fuse_quantizer(p)) {
        p.x = (const half_t *)x;
        const int e = launch_linear_decode(p, st);
        if (e != (int)hipErrorInvalidValue) return hip_status(e);
        p.x = nullptr;   // no variant took the shape after all (nothing was launched): two kernels
    }
    // two kernels: the stand-alone quantizer into the scratch area, then the linear; the kernel of the
    // linear is chosen, and the call refused if none takes the shape, before the quantizer is enqueued
    if (!scratch || !aligned16(scratch)) return MIXLLM_EINVAL;
    const size_t quant_bytes = round_up_sz(s.xq_bytes, 256) + round_up_sz(s.xscale_bytes, 256);
    if (scratch_bytes < quant_bytes) return MIXLLM_EWORKSPACE;
    int8_t *xq = (int8_t *)scratch;
    void *xscale = (uint8_t *)scratch + round_up_sz(s.xq_bytes, 256);
    p.xq = xq;
    p.xscale = (const half_t *)xscale;
    // what is left of the scratch area serves the tiled kernel's K split, if it is enough for that
    if (scratch_bytes > quant_bytes) {
        p.partials = (float *)((uint8_t *)scratch + quant_bytes);
        p.partials_cap = scratch_bytes - quant_bytes;
    }
    LinearParams q;
    const int path = resolve_path(*d, p, MIXLLM_PATH_AUTO, q);
    if (path < 0) return path;
    if (int rc = hip_status(launch_quantize_activations(*d, x, xq, xscale, st))) return rc;
    return run_path(q, path, st);
}

int mixllm_mixed_linear_fp16(const mixllm_desc *d, const void *x, const void *packed_w4, const void *packed_w8,
                             const void *scales4, const void *scales8, const void *zeros4,
                             const int32_t *feature_perm, void *y, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    return linear_from_fp16(d, x, packed_w4, packed_w8, scales4, scales8, zeros4, feature_perm, y, workspace,
                            workspace_bytes, (hipStream_t)stream);
}

// Device address of `scratch` on the current device; looked up once per device, with that device
// current, and kept.  Returns nullptr (and the HIP error in *err) when the lookup fails.
static void *static_scratch_ptr(hipError_t *err)
{
    static void *ptr[64] = {nullptr};
    static std::mutex mu;
    int dev = 0;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= 64) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *q = nullptr;
        *err = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !q) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        ptr[dev] = q;
    }
    return ptr[dev];
}

int mixllm_mixed_linear_fp16_static(const mixllm_desc *d, const void *x, const void *packed_w4, const void *packed_w8,
                                    const void *scales4, const void *scales8, const void *zeros4,
                                    const int32_t *feature_perm, void *y, void *stream)
{
    if (int rc = check_desc(d)) return rc;
    if (d->M == 0) return MIXLLM_OK;
    mixllm_sizes s;
    sizes_of(*d, s);
    // refused before anything is looked up or enqueued; a shape that runs as one kernel does not
    // touch the array, but the limit is the same for every call so that it does not depend on
    // which kernel the library happens to choose
    if (round_up_sz(s.xq_bytes, 256) + round_up_sz(s.xscale_bytes, 256) > (size_t)MIXLLM_STATIC_SCRATCH_BYTES) return MIXLLM_EWORKSPACE;
    hipError_t e = hipSuccess;
    void *area = static_scratch_ptr(&e);
    if (!area) return MIXLLM_EHIP;
    return linear_from_fp16(d, x, packed_w4, packed_w8, scales4, scales8, zeros4, feature_perm, y, area,
                            (size_t)MIXLLM_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
}

int mixllm_channel_salience(const mixllm_desc *d, const void *W, const void *G, float weight, int accumulate,
                            float *salience, void *stream)
{
    if (!d) return MIXLLM_EINVAL;
    if (d->K <= 0 || d->N < 0) return MIXLLM_EINVAL;
    if (d->group != MIXLLM_GROUP || d->K % MIXLLM_GROUP != 0) return MIXLLM_EUNSUPPORTED;
    if (d->N == 0) return MIXLLM_OK;
    if (!W || !G || !salience || !aligned16(W) || !aligned16(G)) return MIXLLM_EINVAL;
    return hip_status(mixllm::launch_channel_salience(W, G, d->N, d->K, weight, accumulate, salience,
                                                      (hipStream_t)stream));
}

size_t mixllm_select_salient_workspace(int32_t L) { return L > 0 ? mixllm::select_salient_workspace_bytes(L) : 0; }

int mixllm_select_salient(const float *salience, const int64_t *layer_offsets, int32_t L, int64_t T,
                          int32_t *selected, int32_t *layer_counts, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (L <= 0 || !layer_offsets || layer_offsets[0] != 0) return MIXLLM_EINVAL;
    for (int l = 0; l < L; ++l)
        if (layer_offsets[l + 1] < layer_offsets[l]) return MIXLLM_EINVAL;
    const int64_t total = layer_offsets[L];
    if (total >= (1ll << 31) || T < 0 || T > total) return MIXLLM_EINVAL;
    if (!layer_counts || (total > 0 && !salience) || (T > 0 && !selected)) return MIXLLM_EINVAL;
    if (!workspace || !aligned16(workspace)) return MIXLLM_EINVAL;
    if (workspace_bytes < mixllm::select_salient_workspace_bytes(L)) return MIXLLM_EWORKSPACE;
    return hip_status(mixllm::launch_select_salient(salience, layer_offsets, L, T, selected, layer_counts, workspace,
                                                    (hipStream_t)stream));
}

int mixllm_debug_check_fast_division(uint64_t *mismatches, void *stream)
{
    if (!mismatches || ((uintptr_t)mismatches & 7u)) return MIXLLM_EINVAL;
    return hip_status(launch_check_fast_division((unsigned long long *)mismatches, (hipStream_t)stream));
}

int mixllm_debug_work_split(const mixllm_desc *d, int path, int32_t *plan)
{
    if (int rc = check_desc(d)) return rc;
    if (!plan) return MIXLLM_EINVAL;
    LinearParams p = make_params(*d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    int out[16] = {0};
    bool ok;
    if (path == MIXLLM_PATH_DECODE_SPLIT) ok = decode_split_plan(p, out);
    else if (path == MIXLLM_PATH_MID) ok = mid_plan(p, out);
    else if (path == MIXLLM_PATH_PREFILL) ok = prefill_plan(p, out);
    else return MIXLLM_EINVAL;
    if (!ok) return MIXLLM_EUNSUPPORTED;
    for (int i = 0; i < 16; ++i) plan[i] = out[i];
    return MIXLLM_OK;
}

int mixllm_debug_group_partials(const mixllm_desc *d, const int8_t *xq, const void *packed_w4,
                                const void *packed_w8, const void *zeros4, const int32_t *feature_perm,
                                int32_t *P, int path, void *stream)
{
    if (!P) return MIXLLM_EINVAL;
    return linear_common(d, xq, nullptr, packed_w4, packed_w8, nullptr, nullptr, zeros4, feature_perm,
                         nullptr, P, nullptr, path, nullptr, 0, stream);
}

int mixllm_debug_channel_sums(const mixllm_desc *d, const int8_t *xq, const void *xscale, const void *packed_w4,
                              const void *packed_w8, const void *scales4, const void *scales8,
                              const void *zeros4, const int32_t *feature_perm, int32_t *S, int path, void *stream)
{
    if (!S) return MIXLLM_EINVAL;
    return linear_common(d, xq, xscale, packed_w4, packed_w8, scales4, scales8, zeros4, feature_perm, nullptr,
                         nullptr, S, path, nullptr, 0, stream);
}

}  // extern "C"
