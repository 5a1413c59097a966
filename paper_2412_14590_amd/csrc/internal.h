// Internal declarations shared by the HIP translation units of libmixllm_hip.so.
// Not part of the public ABI (that is include/mixllm.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mixllm.h"

namespace mixllm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 half_t;

constexpr int G = MIXLLM_GROUP;   // quantization group along K (Sec. 4.1)
constexpr int TILE_N = 16;        // rows of one packed weight tile

static inline __host__ __device__ int round_up(int a, int b) { return (a + b - 1) / b * b; }

// Everything a linear / partials kernel needs, by value.
// decode variants a caller can name through the path argument of the linear entry points
enum DecodeVariant { DECODE_ANY = 0, DECODE_STREAM, DECODE_RESIDENT, DECODE_SPLIT };

struct LinearParams {
    int M, K, N, n8, n4;
    int ng;         // K / 128
    int ngp;        // ng rounded up to 8: row stride of scales4 / per-group scales8 (elements)
    int ntiles8;    // n8p / 16
    int ntiles4;    // n4p / 16
    int act_per_token;   // 1: xscale [M], 0: xscale [M][ng]
    int w8_per_channel;  // 1: scales8 [n8p], 0: scales8 [n8p][ngp]
    int variant;         // decode variant requested by the caller's path argument (DECODE_ANY = library's choice)
    int prefill_tm;      // token tiles of 32 per wave of the tiled kernel requested by the caller's path argument (0 = library's choice)
    // tiled kernel with K split over several blocks: fp32 sums of every part in caller-provided scratch
    int kparts;          // blocks that share the K range of one output tile (1 = no split)
    int quads_per_part;  // groups of 4 quantization groups per part
    int np;              // row stride of `partials`: ntiles8 * 16 + ntiles4 * 16 (the concatenated rows, each part padded)
    float *partials;     // [kparts][M][np], or null when the caller brought no scratch
    size_t partials_cap; // bytes behind `partials`: the launcher splits K only as far as they reach
    const half_t *x;   // fp16 activations [M][K]: set only by the fused quantize + linear entry point
    const int8_t *xq;
    const half_t *xscale;
    const uint8_t *w4;
    const int8_t *w8;
    const half_t *s4;
    const half_t *s8;
    const uint8_t *z4;
    const int32_t *perm;
    half_t *y;        // linear output, or
    int32_t *P;       // per-group partial sums [M][N][ng] (debug entry point), or
    int32_t *S;       // their sums over the groups [M][N] (debug entry point); exactly one of y / P / S is used
};

// ---- packed-layout addressing (see mixllm.h for the layout description) ----

// byte offset of the 16-byte slot holding row `r` (of the 4-bit part), group g, k-slot ks
static inline __host__ __device__ size_t w4_slot_offset(int r, int g, int ks, int ng)
{
    return (((size_t)(r / TILE_N) * ng + g) * 64 + (r % TILE_N) + 16 * ks) * 16;
}
// byte offset of the 16-byte slot holding row r (of the 8-bit part), k = 64*step + 16*ks..+15
static inline __host__ __device__ size_t w8_slot_offset(int r, int step, int ks, int nsteps)
{
    return (((size_t)(r / TILE_N) * nsteps + step) * 64 + (r % TILE_N) + 16 * ks) * 16;
}

// zero point of (row r, group g) from the nibble-packed array
static inline __device__ int z4_load(const uint8_t *z4, int r, int g, int ngp)
{
    uint8_t b = z4[(size_t)r * (ngp / 2) + (g >> 1)];
    return (g & 1) ? (b >> 4) : (b & 15);
}

// Unpack one dword of 8 uint4 codes into two dwords of 4 int8 each, subtracting the zero
// point on the way (step 1 of the two-step dequantization, Sec. 3.3).  `zb` holds
// (0x80 - z) in every byte: code + (0x80 - z) never carries between bytes (<= 0x8F), and
// flipping the top bit of each byte afterwards leaves code - z in two's complement.
static inline __device__ void unpack_sub(uint32_t w, uint32_t zb, int &lo, int &hi)
{
    lo = (int)(((w & 0x0F0F0F0Fu) + zb) ^ 0x80808080u);
    hi = (int)((((w >> 4) & 0x0F0F0F0Fu) + zb) ^ 0x80808080u);
}
// 16 codes (two packed dwords) -> the four int8 dwords one lane feeds to an MFMA, k order 0..15
static inline __device__ v4i unpack16(uint32_t w0, uint32_t w1, uint32_t zb)
{
    int a, b, c, d;
    unpack_sub(w0, zb, a, b);
    unpack_sub(w1, zb, c, d);
    return v4i{a, b, c, d};
}
static inline __device__ uint32_t zbias(int z) { return 0x80808080u - 0x01010101u * (uint32_t)z; }

// ---- activation quantizer arithmetic (Sec. 2 formula with z = 0), shared by the stand-alone
// quantizer kernel and the decode kernel that quantizes its own activations ----

// fp32 scale -> stored fp16 scale; a scale that is (or rounds to) zero becomes 1.
static inline __device__ half_t store_scale(float s32)
{
    half_t s16 = (half_t)s32;   // round-to-nearest-even conversion
    if ((float)s16 == 0.0f) s16 = (half_t)1.0f;
    return s16;
}
// The quantizers need round(v / s) with v and s both fp16-valued and the true (IEEE) quotient
// rounded half to even.  A full fp32 division is a dozen vector instructions; the quantizers are
// bound by them.  quotient() takes the reciprocal r = rcp(s) (one instruction per scale, 1 ulp),
// the product v r and one residual correction.  Its result is not always the correctly rounded
// quotient, but rint() of it equals rint() of the correctly rounded quotient for EVERY pair of
// finite fp16 values: a quotient of two 11-bit significands that is not itself a multiple of 1/2 is
// at least 2^-15 away from one, far more than the error left after the correction, and an exact
// multiple of 1/2 comes out exactly.  mixllm_debug_check_fast_division compares the two for all
// 2.0e9 pairs on the GPU (no mismatch); the parity tests compare the codes with the oracle's,
// which divides.
static inline __device__ float recip(float s) { return __builtin_amdgcn_rcpf(s); }
static inline __device__ float quotient(float v, float s, float r)
{
    const float t0 = v * r;
    const float e = __builtin_fmaf(-t0, s, v);
    return __builtin_fmaf(e, r, t0);
}
// one int8 code: v / s rounded half to even, clamped to [-127, 127]; returned in the low byte
static inline __device__ uint32_t quant_code(half_t v, float s, float r)
{
    float t = __builtin_rintf(quotient((float)v, s, r));
    t = fminf(fmaxf(t, -127.0f), 127.0f);
    return (uint32_t)(int)t & 0xffu;
}
// the same with the IEEE division (the reference of the exhaustive check)
static inline __device__ uint32_t quant_code_ieee(half_t v, float s)
{
    float t = __builtin_rintf((float)v / s);
    t = fminf(fmaxf(t, -127.0f), 127.0f);
    return (uint32_t)(int)t & 0xffu;
}

// ---- launchers (defined one per .hip file); return a hipError_t as int ----
int launch_quantize_activations(const mixllm_desc &d, const void *x, int8_t *xq, void *xs,
                                hipStream_t st);
int launch_check_fast_division(unsigned long long *mismatches, hipStream_t st);
int launch_quantize_weights(const mixllm_desc &d, const void *W, void *w8, void *w4, void *s8,
                            void *s4, void *z4, const int32_t *perm, hipStream_t st);
// feature_perm [N] from a device list of the n8 channels kept at 8 bits (quant_weights.hip)
int launch_build_feature_perm(int N, int n8, const int32_t *salient_idx_dev, int32_t *perm, hipStream_t st);
int launch_pack_weights(const mixllm_desc &d, const int8_t *q8, const void *s8c, const uint8_t *q4,
                        const void *s4c, const uint8_t *z4c, void *w8, void *w4, void *s8,
                        void *s4, void *z4, hipStream_t st);
int launch_unpack_weights(const mixllm_desc &d, const void *w8, const void *w4, const void *s8,
                          const void *s4, const void *z4, int8_t *q8, void *s8c, uint8_t *q4,
                          void *s4c, uint8_t *z4c, hipStream_t st);
int launch_linear_generic(const LinearParams &p, hipStream_t st);
int launch_linear_decode(const LinearParams &p, hipStream_t st);
// evenly split decode variant
int launch_linear_decode_split(const LinearParams &p, hipStream_t st);
bool decode_split_covers(const LinearParams &p);
bool decode_split_plan(const LinearParams &p, int out[6]);
bool mid_plan(const LinearParams &p, int out[5]);
// Raise a kernel's dynamic-LDS limit (a per-function, per-device attribute; set once).  Returns a hipError_t.
int ensure_dynamic_lds(const void *kernel, size_t bytes);
// compute units of the current device (256 where the query fails)
int cu_count();
// true when launch_linear_decode can take fp16 activations (p.x) and quantize them itself
bool decode_can_fuse_quantizer(const LinearParams &p);
int launch_linear_prefill(const LinearParams &p, hipStream_t st);
bool prefill_covers(const LinearParams &p);
// scratch bytes the tiled kernel would like for `p` (0 where it does not split K)
size_t prefill_scratch_bytes(const LinearParams &p);
// true when the tiled kernel, given p.partials / p.partials_cap, would split K for `p`
bool prefill_would_split(const LinearParams &p);
bool prefill_plan(const LinearParams &p, int out[13]);
// path for 17..128 tokens (linear_mid.hip)
bool mid_covers(const LinearParams &p);
int launch_linear_mid(const LinearParams &p, hipStream_t st);
// global precision search (salience.hip)
int launch_channel_salience(const void *W, const void *Gr, int N, int K, float weight, int accumulate, float *salience,
                            hipStream_t st);
size_t select_salient_workspace_bytes(int L);
int launch_select_salient(const float *salience, const int64_t *layer_offsets_host, int L, int64_t T, int32_t *selected,
                          int32_t *layer_counts, void *workspace, hipStream_t st);

}  // namespace mixllm
