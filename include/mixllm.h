/*
 * mixllm.h -- C ABI of the MI355X (gfx950) implementation of the MixLLM quantized
 * linear layer (arxiv 2412.14590): weights mix bit-widths between OUTPUT features
 * (Sec. 3.1.1): a salient set of n8 output channels is int8 symmetric, the other
 * N - n8 channels are uint4 asymmetric with one fp16 scale and one uint4 zero point
 * per group of 128 input features; activations are int8 symmetric (Sec. 3.1.2,
 * Sec. 4.1).  The linear is a fused dequantize + int8 MatMul with an int32 partial
 * sum per quantization group, rescaled in float (two-step dequantization, Sec. 3.3),
 * and both parts scatter into one output tensor in the original channel order
 * (Sec. 3.4).
 *
 * Conventions
 *   - Every function returns an int status: MIXLLM_OK or a negative error code.
 *     Arguments are validated on the host BEFORE anything is launched, so an error
 *     return means nothing ran.  No function throws.
 *   - Unless a parameter says "host", every data pointer is DEVICE memory, owned by
 *     the caller, 16-byte aligned, of the size mixllm_query_sizes() reports.  The
 *     library allocates no memory and keeps no state between calls (one entry point,
 *     mixllm_mixed_linear_fp16_static, keeps its scratch in a device array of its own).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it and the call returns without synchronizing and without blocking
 *     copies: no entry point waits for the device.
 *   - fp16 values are IEEE binary16, stored as 2-byte words.
 *   - Inputs holding Inf or NaN are not supported (results unspecified, no fault).
 *
 * Granularity variants (mixllm_desc):
 *   act_group = K   one activation scale per token          (default workload)
 *   act_group = 128 one activation scale per (token, group) (the paper's Sec. 3.1.2 choice)
 *   w8_group  = K   one scale per 8-bit channel             (default workload)
 *   w8_group  = 128 one scale per (8-bit channel, group)    (the paper's Sec. 4.1 choice)
 * The integer partial sums are the same in every variant; only the scale lookup changes.
 */
#ifndef MIXLLM_H
#define MIXLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIXLLM_GROUP 128
/* Largest K: an 8-bit channel with one scale keeps a single int32 sum over all of K, and
 * K * 127 * 127 must stay below 2^31. */
#define MIXLLM_MAX_K 131072
/* Bytes of the device array behind mixllm_mixed_linear_fp16_static. */
#define MIXLLM_STATIC_SCRATCH_BYTES (8u * 1024u * 1024u + 256u * 1024u)

enum {
    MIXLLM_OK = 0,
    MIXLLM_EINVAL = -1,       /* null or misaligned pointer, negative size, bad index list */
    MIXLLM_EUNSUPPORTED = -2, /* shape or variant the kernels do not cover (e.g. K % 128 != 0) */
    MIXLLM_EWORKSPACE = -3,   /* workspace smaller than mixllm_query_sizes() asked for */
    MIXLLM_EHIP = -4          /* a HIP runtime call failed (launch error, bad stream, ...) */
};

/* Kernel selection for the entry points that take a `path` argument. */
enum {
    MIXLLM_PATH_AUTO = 0,    /* decode path for M <= 16; 17..64 tokens: the path for a few dozen tokens or the tiled path,
                                whichever measured faster for the shape; tiled MFMA path otherwise */
    MIXLLM_PATH_GENERIC = 1, /* one thread per output element, no MFMA; any shape; slow */
    MIXLLM_PATH_DECODE = 2,  /* weight-streaming path, M <= 16; picks one of the three variants below */
    MIXLLM_PATH_PREFILL = 3, /* LDS-staged tiled MFMA path, any M */
    /* the variants of the decode path, for tests and benchmarks */
    MIXLLM_PATH_DECODE_STREAM = 4,   /* a wave per tile (or per K part of a tile), activations re-read per tile */
    MIXLLM_PATH_DECODE_RESIDENT = 5, /* activation fragments kept in registers; falls back to STREAM where it cannot run */
    MIXLLM_PATH_DECODE_SPLIT = 6,    /* equal byte shares per block, activations in LDS; EUNSUPPORTED where it cannot run */
    MIXLLM_PATH_MID = 7,             /* weight-streaming path for a few dozen tokens, M <= 64 (M <= 32 with one activation
                                        scale per (token, group)); EUNSUPPORTED where it cannot run */
    /* the tiled path with the block shape chosen by the caller instead of by the grid size, for tests
       and benchmarks: 32, 64 or 128 token rows x 128 channels */
    MIXLLM_PATH_PREFILL_32 = 8,
    MIXLLM_PATH_PREFILL_64 = 9,
    MIXLLM_PATH_PREFILL_128 = 10     /* EUNSUPPORTED with one activation scale per (token, group) */
};

typedef struct mixllm_desc {
    int32_t M;         /* tokens (rows of x and y); may be 0 for the offline calls */
    int32_t K;         /* input features, multiple of 128, at most MIXLLM_MAX_K */
    int32_t N;         /* output features */
    int32_t n8;        /* how many of the N output channels are int8, 0..N */
    int32_t group;     /* quantization group size along K for the uint4 part: must be 128 */
    int32_t act_group; /* K or 128, see above */
    int32_t w8_group;  /* K or 128, see above */
} mixllm_desc;

/*
 * Buffer sizes in bytes.  Packed layouts (opaque to callers; use pack/unpack to cross):
 *   rows of each part are padded to a multiple of 16 (n8p, n4p), groups of metadata to a
 *   multiple of 8 (ngp), padding is zero-filled by the library.
 *   packed_w8  [n8p/16][K/64][64][16 B]  int8; 16-row tile x 64-k step in MFMA B-operand
 *              order: slot (c + 16*ks) holds row c, k = 64*step + 16*ks .. +15
 *   packed_w4  [n4p/16][K/128][64][16 B] uint4 pairs; slot (c + 16*ks) holds row c of the
 *              tile: bytes 0-7 -> k = 128*g + 16*ks .. +15, bytes 8-15 -> the same + 64;
 *              inside 8 bytes, byte b of dword d holds k-local 8d+b (low nibble) and
 *              8d+4+b (high nibble)
 *   scales4    fp16 [n4p][ngp]           zeros4   uint4 pairs [n4p][ngp/2]
 *   scales8    fp16 [n8p] (w8_group = K) or fp16 [n8p][ngp] (w8_group = 128)
 *   feature_perm int32 [N]: row j of the concatenation [8-bit rows ; 4-bit rows] is
 *              output channel feature_perm[j]; a bijection on [0,N)
 *   xq int8 [M][K] row-major     xscale fp16 [M][K/act_group]     y fp16 [M][N]
 */
typedef struct mixllm_sizes {
    size_t w8_bytes, w4_bytes, scales8_bytes, scales4_bytes, zeros4_bytes, perm_bytes;
    size_t xq_bytes, xscale_bytes, y_bytes;
    size_t workspace_bytes;   /* scratch mixllm_mixed_linear_fp16 makes use of: xq, then xscale (each rounded up to
                                 256 B), then linear_workspace_bytes.  It runs with as little as the first two. */
    size_t linear_workspace_bytes; /* optional scratch of mixllm_mixed_linear: where the tiled path has too few output
                                 tiles to fill the chip (a few hundred tokens, or few channels) it splits K over several
                                 blocks and adds their fp32 sums, in a fixed order, from this area; 0 for shapes it
                                 does not split.  Without it the same kernel runs unsplit. */
} mixllm_sizes;

const char *mixllm_status_string(int status);

/* Library/ABI version, bumped when a packed layout or a signature changes. */
int mixllm_abi_version(void);

/* Sizes of the buffers of one layer in the packed layouts described above (footprints of Sec. 3.5:
 * 0.5 + 2.5/G bytes per 4-bit weight, 1 + 2/G per 8-bit weight with group-wise scales).
 * Pure host arithmetic; never touches the GPU.  Errors: EINVAL (null), EUNSUPPORTED (dims). */
int mixllm_query_sizes(const mixllm_desc *d, mixllm_sizes *out);

/*
 * Order of the concatenated rows (Sec. 3.4: the two parts own different channel indices):
 * the n8 salient channels ascending, then all other channels ascending.  HOST pointers
 * in and out; pure host code.  salient_idx may be in any order.
 * Errors: EINVAL for null pointers, an index outside [0,N) or a duplicate.
 */
int mixllm_build_feature_perm(int32_t N, int32_t n8, const int32_t *salient_idx_host,
                              int32_t *perm_host /* [N] */);

/*
 * Offline weight quantization and packing (Sec. 2 quantizer; configuration of Sec. 3.1.2 and
 * Sec. 4.1; ahead-of-time layout prepacking, Sec. 3.3 last paragraph).
 *   W            fp16 [N][K] row-major, device
 *   salient_idx  DEVICE int32 [n8] (4-byte aligned; may be NULL when n8 = 0): the channels to
 *                keep at 8 bits, distinct, in [0, N), in any order - the per-layer slice of the
 *                global search result (Alg. 1), i.e. what mixllm_select_salient leaves in
 *                `selected`; choosing them is the caller's business.  The list stays on the
 *                device, so its contents are not validated: an index outside [0, N) is ignored,
 *                a repeated one counts once, and with fewer than n8 distinct valid entries the
 *                order of the rows is unspecified (never an access out of bounds).
 *                mixllm_build_feature_perm validates a host copy of the list.
 * 8-bit rows: s = fp16(absmax/127) per channel (or per group), q = clamp(rne(w/s),-127,127).
 * 4-bit rows, per group of 128: mn = min(w,0), mx = max(w,0), s = fp16((mx-mn)/15),
 * z = clamp(rne(-mn/s),0,15), q = clamp(rne(w/s)+z,0,15).  A scale that comes out 0 is
 * stored as 1.  All in fp32 with true division and round-half-to-even.
 * Writes packed_w8, packed_w4, scales8, scales4, zeros4, feature_perm (all device).
 * feature_perm is built on the device from the list (the listed channels ascending, then the
 * others ascending); everything is enqueued on `stream`, nothing crosses to the host.
 */
int mixllm_quantize_weights(const mixllm_desc *d, const void *W, const int32_t *salient_idx,
                            void *packed_w8, void *packed_w4, void *scales8, void *scales4,
                            void *zeros4, int32_t *feature_perm, void *stream);

/*
 * Canonical <-> packed conversion (the ahead-of-time layout prepacking of Sec. 3.3, last
 * paragraph, and its inverse), so that callers (and tests) can inject codes produced
 * elsewhere and read the library's codes back.  Canonical device arrays:
 *   q8 int8 [n8][K]; s8 fp16 [n8][K/w8_group]; q4 uint8 [n4][K] one code (0..15) per byte;
 *   s4 fp16 [n4][K/128]; z4 uint8 [n4][K/128] one zero point (0..15) per byte;
 *   perm int32 [N] as above.  Arrays of an empty part may be NULL.
 * pack copies perm to feature_perm; unpack copies it back.  Code values above 15 are
 * masked to 4 bits.  Asynchronous on `stream`.
 */
int mixllm_pack_weights(const mixllm_desc *d, const int8_t *q8, const void *s8, const uint8_t *q4,
                        const void *s4, const uint8_t *z4, const int32_t *perm, void *packed_w8,
                        void *packed_w4, void *scales8, void *scales4, void *zeros4,
                        int32_t *feature_perm, void *stream);
int mixllm_unpack_weights(const mixllm_desc *d, const void *packed_w8, const void *packed_w4,
                          const void *scales8, const void *scales4, const void *zeros4,
                          const int32_t *feature_perm, int8_t *q8, void *s8, uint8_t *q4, void *s4,
                          uint8_t *z4, int32_t *perm, void *stream);

/*
 * Activation quantizer (Sec. 2 formula with z = 0; 8-bit symmetric, Sec. 3.1.2):
 * per token (or per token and group): s = fp16(absmax/127), 0 -> 1;
 * xq = clamp(rne(x/s), -127, 127), computed in fp32 with true division.
 *   x fp16 [M][K] -> xq int8 [M][K], xscale fp16 [M][K/act_group].  M = 0 is a no-op.
 */
int mixllm_quantize_activations(const mixllm_desc *d, const void *x, int8_t *xq, void *xscale,
                                void *stream);

/*
 * The quantized linear (Fig. 1; Sec. 3.3 two-step dequantization; Sec. 3.4 scatter):
 *   P[m,j,g]  = sum_{k in group g} xq[m,k] * (q4[j,k] - z[j,g])   (int32, exact; 8-bit rows: q8)
 *   y[m, feature_perm[j]] = fp16( sum_g float(P[m,j,g]) * s_w[j,g] * s_a[m,g] )   (fp32 sums)
 * One launch covers both parts (plus a second, small one where K is split, see below).  M = 0 is a
 * no-op.  workspace is optional (NULL and 0 are fine): with mixllm_query_sizes().linear_workspace_bytes
 * of it (16-byte aligned) the tiled path splits K over several blocks where its grid of output tiles
 * would leave most of the chip idle; with less it splits as far as the bytes reach, or not at all.
 * The split changes the order of the fp32 additions, nothing else.
 * Errors: EINVAL, EUNSUPPORTED (path cannot run this shape, e.g. DECODE with M > 16),
 * EWORKSPACE, EHIP.
 */
int mixllm_mixed_linear(const mixllm_desc *d, const int8_t *xq, const void *xscale,
                        const void *packed_w4, const void *packed_w8, const void *scales4,
                        const void *scales8, const void *zeros4, const int32_t *feature_perm,
                        void *y, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Activation quantizer and quantized linear in one call (Fig. 1 end to end: fp16 activations in,
 * fp16 outputs in the original channel order out):
 *   x fp16 [M][K] -> y fp16 [M][N], same definition as mixllm_quantize_activations followed by
 *   mixllm_mixed_linear (the same codes and scales; the fp32 sums may be taken in another order).
 * For up to 16 tokens with M K <= 16384 (several tokens with one activation scale per token: K a
 * multiple of 512) this is ONE kernel: every block of the decode kernel quantizes the activations itself while its first
 * weight loads are in flight, and `workspace` is not touched (may be NULL).  Otherwise the two
 * kernels run back to back on `stream` with xq and xscale placed in `workspace` (at least
 * mixllm_query_sizes().workspace_bytes, 16-byte aligned).
 * Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP.  M = 0 is a no-op.
 */
int mixllm_mixed_linear_fp16(const mixllm_desc *d, const void *x, const void *packed_w4,
                             const void *packed_w8, const void *scales4, const void *scales8,
                             const void *zeros4, const int32_t *feature_perm, void *y, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * mixllm_mixed_linear_fp16 for callers that can neither allocate device memory nor hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments without the workspace, same kernels; the scratch area (xq, xscale, then whatever is
 * left for the tiled path's K split) is a device array inside the library,
 * MIXLLM_STATIC_SCRATCH_BYTES long, that every GPU the library runs on holds until the process
 * ends.  The call allocates nothing.  Results are those of mixllm_mixed_linear_fp16 with a
 * workspace of that size: bit-identical where both have room for the same K split (always when
 * K < 8192), otherwise the fp32 additions may come in another order.
 *   - A shape whose xq and xscale (each rounded up to 256 bytes) exceed the array is refused
 *     with MIXLLM_EWORKSPACE before anything is enqueued.  8 MiB + 256 KiB covers M K up to
 *     8 Mi activation values, e.g. 2048 tokens of K = 4096 with either scale granularity.
 *   - Every call on a GPU shares that GPU's array: calls that overlap on one GPU (different
 *     streams, or different threads) race on it.  Calls on one stream are ordered and safe.
 *     Nothing in the array has to start at zero: the quantizer writes every byte the linear
 *     reads, whatever an earlier call left there.
 * Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP.  M = 0 is a no-op.
 */
int mixllm_mixed_linear_fp16_static(const mixllm_desc *d, const void *x, const void *packed_w4,
                                    const void *packed_w8, const void *scales4, const void *scales8,
                                    const void *zeros4, const int32_t *feature_perm, void *y, void *stream);

/* Same as mixllm_mixed_linear, with the kernel chosen by the caller (MIXLLM_PATH_*); for tests and benchmarks. */
int mixllm_mixed_linear_path(const mixllm_desc *d, const int8_t *xq, const void *xscale,
                             const void *packed_w4, const void *packed_w8, const void *scales4,
                             const void *scales8, const void *zeros4, const int32_t *feature_perm,
                             void *y, void *workspace, size_t workspace_bytes, int path,
                             void *stream);

/*
 * Global precision search, step 1 (Sec. 3.2, Eq. 4; lines 3-6 of Alg. 1): salience of every
 * output channel of one layer for one gradient sample,
 *     S1[n] = sum_k G[n][k] * (Qdq(W)[n][k] - W[n][k]),     S[n] = | S1[n] + S1[n]^2 / 2 |,
 * where Qdq is the 4-bit group-wise quantizer of mixllm_quantize_weights followed by its
 * dequantization (q - z) * s (the same codes, bit for bit).
 *   W, G      device, fp16 [N][K] row-major (weights and the loss gradient w.r.t. them), 16-byte aligned
 *   salience  device, fp32 [N]: salience[n] = (accumulate ? salience[n] : 0) + weight * S[n].
 *             Eq. 4's mean over the calibration set is one call per sample with weight = 1 / |D|,
 *             accumulate = 0 for the first sample.
 * Only d->K, d->N and d->group are read.  Sums run in fp32.  Errors: EINVAL, EUNSUPPORTED, EHIP.
 */
int mixllm_channel_salience(const mixllm_desc *d, const void *W, const void *G, float weight,
                            int accumulate, float *salience, void *stream);

/*
 * Global precision search, step 2 (last two lines of Alg. 1): of all channels of all layers the
 * T with the largest salience are the 8-bit ones.  Equal saliences (the paper does not order
 * them): the channel that comes first in the concatenation is taken first.
 *   salience        device, fp32 [layer_offsets[L]]: the layers' saliences one after another;
 *                   every value finite and >= 0
 *   layer_offsets   HOST, int64 [L + 1], ascending from 0: layer l owns [offsets[l], offsets[l+1]);
 *                   read before the call returns (the values travel as kernel arguments: no copy,
 *                   no wait)
 *   T               0 <= T <= layer_offsets[L] < 2^31
 *   selected        device, int32 [T]: the chosen channels as indices INSIDE their layer, layer after
 *                   layer, ascending inside a layer - layer l's slice is what mixllm_quantize_weights
 *                   takes as salient_idx, where it lies
 *   layer_counts    device, int32 [L]: length of every layer's slice (the layer's n8)
 *   workspace       device, at least mixllm_select_salient_workspace(L) bytes, 16-byte aligned
 * Errors: EINVAL, EWORKSPACE, EHIP.
 */
size_t mixllm_select_salient_workspace(int32_t L);
int mixllm_select_salient(const float *salience, const int64_t *layer_offsets, int32_t L, int64_t T,
                          int32_t *selected, int32_t *layer_counts, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Test hook: the quantizer kernels round v / s (v, s fp16 values) with a reciprocal, a product and
 * one residual correction instead of a division.  This call compares, on the GPU, the rounded
 * result with that of the IEEE division for every finite fp16 v and every positive finite fp16 s
 * (2.0e9 pairs) and adds the number of differences to *mismatches (device, uint64, zeroed by the
 * caller).  Errors: EINVAL, EHIP.
 */
int mixllm_debug_check_fast_division(uint64_t *mismatches, void *stream);

/*
 * Test hook (host only, launches nothing): how a kernel of the given path would split the layer
 * of `d` over its blocks.  path = MIXLLM_PATH_DECODE_SPLIT: plan[0..5] = blocks of the 8-bit part,
 * blocks of the 4-bit part, virtual tiles covered by a block's LDS cells, bytes of LDS, windows over K
 * the int8 activations are staged in (1 = the whole matrix at once), chunk columns (512 values of K)
 * per window;
 * path = MIXLLM_PATH_MID: plan[0..4] = blocks of the 8-bit part, of the 4-bit part, quarter tiles
 * per virtual tile of the 8-bit and of the 4-bit part, bytes of LDS; path = MIXLLM_PATH_PREFILL:
 * plan[0..12] = token rows and channels of a block tile of the 4-bit part, its token tiles, channel
 * tiles of the 8-bit and of the 4-bit part, blocks launched per K part, token tiles per band of the
 * block order (4-bit part), bytes of LDS, K parts (with linear_workspace_bytes of scratch),
 * quantization groups per K part, then token rows of a block tile of the 8-bit part (the 4-bit
 * part's, or half of that in a short launch of 128-row tiles), its token tiles and its token tiles per band.  plan must hold
 * 16 ints.  Returns EUNSUPPORTED when the path does not cover the shape, EINVAL for other
 * paths.
 */
int mixllm_debug_work_split(const mixllm_desc *d, int path, int32_t *plan);

/*
 * Test hook: the exact int32 partial sum of every (token, channel, group) (Sec. 3.3: the MMA of the
 * two-step dequantization, before the float step), written in ORIGINAL channel order:
 * P int32 [M][N][K/128].  Decode paths, the path for a few dozen tokens and the tiled path run the
 * body of the linear's own kernel with the rescale replaced by a store: the same hand-issued loads
 * and waits, the same unpacking and MFMA sequence.  Two differences from the linear remain, both in
 * the tiled path: no scales are passed, so the group metadata request is one load instead of two;
 * and 8-bit tiles with one scale per channel, which the linear accumulates over all of K in one
 * int32 (no per-group value exists there), take the per-group pipeline of the group-wise 8-bit
 * scales.  mixllm_debug_channel_sums covers that accumulator.
 */
int mixllm_debug_group_partials(const mixllm_desc *d, const int8_t *xq, const void *packed_w4,
                                const void *packed_w8, const void *zeros4,
                                const int32_t *feature_perm, int32_t *P, int path, void *stream);

/*
 * Test hook: S[m][n] = sum over the groups of P[m][n][g], int32 [M][N] in ORIGINAL channel order,
 * from the kernels the linear itself launches for `d` (same arguments, same block shape, same loads,
 * waits, unpacking and MFMAs; only the float rescale of a group partial is replaced by an integer
 * add, and the epilogue stores the integer).  For 8-bit tiles with one scale per channel this is the
 * very accumulator the linear converts and scales (Sec. 3.3 step 2 applied once per channel).
 * path: MIXLLM_PATH_GENERIC, MIXLLM_PATH_PREFILL and its block-shape variants; others EUNSUPPORTED.
 */
int mixllm_debug_channel_sums(const mixllm_desc *d, const int8_t *xq, const void *xscale,
                              const void *packed_w4, const void *packed_w8, const void *scales4,
                              const void *scales8, const void *zeros4, const int32_t *feature_perm,
                              int32_t *S, int path, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MIXLLM_H */
