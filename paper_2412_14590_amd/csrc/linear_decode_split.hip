// Decode path, evenly split variant (M <= 16): every block streams (nearly) the same number of
// weight bytes, whatever the layer's shape, and no block depends on another.
//
// A layer of N channels has N / 16 packed tiles; with K = 4096 a 4-bit tile is 32 KB and a CU's
// share of the gate+up projection is about eight of them, of the output projection one and a
// bit, and a tile of the down projection (K = 14336) is 112 KB or 224 KB.  Handing out whole
// tiles leaves the chip a fifth to two thirds idle at the end.  Here
//  * the unit handed to a block is a quarter tile: 4 channels, all of K.  In the packed layout
//    the 4 channels are 64 contiguous bytes of every 256-byte row, so quarter tiles cost no
//    extra memory traffic.  Four quarter tiles make a virtual tile: the 16 columns of the
//    MFMA's B operand are independent, so they may come from two neighbouring packed tiles
//    (only the lanes' addresses differ);
//  * whole tiles are dealt round robin (block b takes tiles b, b + B, b + 2B, ...: at any moment
//    the chip reads one contiguous window, which HBM serves faster than as many separate
//    streams as there are blocks), the tiles left after the last full round in quarter tiles,
//    one partly filled virtual tile per block; the numbers of blocks given to the 8-bit and to
//    the 4-bit tiles are chosen so that the largest share (in bytes) is as small as possible;
//  * inside the block the unit of work is a chunk (four quantization groups of a virtual
//    tile: 4 KB of 4-bit or 8 KB of 8-bit weights) and wave w takes chunks w, w + 8, w + 16,
//    ... of the share: the eight waves read eight consecutive chunks at a time and end within
//    one chunk of each other;
//  * a wave keeps a ring of chunk requests in flight: two chunks are requested before the block
//    quantizes and stages its activations, then one beyond the chunk being consumed.  The loads
//    are issued and awaited by hand (async_loads.h): left to the compiler they are moved next to
//    their first use, and the ring collapses to one request at a time;
//  * the int8 activations sit in LDS, staged once per block (with fp16 input of up to 16 Ki
//    values the block runs the activation quantizer itself, same arithmetic, identical codes;
//    more than 128 Ki values - 5..16 tokens of a long K - pass through two LDS buffers in windows
//    over K, see WIN below);
//  * the zero point is hoisted out of the unpack, sum a (q - z) = sum a q - z sum a, with
//    sum a from an MFMA against an all-ones operand (int32-exact);
//  * a wave adds each chunk's contribution to its own LDS cell of the chunk's virtual tile;
//    after one barrier the cells of a virtual tile are summed in wave order (a fixed order of
//    floating point additions), scaled, converted and scattered.
// For up to 4 tokens the tokens sit in rows 0, 4, 8, 12 of the MFMA's A operand, so that one
// accumulator register per lane holds everything (NR = 1); for 5..16 tokens NR = 4.
// Two-step dequantization, Sec. 3.3; scatter to the original channel order, Sec. 3.4.
#include <algorithm>
#include <type_traits>

#include "async_loads.h"
#include "internal.h"

namespace mixllm {

namespace {

constexpr int NW = 8;              // waves per block
constexpr int NT = NW * 64;
constexpr int A_PAD = 16;          // bytes added to every staged activation row
constexpr int LDS_HEADER = 128;    // row maxima of the built-in quantizers in front of the cells
constexpr int MAX_BLOCKS = 2048;
constexpr size_t LDS_LIMIT = 156 * 1024;
#ifndef MIXLLM_SPLIT_RING
#define MIXLLM_SPLIT_RING 2    // chunks requested before the first is consumed
#endif
#ifndef MIXLLM_SPLIT_EARLY
#define MIXLLM_SPLIT_EARLY 1   // how many of them go out together with the activation loads
#endif

typedef half_t h8 __attribute__((ext_vector_type(8)));

struct SplitArgs {
    int nblk8, nblk4;   // blocks of the 8-bit and of the 4-bit part
    uint32_t magic;     // ceil(2^32 / chunks per tile)
    int tcap;           // virtual tiles a block's LDS cells cover
    // activation matrices beyond the LDS stage (WIN): K is walked in nwin windows of wq chunk
    // columns (the last one may be shorter); magic_w, magic_l = ceil(2^32 / chunk columns) of a
    // full window and of the last one
    int nwin, wq;
    uint32_t magic_w, magic_l;
};

template <int I, int N, typename F>
__device__ inline void sfor(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        sfor<I + 1, N>(f);
    }
}

// block barrier that waits for this wave's LDS traffic but not for its outstanding global loads
__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <bool PART8>
struct Slot {   // one chunk in flight
    v4i w[4][PART8 ? 2 : 1];
    uint2 s;       // 4 fp16 group scales
    uint32_t z;    // 4 zero points (4-bit) or the fp16 channel scale (8-bit with one scale per channel)
};

template <int N>
__device__ inline void await_slot(Slot<false> &k)
{
    asm volatile("s_waitcnt vmcnt(%6)"
                 : "+v"(k.w[0][0]), "+v"(k.w[1][0]), "+v"(k.w[2][0]), "+v"(k.w[3][0]), "+v"(k.s), "+v"(k.z)
                 : "n"(N)
                 : "memory");
}
template <int N>
__device__ inline void await_slot(Slot<true> &k)
{
    asm volatile("s_waitcnt vmcnt(%10)"
                 : "+v"(k.w[0][0]), "+v"(k.w[0][1]), "+v"(k.w[1][0]), "+v"(k.w[1][1]), "+v"(k.w[2][0]),
                   "+v"(k.w[2][1]), "+v"(k.w[3][0]), "+v"(k.w[3][1]), "+v"(k.s), "+v"(k.z)
                 : "n"(N)
                 : "memory");
}
template <int N>
__device__ inline void await_vec(v4i &a)
{
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}

// FUSED: 0 = int8 codes and scales come from the stand-alone quantizer; 1 = one token of fp16
// activations, 2 = several tokens of them (K a multiple of 512), quantized by every block for itself
// WIN: the int8 activation matrix is larger than the LDS stage (5..16 tokens of a long K).  The block
// then walks K in windows: its chunks are ordered window by window (inside a window as before:
// virtual tile by virtual tile, wave w taking chunks w, w + 8, ...), and the stage is two buffers,
// one holding the window being read, the other being filled with the next one by loads that write
// straight to LDS (no registers), requested a whole window ahead.  A change of window is one barrier.
// The ring of weight requests runs on across it; the LDS cells collect a virtual tile's
// contributions over all windows.
template <int NR, bool DUMP, bool ACT_PT, bool PART8, int FUSED, bool WIN>
__device__ inline void split_block(const LinearParams &p, const SplitArgs &a, uint8_t *smem)
{
    static_assert(!WIN || FUSED == 0, "windows are for int8 activations from the stand-alone quantizer");
    // Chunk requests: R chunks are requested before the first one is consumed - E of them in the
    // same instant as the activations, the others as soon as the activations have landed, so that
    // the memory system has work while the block quantizes and stages them - and from then on one
    // chunk beyond the one being consumed (a ring that stays R deep measured slower: 0.3 to 0.7 us
    // per slot beyond two on 8 to 67 MB layers).
    constexpr int R = MIXLLM_SPLIT_RING, E = MIXLLM_SPLIT_EARLY;
    static_assert(R >= 2 && E >= 1 && E <= R, "ring of at least two slots, at least one early request");
    constexpr int GB = PART8 ? 2048 : 1024;     // bytes of one group of one tile
    constexpr int NLW = PART8 ? 8 : 4;
    constexpr int NLM = PART8 ? (DUMP ? 0 : 1) : (DUMP ? 1 : 2);
    constexpr int NL = NLW + NLM;               // loads per chunk
    constexpr int MAXV = FUSED ? 4 : 16;   // staging loads per thread (up to 128 KB of int8 codes, or 32 KB of fp16 values)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, ks = lane >> 4;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;
    const int joff = PART8 ? 0 : p.n8;
    const int ng = p.ng, ngp = p.ngp;
    const int nquads = (ng + 3) / 4;
    const bool per_group_s8 = PART8 && !p.w8_per_channel;
    const int wq = WIN ? a.wq : nquads, nwin = WIN ? a.nwin : 1;   // chunk columns of a window, windows
    const int wql = nquads - (nwin - 1) * wq;                       // chunk columns of the last window
    const int xstride = (WIN ? wq * 4 * G : p.K) + A_PAD;

    // ---- the block's virtual tiles, the wave's chunks ----
    // Full rounds: virtual tile t of block b is packed tile b + nblk t, so that at any moment the
    // blocks together read one contiguous window of the weights (measured: 2 us faster on 64 MB
    // than giving every block a contiguous range of its own).  The tiles left over after the
    // last full round are dealt out in quarter tiles and make one more, partly filled, virtual tile.
    const int nblk = PART8 ? a.nblk8 : a.nblk4;
    const int b = (int)blockIdx.x - (PART8 ? 0 : a.nblk8);
    const int rounds = ntiles / nblk;
    const int left_base = 4 * rounds * nblk;                  // first left-over quarter tile
    const unsigned left = 4u * (unsigned)ntiles - (unsigned)left_base;   // < 4 nblk
    const int L_lo = (int)(left * (unsigned)b / (unsigned)nblk), L_hi = (int)(left * (unsigned)(b + 1) / (unsigned)nblk);   // L_hi - L_lo <= 4
    const int nvt = rounds + (L_hi > L_lo ? 1 : 0);   // >= 1: the host never launches more blocks than quarter tiles
    const int n = nvt * nquads;                       // chunks of the block
    auto share = [&](int chunks) { return wave < chunks ? (chunks - wave + NW - 1) / NW : 0; };
    const int cnt_w = WIN ? share(nvt * wq) : 0, cnt_l = WIN ? share(nvt * wql) : 0;   // this wave's chunks in a full window, in the last one
    const int n_my = WIN ? (nwin - 1) * cnt_w + cnt_l : share(n);
    auto vtile_of = [&](int j) { return nquads == 1 ? j : (int)__umulhi((unsigned)j, a.magic); };
    // chunk i of this wave's list: its virtual tile, its chunk column in K and (WIN) its window
    auto locate = [&](int i, int &vt, int &q, int &win) {
        if (!WIN) {
            const int j = wave + NW * i;
            vt = vtile_of(j);
            q = j - vt * nquads;
            win = 0;
        } else {
            win = 0;
            while (win < nwin - 1 && i >= cnt_w) {
                i -= cnt_w;
                ++win;
            }
            const int j = wave + NW * i;
            const bool lastw = win == nwin - 1;
            const int cols = lastw ? wql : wq;
            vt = cols == 1 ? j : (int)__umulhi((unsigned)j, lastw ? a.magic_l : a.magic_w);
            q = win * wq + (j - vt * cols);
        }
    };

    // ---- LDS ----
    float *wmax = (float *)smem;                                     // [NW] row maxima (built-in quantizer)
    uint32_t *tokmax = (uint32_t *)(smem + 64);                      // [16] row maxima as float bits (built-in quantizer, several tokens)
    float *red = (float *)(smem + LDS_HEADER);                       // [tcap][NW][NR][64]
    float *xsg = red + (size_t)a.tcap * NW * NR * 64;                // [M][ng] group scales of the activations
    int8_t *lds_x = (int8_t *)(xsg + (ACT_PT ? 0 : (p.M * ng + 3) / 4 * 4));

    const uint8_t *wpart = PART8 ? (const uint8_t *)p.w8 : p.w4;
    // Lane (c, ks) of virtual tile vt holds channel (c & 3) of the vt's quarter tile number c >> 2;
    // where the left-over virtual tile has fewer than four quarters its last one is read again
    // and the results are dropped.  Returns the lane's row in the part; base_tile = the packed
    // tile of the first quarter (the lane's own is that one or the next).
    auto lane_row = [&](int vt, int &base_tile, bool &valid) {
        const bool full = vt < rounds;
        const int u0 = full ? 4 * (b + nblk * vt) : left_base + L_lo;
        const int cnt = full ? 4 : L_hi - L_lo;
        valid = (c >> 2) < cnt;
        const int uc = u0 + min(c >> 2, cnt - 1);
        base_tile = u0 >> 2;
        return (uc >> 2) * TILE_N + 4 * (uc & 3) + (c & 3);
    };
    // request chunk i of this wave into k; past the end of the wave's list the same number of
    // loads is issued (the waits count them), all lanes reading the first bytes of the share
    auto issue = [&](int i, Slot<PART8> &k) {
        const bool real = i < n_my;
        int vt = 0, q = 0, win = 0;   // (a dummy request reads the first bytes of the share)
        if (real) locate(i, vt, q, win);
        const int g0 = 4 * q;
        const int last = ng - 1 - g0;   // at the ragged end of K the last group is re-read (its scale is forced to zero)
        int base_tile;
        bool valid;
        const int row = lane_row(vt, base_tile, valid);
        const int rel = real ? row - base_tile * TILE_N : 0;   // 0..31: the lane's row relative to the first packed tile
        const uint32_t w_voff = real ? (uint32_t)((rel >> 4) * ng * GB + ((rel & 15) + 16 * ks) * 16) : 0u;
        const uint8_t *wb = wpart + ((size_t)base_tile * ng + g0) * GB;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint8_t *wu = wb + (size_t)min(u, last) * GB;
            load_reg16_nt<0>(k.w[u][0], w_voff, wu);
            if (PART8) load_reg16_nt<1024>(k.w[u][PART8 ? 1 : 0], w_voff, wu);
        }
        k.s = make_uint2(0, 0);
        k.z = 0;
        if (!PART8) {
            if (!DUMP) load_reg8(k.s, (uint32_t)(rel * ngp * 2), p.s4 + ((size_t)base_tile * TILE_N * ngp + g0));
            load_reg_u16(k.z, (uint32_t)(rel * (ngp / 2)), p.z4 + ((size_t)base_tile * TILE_N * (ngp / 2) + g0 / 2));
        } else if (!DUMP) {
            if (per_group_s8) load_reg8(k.s, (uint32_t)(rel * ngp * 2), p.s8 + ((size_t)base_tile * TILE_N * ngp + g0));
            else load_reg_u16(k.z, (uint32_t)(rel * 2), p.s8 + (size_t)base_tile * TILE_N);
        }
    };

    // ---- 1. activations on their way, then the first weight requests ----
    v4i xv[MAXV];
    const int npiece = FUSED ? p.M * (p.K / 8) : p.M * (p.K / 16);   // 16-byte pieces of the activation matrix
    const void *xsrc = FUSED ? (const void *)p.x : (const void *)p.xq;
    // WIN: window win goes to buffer win & 1, row by row in pieces of 1 KB (one load instruction of
    // a wave: lane l writes 16 bytes at the piece's address + 16 l); the pieces of a window are dealt
    // round robin to the waves.  Lanes past the end of K read the row's last 16 bytes again, into
    // columns that no chunk reads.
    const int xbuf = p.M * xstride;
    auto request_window = [&](int win) {
        const int segs = ((win == nwin - 1 ? wql : wq) + 1) / 2;   // pieces per row
        const uint32_t dst0 = lds_address(lds_x) + (uint32_t)((win & 1) * xbuf);
        int row = 0, seg = wave;   // piece t = wave + NW k as (row, piece of the row)
        while (seg >= segs) {
            seg -= segs;
            ++row;
        }
        while (row < p.M) {
            const uint32_t col = (uint32_t)min(win * wq * 4 * G + seg * 1024 + lane * 16, p.K - 16);
            load_lds16(dst0 + (uint32_t)(row * xstride + seg * 1024), (uint32_t)row * (uint32_t)p.K + col, p.xq);
            seg += NW;
            while (seg >= segs) {
                seg -= segs;
                ++row;
            }
        }
    };
    if (WIN) {
        request_window(0);
    } else {
#pragma unroll
        for (int j = 0; j < MAXV; ++j)
            if (j * NT < npiece) load_reg16<0>(xv[j], (uint32_t)min(tid + NT * j, npiece - 1) * 16u, xsrc);
    }
    Slot<PART8> ring[R];
    sfor<0, E>([&](auto dc) { issue(decltype(dc)::value, ring[decltype(dc)::value]); });   // always E chunks, past the end of the list dummy ones (the staging waits count them)
    // the output channel and token scales of the first virtual tile this wave will finish:
    // requested now, needed at the very end
    int ch_first = -1;
    if (!DUMP && wave < nvt) {
        int bt;
        bool valid;
        const int row = lane_row(wave, bt, valid);
        if (valid && row < nrows) ch_first = p.perm[joff + row];
    }
    float xs_tok[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int m = NR == 1 ? ks : 4 * ks + r;
        xs_tok[r] = (!FUSED && !DUMP && ACT_PT) ? (float)p.xscale[min(m, p.M - 1)] : 1.0f;
    }
    // this wave's LDS cells start at zero
    for (int vt = 0; vt < nvt; ++vt)
#pragma unroll
        for (int r = 0; r < NR; ++r) red[((vt * NW + wave) * NR + r) * 64 + lane] = 0.0f;
    if (!ACT_PT && !DUMP && !FUSED)
        for (int i = tid; i < p.M * ng; i += NT) xsg[i] = (float)p.xscale[i];
    if (FUSED == 2 && ACT_PT) {
        if (tid < 16) tokmax[tid] = 0u;
        lds_barrier();   // while the activations are still on their way
    }
    if (WIN) {
        await_loads<E * NL>();               // the first window has landed (this wave's part of it)
        if (nwin > 1) request_window(1);     // (ahead of the chunk requests that follow, as at every change of window)
    }
#pragma unroll
    for (int j = 0; j < MAXV; ++j)
        if (!WIN && j * NT < npiece) await_vec<E * NL>(xv[j]);
    sfor<E, R>([&](auto dc) {   // the rest of the first R chunks, where the wave's list has them
        if (decltype(dc)::value < n_my) issue(decltype(dc)::value, ring[decltype(dc)::value]);
    });
    const int primed = max(min(R, n_my), E);   // chunk requests made so far (dummy ones included)

    // ---- 2. stage the activations ----
    if (FUSED && !ACT_PT) {
        // One scale per (token, group): the 16 lanes that hold a group of 128 values find its
        // maximum among themselves (K is a multiple of 128, so such a run of 16 pieces lies in
        // one token row and one group, and is loaded completely or not at all).
        const int per_row = p.K / 8;
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int i = tid + NT * j;
            if (j * NT < npiece) {
                const h8 hv = __builtin_bit_cast(h8, xv[j]);   // the whole register, after its wait
                float amax = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf((float)hv[e]));
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
                const float sc = (float)store_scale(amax / 127.0f);
                const float rc = recip(sc);
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w0 |= quant_code(hv[e], sc, rc) << (8 * e);
                    w1 |= quant_code(hv[4 + e], sc, rc) << (8 * e);
                }
                if (i < npiece) {
                    const int tok = i / per_row, pos = i - tok * per_row;
                    *(uint2 *)(lds_x + tok * xstride + pos * 8) = make_uint2(w0, w1);
                    if ((lane & 15) == 0) xsg[tok * ng + (pos >> 4)] = sc;
                }
            }
        }
    } else if (FUSED == 2) {
        // Several tokens.  K is a multiple of 512, so the 64 pieces of one load of a wave lie in
        // one token row: the wave reduces their maximum and one lane folds it into the row's
        // cell (non-negative floats order like their bit patterns).
        const int per_row = p.K / 8;
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int i0 = wave * 64 + NT * j;   // first piece of the wave's load j
            if (j * NT < npiece && i0 < npiece) {
                const h8 hv = __builtin_bit_cast(h8, xv[j]);   // the whole register, after its wait
                float amax = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf((float)hv[e]));
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
                if (lane == 0) atomicMax(&tokmax[i0 / per_row], __builtin_bit_cast(uint32_t, amax));
            }
        }
        lds_barrier();
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int i0 = wave * 64 + NT * j;
            if (j * NT < npiece && i0 < npiece) {
                const int tok = i0 / per_row, pos = i0 - tok * per_row + lane;
                const float sc = (float)store_scale(__builtin_bit_cast(float, tokmax[tok]) / 127.0f);
                const float rc = recip(sc);
                const h8 hv = __builtin_bit_cast(h8, xv[j]);
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w0 |= quant_code(hv[e], sc, rc) << (8 * e);
                    w1 |= quant_code(hv[4 + e], sc, rc) << (8 * e);
                }
                *(uint2 *)(lds_x + tok * xstride + pos * 8) = make_uint2(w0, w1);
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int m = min(NR == 1 ? ks : 4 * ks + r, p.M - 1);
            xs_tok[r] = (float)store_scale(__builtin_bit_cast(float, tokmax[m]) / 127.0f);
        }
    } else if (FUSED == 1) {
        // one token: row maximum over all threads, then the codes
        float amax = 0.0f;
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            if (j * NT < npiece && tid + NT * j < npiece) {
                const h8 hv = __builtin_bit_cast(h8, xv[j]);   // the whole register, after its wait
#pragma unroll
                for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf((float)hv[e]));
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
        if (lane == 0) wmax[wave] = amax;
        lds_barrier();
        float rowmax = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) rowmax = fmaxf(rowmax, wmax[w]);
        const float sc = (float)store_scale(rowmax / 127.0f);
        const float rc = recip(sc);
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int i = tid + NT * j;
            if (j * NT < npiece && i < npiece) {
                const h8 hv = __builtin_bit_cast(h8, xv[j]);   // the whole register, after its wait
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w0 |= quant_code(hv[e], sc, rc) << (8 * e);
                    w1 |= quant_code(hv[4 + e], sc, rc) << (8 * e);
                }
                *(uint2 *)(lds_x + i * 8) = make_uint2(w0, w1);
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) xs_tok[r] = sc;
    } else if (!WIN) {
        const int per_row = p.K / 16;
#pragma unroll
        for (int j = 0; j < MAXV; ++j) {
            const int i = tid + NT * j;
            if (j * NT < npiece && i < npiece) *(v4i *)(lds_x + (i / per_row) * xstride + (i % per_row) * 16) = xv[j];
        }
    }
    lds_barrier();

    // ---- 3. the wave's chunks ----
    const int tok_a = min(NR == 1 ? (c >> 2) : c, p.M - 1);   // token in row c of the A operand
    const int8_t *arow = lds_x + tok_a * xstride + ks * 16;
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    auto compute = [&](int i, const Slot<PART8> &k) {
        int vt, q, win;
        locate(i, vt, q, win);
        const int8_t *awin = arow + (WIN ? (win & 1) * xbuf - win * wq * 4 * G : 0);   // the window's buffer holds its columns only
        // The four fp16 scales are taken out of the two loaded dwords with integer operations
        // only: a reinterpreting copy of k.s makes the compiler keep k.s as 16-bit pieces, and
        // it then splits the dwords right after the load is issued, before the data is there.
        const float sh[4] = {half_bits_to_float(k.s.x & 0xffffu), half_bits_to_float(k.s.x >> 16),
                             half_bits_to_float(k.s.y & 0xffffu), half_bits_to_float(k.s.y >> 16)};
        const float sw_row = (PART8 && !DUMP) ? half_bits_to_float(k.z) : 0.0f;
        int ch = -1;
        if (DUMP) {
            int bt;
            bool valid;
            const int row = lane_row(vt, bt, valid);
            if (valid && row < nrows) ch = p.perm[joff + row];
        }
        float acc[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = 4 * q + u;
            const bool gvalid = g < ng;
            const int gc = min(g, ng - 1);
            const v4i a0 = *(const v4i *)(awin + gc * G), a1 = *(const v4i *)(awin + gc * G + 64);
            v4i P;
            float sw;
            if (PART8) {
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, k.w[u][0], v4i{0, 0, 0, 0}, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, k.w[u][PART8 ? 1 : 0], P, 0, 0, 0);
                sw = per_group_s8 ? sh[u] : sw_row;
            } else {
                const v4i w = k.w[u][0];
                const int m4 = 0x0F0F0F0F;
                const v4i b0 = {w[0] & m4, (int)((uint32_t)w[0] >> 4) & m4, w[1] & m4, (int)((uint32_t)w[1] >> 4) & m4};
                const v4i b1 = {w[2] & m4, (int)((uint32_t)w[2] >> 4) & m4, w[3] & m4, (int)((uint32_t)w[3] >> 4) & m4};
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, v4i{0, 0, 0, 0}, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, P, 0, 0, 0);
                v4i S = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, ones, v4i{0, 0, 0, 0}, 0, 0, 0);
                S = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, ones, S, 0, 0, 0);
                const int z = (int)((k.z >> (4 * u)) & 15);
                // |z| <= 15 and |sum a| <= 128 * 127: the 24-bit multiply is exact
#pragma unroll
                for (int r = 0; r < NR; ++r) P[r] -= __mul24(z, S[r]);
                sw = sh[u];
            }
            if (!gvalid) sw = 0.0f;   // a clamped re-read past the end of K contributes nothing
            if (DUMP) {
                if (gvalid && ch >= 0) {
#pragma unroll
                    for (int r = 0; r < NR; ++r) {
                        const int m = NR == 1 ? ks : 4 * ks + r;
                        if (m < p.M) p.P[((size_t)m * p.N + ch) * ng + g] = P[r];
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    float s = sw;
                    if (!ACT_PT) s *= xsg[min(NR == 1 ? ks : 4 * ks + r, p.M - 1) * ng + gc];
                    acc[r] = __builtin_fmaf((float)P[r], s, acc[r]);
                }
            }
        }
        if (!DUMP) {
#pragma unroll
            for (int r = 0; r < NR; ++r) red[((vt * NW + wave) * NR + r) * 64 + lane] += acc[r];
        }
    };
    // WIN: the window being read and the end of its chunks in this wave's list.  The window after it
    // was requested when this one became the present one.  When the wave comes to a chunk of a later
    // window (or to the end of its list) it waits for all of its loads - its part of the next window,
    // long landed, and the chunk it is about to consume; the request for the chunk after that is held
    // back until after the change - meets the other waves, who have then all finished with the
    // present window and landed their parts of the next, and requests the window after the next
    // into the buffer that has become free.  Those loads stand in the queue BEFORE the next chunk
    // request: a wait for that chunk then covers them at no cost (they come from L2 and were made
    // at the same time), whereas behind it every later wait would count them as younger loads and
    // the immediate counts of the waits would have to know how many there are.
    constexpr int XLMAX = 16;   // loads of a window per wave at most (16 rows of 8 KB in pieces of 1 KB over 8 waves)
    int win_now = 0, win_end = nwin == 1 ? cnt_l : cnt_w;
    auto next_window = [&]() {
        await_loads<0>();
        lds_barrier();
        ++win_now;
        win_end += win_now == nwin - 1 ? cnt_l : cnt_w;
        if (win_now + 1 < nwin) request_window(win_now + 1);
    };
    for (int i0 = 0; i0 < n_my; i0 += R) {
        sfor<0, R>([&](auto dc) {
            constexpr int d = decltype(dc)::value;
            const int i = i0 + d;
            if (i < n_my) {
                bool landed = false;   // (a change of window has waited for chunk i as well)
                if (WIN) {
                    while (i >= win_end) {   // (more than once where the wave has no chunk in a window)
                        next_window();
                        landed = true;
                    }
                }
                // The first `primed` chunks were requested at the start; from chunk R - 1 on, chunk
                // i + 1 is requested before chunk i is awaited, into the slot chunk i + 1 - R has
                // left.  Nothing is requested past the end of the list, so the last wait leaves
                // nothing in flight.
                if (i >= R - 1 && i + 1 < n_my) issue(i + 1, ring[(d + 1) % R]);
                const int younger = i < R - 1 ? primed - 1 - i : (i + 1 < n_my ? 1 : 0);   // chunks requested after chunk i
                if (!landed) {
                    sfor<0, R>([&](auto yc) {
                        constexpr int y = decltype(yc)::value;
                        if (younger == y) await_loads<y * NL>();
                    });
                }
                await_slot<(R - 1) * NL + (WIN ? XLMAX : 0)>(ring[d]);   // ties the registers to the wait above (its own wait is the weakest of them)
                compute(i, ring[d]);
            }
        });
    }
    if (WIN)
        while (win_now < nwin - 1) next_window();   // every wave passes every window's barrier
    // nothing may still be on its way into a register when the registers get other uses
    sfor<0, R>([&](auto dc) { await_slot<0>(ring[decltype(dc)::value]); });
    if (DUMP) return;
    lds_barrier();

    // ---- 4. the virtual tiles of the share: sum the waves' cells, token scale, fp16, scatter (Sec. 3.4) ----
    for (int vt = wave; vt < nvt; vt += NW) {
        int ch = ch_first;
        if (vt != wave) {
            int bt;
            bool valid;
            const int row = lane_row(vt, bt, valid);
            ch = (valid && row < nrows) ? p.perm[joff + row] : -1;
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) v += red[((vt * NW + w) * NR + r) * 64 + lane];
            const int m = NR == 1 ? ks : 4 * ks + r;
            if (m < p.M && ch >= 0) p.y[(size_t)m * p.N + ch] = (half_t)(v * xs_tok[r]);
        }
    }
}

template <int NR, bool DUMP, bool ACT_PT, int FUSED, bool WIN = false>
__global__ __launch_bounds__(NT) void linear_decode_split_kernel(LinearParams p, SplitArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    if ((int)blockIdx.x < a.nblk8)
        split_block<NR, DUMP, ACT_PT, true, FUSED, WIN>(p, a, smem);
    else
        split_block<NR, DUMP, ACT_PT, false, FUSED, WIN>(p, a, smem);
}

// ---- host side ------------------------------------------------------------------------------

struct Plan {
    int nblk8, nblk4, tcap, nr;
    int nwin, wq;   // windows over K and chunk columns per window (nwin = 1: the whole matrix is staged once)
    size_t lds_bytes;
};

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Blocks for the 8-bit and for the 4-bit quarter tiles (units8, units4 of them; an 8-bit one has
// twice the bytes), nb blocks in all: the split that makes the largest share smallest.
void split_blocks(int units8, int units4, int nb, int &nblk8, int &nblk4)
{
    if (units8 == 0 || units4 == 0) {
        nblk8 = std::min(units8, nb);
        nblk4 = std::min(units4, nb);
        return;
    }
    long best = -1;
    for (int b8 = 1; b8 < nb; ++b8) {
        const int n8 = std::min(b8, units8), n4 = std::min(nb - b8, units4);
        const long cost = std::max(2L * ceil_div(units8, n8), (long)ceil_div(units4, n4));
        if (best < 0 || cost < best) {
            best = cost;
            nblk8 = n8;
            nblk4 = n4;
        }
    }
}

bool compute_plan(const LinearParams &p, Plan &o)
{
    if (p.M < 1 || p.M > 16 || p.ng < 1) return false;
    const bool fused = p.x != nullptr;
    // fp16 activations: at most 4 loads per thread (16 Ki values); several tokens with one scale
    // per token need K = a multiple of 512.  Every block repeats the quantizer: measured on the
    // Llama-3-8B block, 16 Ki values cost as much as the stand-alone kernel they replace
    // (52.2 against 52.7 us per step at M = 4), 32 Ki values much more (68.0 against 57.7 at M = 8).
    if (fused && (p.P || (size_t)p.M * p.K > (size_t)NT * 8 * 4)) return false;
    if (fused && p.act_per_token && p.M > 1 && p.K % 512 != 0) return false;
    // int8 activations beyond 16 loads of 16 bytes per thread are staged window by window (built for
    // 5..16 tokens)
    const bool windows = !fused && (size_t)p.M * p.K > (size_t)NT * 16 * 16;
    if (windows && (p.M <= 4 || (size_t)p.M * p.K >= ((size_t)1 << 31))) return false;
    o.nr = p.M <= 4 ? 1 : 4;
    o.nwin = 1;
    const int nquads = (p.ng + 3) / 4;
    o.wq = nquads;
    const long long units8 = 4ll * p.ntiles8, units4 = 4ll * p.ntiles4;
    if (units8 + units4 == 0 || std::max(units8, units4) * MAX_BLOCKS >= (1ll << 31)) return false;
    const size_t scales = LDS_HEADER + (p.act_per_token ? 0 : ((size_t)p.M * p.ng + 3) / 4 * 16);
    if (windows) {
        // one block per CU; two buffers of the widest window (in chunk columns of 512 values) that fit
        // next to the cells - multiples of 8 keep the waves' shares of a window even
        const int nb = cu_count();
        int nblk8 = 0, nblk4 = 0;
        split_blocks((int)units8, (int)units4, nb, nblk8, nblk4);
        // virtual tiles of a block, exactly: the full rounds of whole tiles plus the one made of left-over
        // quarter tiles (every byte of LDS counts here: it decides the width of the windows)
        auto vtiles = [](int ntiles, int nblk) { return nblk ? ntiles / nblk + (ntiles % nblk ? 1 : 0) : 0; };
        const int tcap = std::max(1, std::max(vtiles(p.ntiles8, nblk8), vtiles(p.ntiles4, nblk4)));
        if ((long long)tcap * nquads * nquads >= (1ll << 31)) return false;
        for (int wq : {16, 12, 8, 4, 2}) {   // (even: a window's row is whole pieces of 1 KB, but for the end of K)
            const size_t lds = scales + 2 * (size_t)p.M * (wq * 4 * G + A_PAD) + (size_t)tcap * NW * o.nr * 256;
            if (lds > LDS_LIMIT) continue;
            o.nblk8 = nblk8;
            o.nblk4 = nblk4;
            o.tcap = tcap;
            o.wq = wq;
            o.nwin = ceil_div(nquads, wq);
            o.lds_bytes = lds;
            return o.nwin >= 2;   // (a matrix of more than 128 KB never fits one window)
        }
        return false;
    }
    const size_t fixed = scales + (size_t)p.M * (p.K + A_PAD);
    for (int nb = cu_count(); nb <= MAX_BLOCKS; nb *= 2) {
        // every block stages the whole activation matrix: with more than 64 KB of it, more than one
        // block per CU costs more than it gains (the kernel for a few dozen tokens takes those shapes)
        if (nb > cu_count() && fixed > 64 * 1024 + 4096) return false;
        int nblk8 = 0, nblk4 = 0;
        split_blocks((int)units8, (int)units4, nb, nblk8, nblk4);
        int share = 1;   // most quarter tiles in one block
        if (nblk8) share = std::max(share, ceil_div((int)units8, nblk8));
        if (nblk4) share = std::max(share, ceil_div((int)units4, nblk4));
        const int tcap = ceil_div(share, 4) + 1;   // full rounds plus the left-over virtual tile
        if ((long long)tcap * nquads * nquads >= (1ll << 31)) return false;   // chunk index / nquads by multiplication
        const size_t lds = fixed + (size_t)tcap * NW * o.nr * 256;
        if (lds <= LDS_LIMIT) {
            o.nblk8 = nblk8;
            o.nblk4 = nblk4;
            o.tcap = tcap;
            o.lds_bytes = lds;
            return true;
        }
    }
    return false;
}

// The plan depends on a handful of integers; a decoder block cycles through four shapes, so the
// last few plans are kept per thread.
bool make_plan(const LinearParams &p, Plan &o)
{
    struct Entry {
        int key[9];
        bool ok;
        Plan plan;
    };
    thread_local Entry cache[8];
    thread_local int used = 0, next = 0;
    int dev = 0;
    (void)hipGetDevice(&dev);
    const int key[9] = {p.M, p.K, p.ntiles8, p.ntiles4, p.act_per_token, p.x != nullptr, p.P != nullptr, p.ng, dev};
    for (int i = 0; i < used; ++i)
        if (std::equal(key, key + 9, cache[i].key)) {
            o = cache[i].plan;
            return cache[i].ok;
        }
    Entry &e = cache[next];
    next = (next + 1) % 8;
    used = std::min(used + 1, 8);
    std::copy(key, key + 9, e.key);
    e.plan = Plan{};
    e.ok = compute_plan(p, e.plan);
    o = e.plan;
    return e.ok;
}

template <int NR>
int launch_nr(const LinearParams &p, const SplitArgs &a, size_t lds_bytes, hipStream_t st)
{
    dim3 grid(a.nblk8 + a.nblk4), block(NT);
    auto go = [&](auto kernel) {
        if (lds_bytes > 48 * 1024)
            if (int e = ensure_dynamic_lds((const void *)kernel, lds_bytes)) return e;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, p, a);
        return (int)hipGetLastError();
    };
    if (a.nwin > 1) {   // activations staged window by window
        if constexpr (NR == 4) {
            if (p.P) return go(linear_decode_split_kernel<4, true, true, 0, true>);
            if (p.act_per_token) return go(linear_decode_split_kernel<4, false, true, 0, true>);
            return go(linear_decode_split_kernel<4, false, false, 0, true>);
        }
        return (int)hipErrorInvalidValue;
    }
    if (p.P) return go(linear_decode_split_kernel<NR, true, true, 0>);
    if (p.x && !p.act_per_token) return go(linear_decode_split_kernel<NR, false, false, 2>);
    if (p.x && p.M > 1) return go(linear_decode_split_kernel<NR, false, true, 2>);
    if (p.x) {
        if constexpr (NR == 1) return go(linear_decode_split_kernel<1, false, true, 1>);
        return (int)hipErrorInvalidValue;
    }
    if (p.act_per_token) return go(linear_decode_split_kernel<NR, false, true, 0>);
    return go(linear_decode_split_kernel<NR, false, false, 0>);
}

}  // namespace

bool decode_split_covers(const LinearParams &p)
{
    Plan pl;
    return make_plan(p, pl);
}

// the launch plan as six integers (blocks of the 8-bit part, of the 4-bit part, virtual tiles an
// LDS cell area covers, bytes of LDS, windows the activations are staged in, chunk columns - 512
// values of K - per window), for the host-side test of the work split
bool decode_split_plan(const LinearParams &p, int out[6])
{
    Plan pl;
    if (!make_plan(p, pl)) return false;
    out[0] = pl.nblk8;
    out[1] = pl.nblk4;
    out[2] = pl.tcap;
    out[3] = (int)pl.lds_bytes;
    out[4] = pl.nwin;
    out[5] = pl.wq;
    return true;
}

int launch_linear_decode_split(const LinearParams &p, hipStream_t st)
{
    Plan pl;
    if (!make_plan(p, pl)) return (int)hipErrorInvalidValue;
    SplitArgs a;
    a.nblk8 = pl.nblk8;
    a.nblk4 = pl.nblk4;
    const int nquads = (p.ng + 3) / 4;
    a.magic = nquads == 1 ? 0u : (uint32_t)(((1ull << 32) + nquads - 1) / nquads);
    a.tcap = pl.tcap;
    a.nwin = pl.nwin;
    a.wq = pl.wq;
    const int wql = nquads - (pl.nwin - 1) * pl.wq;
    a.magic_w = (uint32_t)(((1ull << 32) + pl.wq - 1) / pl.wq);   // (unused where a window has one chunk column)
    a.magic_l = (uint32_t)(((1ull << 32) + wql - 1) / wql);
    return pl.nr == 1 ? launch_nr<1>(p, a, pl.lds_bytes, st) : launch_nr<4>(p, a, pl.lds_bytes, st);
}

}  // namespace mixllm
