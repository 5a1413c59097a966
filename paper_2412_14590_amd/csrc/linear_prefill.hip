// Prefill path of the quantized linear (M > 16 tokens): int8-MFMA bound, with the vector
// ALU (unpack + float rescale) as the ceiling right beneath it.
//
// A block of WM x WN waves computes a (WM*TM*32) x (WN*32) tile of y with
// v_mfma_i32_32x32x32_i8; a wave owns TM token tiles of 32 x 32 for one 32-channel tile.
//  * Activations (A operand, rows = tokens) go HBM/L2 -> LDS directly (16-byte
//    global_load_lds, no registers), one quantization group (128 k) per stage, four stages.
//    Rows are 128 bytes; the 16-byte chunk c of row r sits at chunk position c ^ ((r >> 1) & 7),
//    so that the fragment reads of 16 consecutive lanes cover all 64 banks exactly once.
//  * Packed weights (B operand, columns = channels) go L2 -> registers directly in the same
//    packed layout the decode path streams: two 16-byte loads per lane fetch one group of a
//    32-channel tile of 4-bit weights (requested one or two groups ahead), four one of 8-bit
//    weights (three groups ahead, straight into a ring of operand registers).  No weight byte
//    passes through LDS.
//  * uint4 -> int8 unpack with zero-point subtraction in registers (step 1 of the two-step
//    dequantization, Sec. 3.3), once per group per wave, reused by the TM token tiles; the
//    unpack of group g+1 is spread over the second half of group g's MFMAs.
//  * Per group and tile: 4 chained MFMAs (K = 128) from a literal-zero accumulator into int32,
//    then int->float and one FMA per element with the group scale (step 2, Sec. 3.3).  The
//    channel a lane owns is the MFMA column, so the group scale is one register per lane.
//  * Issue order.  A group is TM*4 MFMA slots.  Tiles are processed in pairs (two independent
//    accumulation chains, alternating); the float rescale of the PREVIOUS pair runs in the
//    shadow of the current pair's MFMAs (8 vector instructions per MFMA is what the vector port
//    sustains at full MFMA rate), and the A fragment of slot s+6 (s+4 with two token tiles per
//    wave) is requested at slot s (LDS latency is several MFMAs long).  The pipeline runs across group boundaries; the only
//    block-wide barrier sits in the middle of a group (slot TM*2), where the next group's
//    activations are known to have landed and the stage of the previous group is released.
//  * Group metadata (4 fp16 scales, 4 zero points) is fetched once per 4 groups.
//  * Epilogue: token scale (all of a lane's scales requested by hand in one batch), fp16
//    conversion, scatter to the original channel (Sec. 3.4).
// 8-bit and 4-bit channel tiles are different block ranges of one launch; where the grid of output
// tiles is short and K long, K is split over blocks and a second kernel adds the parts.
#include <algorithm>
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "internal.h"
#include "async_loads.h"

namespace mixllm {

constexpr int NSTAGE = 4;   // LDS stages of the activation tile (one group each)
// Launch constants, each settable at build time for measurements (the values are the measured best):
// groups between the request for packed 4-bit weights and the wait for them, by block shape.  Two
// and three groups ahead measure within 2 % of each other on every Llama-shaped layer from 64 to
// 2048 tokens (the wait in the middle of a group is bound by the activations, which run two groups
// ahead, not by the weights).
#ifndef MIXLLM_PREFILL_WD_SMALL
#define MIXLLM_PREFILL_WD_SMALL 2   // 32 x 128 and 64 x 128 blocks
#endif
#ifndef MIXLLM_PREFILL_WD_LARGE
#define MIXLLM_PREFILL_WD_LARGE 1   // 128 x 128 blocks
#endif
// groups an 8-bit tile requests its weights ahead of their use (1 or 3)
#ifndef MIXLLM_PREFILL_L8
#define MIXLLM_PREFILL_L8 3
#endif
// 1: in a launch of 128 x 128 blocks that is at most MIXLLM_PREFILL_HALF8_ROUNDS rounds of blocks long,
// the 8-bit part runs in blocks of 64 x 128 (0: never).  Measured at 2048 tokens, same machine, equal
// against half-height 8-bit tiles: K = N = 4096 56.2 -> 51.5 us, K = 14336, N = 4096 164.5 -> 157.6,
// K = 4096, N = 6144 75.4 -> 76.0; at 4096 tokens (two to three rounds) 101.5 -> 98, 302 -> 297 and
// 149 -> 143 us; the layer of N = 28672 gains 2 % at 1024 tokens (3.5 rounds), nothing at 2048 (seven:
// 313 -> 324 us in one session, 330 -> 328 in another) and loses 1 % at 4096, which is why long launches
// keep the full tiles; blocks of 32 x 128 for the 8-bit part of a 64 x 128 launch measured 4-7 % slower.
#ifndef MIXLLM_PREFILL_HALF8
#define MIXLLM_PREFILL_HALF8 1
#endif
// token tiles per band of the block order: 4, 8 and 16 measure within 2 % of each other
#ifndef MIXLLM_PREFILL_BAND
#define MIXLLM_PREFILL_BAND 4
#endif
// waves (32 channels each) of the block with 128 token rows.  With 8 (blocks of 128 x 256, one per
// CU, half the activation traffic through the L2s) the gate+up layer at 2048 tokens takes 5 % longer
// (336 against 319 us) and the layers of N <= 6144 10-20 % longer (fewer, coarser blocks): the
// kernel is not bound by its L2 traffic.
#ifndef MIXLLM_PREFILL_WN_LARGE
#define MIXLLM_PREFILL_WN_LARGE 4
#endif

// Measurement builds only (-DMIXLLM_STAMPS): thread 0 of every block records the constant 100 MHz
// clock at a few points of its life into a caller-supplied array [blocks][8].
#ifdef MIXLLM_STAMPS
__device__ unsigned long long *g_stamps;
#define MIXLLM_STAMP(i)                                                                          \
    do {                                                                                         \
        if constexpr (DUMP == 0) {   /* the linear only; used where a template parameter DUMP is in scope */ \
            unsigned long long t_;                                                               \
            asm volatile("s_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t_)::"memory");       \
            unsigned long long *sp_ = g_stamps;                                                  \
            if (sp_ && threadIdx.x == 0) sp_[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 8 + (i)] = t_; \
        }                                                                                        \
    } while (0)
#else
#define MIXLLM_STAMP(i)
#endif

// compile-time loop: f(std::integral_constant<int, I>) for I in [I, N)
template <int I, int N, typename F>
static __device__ inline void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int WM_, int WN_, int TM_, int WD_>
struct Shape {
    static constexpr int WM = WM_, WN = WN_, TM = TM_;
    static constexpr int NW = WM * WN;
    static constexpr int THREADS = 64 * NW;
    static constexpr int BM = WM * TM * 32;       // tokens per block
    static constexpr int BN = WN * 32;            // channels per block
    static constexpr int A_STAGE = BM * G;        // bytes of one LDS stage
    static constexpr int LPW = BM / 8 / NW;       // direct-to-LDS loads (8 rows each) per wave and stage
    // An A fragment is requested DFRAG MFMA slots before its use (LDS latency under load is several
    // MFMAs).  Requests for the next group's stage must come after the barrier in the middle of the
    // group (slot 2 TM), which is what tells a wave that the stage has landed for every wave.
    static constexpr int DFRAG = TM >= 4 ? 6 : 2 * TM;
    static constexpr int RING = TM >= 2 ? 8 : 4;  // fragment registers (at least DFRAG + 2: the slot being overwritten is two MFMAs old)
    static constexpr int NB = TM >= 2 ? 2 : 1;    // token tiles whose MFMA chains alternate (a bundle)
    // the shape the 8-bit part of a short launch runs in: half the token rows (see linear_prefill_kernel)
    using Half = Shape<WM_, WN_, (TM_ == 4 && MIXLLM_PREFILL_HALF8 ? 2 : TM_), WD_>;
    static constexpr int WD = WD_;                // groups between the request for packed 4-bit weights and the wait for them
    static constexpr int L8 = MIXLLM_PREFILL_L8;  // groups between the request for 8-bit weights and their use
    static_assert(TM * 4 - DFRAG >= TM * 2 && DFRAG + 2 <= RING, "fragment requests must not pass the barrier or wrap the ring");
    static_assert(BM % (8 * NW) == 0, "A tile must split evenly over the waves");
    static_assert(TM % NB == 0 && (TM * 4) % RING == 0, "whole bundles of token tiles; slots wrap the fragment ring");
    static_assert((NSTAGE - 1) * A_STAGE + (TM * WM - 1) * 32 * G + 31 * G + 127 < 65536, "LDS offsets must fit 16 bits");
};

// ASYNC: packed weights and metadata are fetched with the hand-issued loads above.  Only valid in a
// kernel that keeps everything in registers: a register spilled between its load and its
// await_loads() would be saved before the data has arrived.  (The build checks that the kernels
// instantiated with ASYNC use no scratch memory.)  Without ASYNC they are ordinary loads, which
// the compiler awaits itself - later than necessary, because it does not see the hand-issued
// activation loads ahead of them in the queue, but always correctly.
// DUMP: 0 = the linear; 1 = debug entry point, the int32 partial of every (token, channel, group)
// leaves the loop instead of being rescaled (no scales are passed, none are loaded); 2 = debug
// entry point, the partials are added up in int32 over the groups instead of being rescaled:
// same arguments, loads, waits, unpack and MFMAs as the linear.
template <typename C, int DUMP, bool ACT_PT, bool PART8, bool PG8, bool ASYNC>
static __device__ inline void prefill_block(const LinearParams &p, int m0, int t16_0, int g_lo, int g_hi, int kp, uint8_t *lds_a,
                                            float *lds_sa)
{
    // The block walks the quantization groups g_lo .. g_hi - 1 (all of K, or - K split over kparts
    // blocks - part kp of it; g_lo is a multiple of 4, and so is g_hi unless it is the last group).
    constexpr int TM = C::TM, WN = C::WN, BM = C::BM, A_STAGE = C::A_STAGE, LPW = C::LPW, DFRAG = C::DFRAG, RING = C::RING;
    constexpr int NSLOT = TM * 4;            // MFMAs per group
    constexpr int NB = C::NB, SB = 4 * NB;   // tiles and MFMA slots of a bundle
    constexpr int NBG = TM / NB;             // bundles per group
    constexpr int HALF = NSLOT / 2;          // slot of the barrier
    constexpr int PPS = 8 / (NSLOT - HALF);  // eighths of the next group's unpack per slot of the second half
    static_assert(PPS * (NSLOT - HALF) == 8, "the unpack is spread evenly over the second half of the group");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = C::WM == 1 ? 0 : wave / WN, wn = wave % WN;
    const int n32 = lane & 31, h = lane >> 5;
    const int ntiles = PART8 ? p.ntiles8 : p.ntiles4;
    const int nrows = PART8 ? p.n8 : p.n4;
    const int joff = PART8 ? 0 : p.n8;
    const int ng = p.ng;
    const int mw0 = wm * TM * 32;   // first row of this wave inside the block tile
    constexpr bool per_group_s8 = PART8 && PG8;   // 8-bit tile with one weight scale per group

    // this lane's channel
    const int t16 = t16_0 + wn * 2 + (n32 >> 4);
    const int tile16 = min(t16, ntiles - 1);
    const int rw = tile16 * TILE_N + (n32 & 15);
    const int ch = (t16 < ntiles && rw < nrows) ? p.perm[joff + rw] : -1;

    // ---- loaders -------------------------------------------------------------------
    // Activation tile of one group, straight to LDS.  Load i of this wave fills rows
    // 8*(wave*LPW+i) .. +7: lane l writes chunk position l&7 of row +(l>>3), which holds the
    // global chunk (l&7) ^ ((row>>1)&7).  Rows past M re-read row M-1: token rows are
    // independent, and outputs of rows >= M are never stored.
    uint32_t a_voff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave * LPW + i) * 8 + (lane >> 3);
        const int cs = (lane & 7) ^ ((row >> 1) & 7);
        a_voff[i] = (uint32_t)min(m0 + row, p.M - 1) * (uint32_t)p.K + cs * 16;
    }
    const uint32_t lds_a_wave = __builtin_amdgcn_readfirstlane(lds_address(lds_a) + wave * LPW * 1024);
    auto load_a = [&](int g, int stage) {
        const int8_t *src = p.xq + (size_t)min(g, g_hi - 1) * G;
#pragma unroll
        for (int i = 0; i < LPW; ++i) load_lds16(lds_a_wave + stage * A_STAGE + i * 1024, a_voff[i], src);
    };
    // fragment read offsets: row mw0 + 32 mt + n32, global chunk 2j + h
    int a_rd[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a_rd[j] = (mw0 + n32) * G + (((2 * j + h) ^ ((n32 >> 1) & 7)) << 4);

    // weights of one group for the wave's 32-channel tile
    //  4-bit: raw[0] = 16-k chunks h and 4+h, raw[1] = chunks 2+h and 6+h (packed nibbles)
    //  8-bit: b[j] = chunk 2j+h (int8), loaded straight into the operand registers
    // (byte offsets of a lane inside the weight and metadata arrays fit 32 bits: checked on the host)
    const uint32_t b_voff = PART8 ? ((uint32_t)tile16 * (uint32_t)(p.K / 64) * 64 + (n32 & 15) + 16 * h) * 16
                                  : ((uint32_t)tile16 * (uint32_t)ng * 64 + (n32 & 15) + 16 * h) * 16;
    // Operand sets.  Unpacked 4-bit groups alternate between two.  8-bit groups are loaded straight
    // into them, L8 groups ahead, and then need L8 + 1 sets: with one group ahead a launch whose
    // weights come from HBM spends 0.6 us per group waiting for them whatever the tile does
    // (K = N = 4096 with 10 % 8-bit channels: 19.4 us from 17 to 256 tokens, 14 us without the
    // 8-bit tiles); three groups ahead cover that latency.
    // (The debug variant that adds the partials up as integers under per-group activation scales has
    // no registers left for the ring and keeps one group of look-ahead.)
    constexpr int L8 = (DUMP == 2 && !ACT_PT) ? 1 : C::L8, NBUF = PART8 ? L8 + 1 : 2;
    static_assert(NBUF == 2 || NBUF == 4, "operand sets are indexed by the group number modulo 4");
    v4i b[NBUF][4];
    // packed 4-bit weights are requested WD groups before the wait for them (hand-issued loads
    // only: with ordinary loads the wait below cannot count what is younger in the queue)
    // Raw (packed) weights of groups g + 1 .. g + 1 + WD are live at the middle of group g: WD + 1
    // ring slots; the slot index is g modulo the ring size, known at compile time only modulo 4
    // (the K loop is unrolled four groups deep), so the ring has 2 or 4 slots and WD is at most 3.
    constexpr int WD = ASYNC ? C::WD : 1, NRAW = WD == 1 ? 2 : 4;
    static_assert(WD >= 1 && WD <= 3, "weight requests run one to three groups ahead");
    constexpr int NMETA = DUMP == 1 ? 1 : 2;   // load instructions load_meta issues for a 4-bit tile in the hand-issued variant
    v4i raw[NRAW][2];
    auto load_b = [&](int g, auto setc) {
        constexpr int set = decltype(setc)::value % NBUF, rset = decltype(setc)::value % NRAW;
        const int gc = min(g, g_hi - 1);
        if (PART8) {
            const uint8_t *base = (const uint8_t *)p.w8 + (size_t)gc * 2048;
            if (ASYNC) {
                load_reg16<0>(b[set][0], b_voff, base);
                load_reg16<512>(b[set][1], b_voff, base);
                load_reg16<1024>(b[set][2], b_voff, base);
                load_reg16<1536>(b[set][3], b_voff, base);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) b[set][j] = *(const v4i *)(base + b_voff + j * 512);
            }
        } else {
            const uint8_t *base = p.w4 + (size_t)gc * 1024;
            if (ASYNC) {
                load_reg16<0>(raw[rset][0], b_voff, base);
                load_reg16<512>(raw[rset][1], b_voff, base);
            } else {
                raw[rset][0] = *(const v4i *)(base + b_voff);
                raw[rset][1] = *(const v4i *)(base + b_voff + 512);
            }
        }
    };
    // metadata of 4 consecutive groups (arrays are zero padded to a multiple of 8 groups)
    struct Meta {
        uint2 s;       // 4 fp16 group scales
        uint32_t z;    // 4 uint4 zero points in the low 16 bits
    };
    const uint32_t s_voff = (uint32_t)rw * (uint32_t)p.ngp * 2, z_voff = (uint32_t)rw * (uint32_t)(p.ngp / 2);
    auto load_meta = [&](int q, Meta &mt) {
        mt.s = make_uint2(0, 0);
        mt.z = 0;
        const int g0 = 4 * min(q, (g_hi - 1) / 4);
        if (ASYNC) {
            if (PART8) {
                if (DUMP != 1 && per_group_s8) load_reg8(mt.s, s_voff, p.s8 + g0);
            } else {
                if (DUMP != 1) load_reg8(mt.s, s_voff, p.s4 + g0);
                load_reg_u16(mt.z, z_voff, p.z4 + g0 / 2);
            }
        } else {
            if (PART8) {
                if (DUMP != 1 && per_group_s8) mt.s = *(const uint2 *)((const uint8_t *)(p.s8 + g0) + s_voff);
            } else {
                if (DUMP != 1) mt.s = *(const uint2 *)((const uint8_t *)(p.s4 + g0) + s_voff);
                mt.z = *(const uint16_t *)(p.z4 + g0 / 2 + z_voff);
            }
        }
    };
    auto scale_of = [&](const Meta &mt, int u) -> float {   // integer operations only, see half_bits_to_float
        const uint32_t d = (u & 2) ? mt.s.y : mt.s.x;
        return half_bits_to_float((u & 1) ? d >> 16 : d & 0xffffu);
    };
    // one eighth of the unpack of a group: raw dword d of `set` -> two operand dwords
    // (`keep`, DUMP == 2 only: all bits set, or zero for a group past the end of K, whose weights
    // then unpack to zeros - together with a zero point of zero - where the linear multiplies the
    // group's partial by a zero scale)
    auto unpack_piece = [&](auto setc, auto dc, uint32_t zb, uint32_t keep) {
        constexpr int set = decltype(setc)::value % NBUF, rset = decltype(setc)::value % NRAW, d = decltype(dc)::value;
        constexpr int bj = d >> 1, e = d & 1;
        int lo, hi;
        uint32_t w = (uint32_t)raw[rset][bj & 1][(bj >> 1) * 2 + e];
        if (DUMP == 2) w &= keep;
        unpack_sub(w, zb, lo, hi);
        b[set][bj][2 * e] = lo;
        b[set][bj][2 * e + 1] = hi;
    };

    v16i zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0;

    float acc[TM][16];
    int isum[TM][16];   // DUMP == 2: the partials added up as integers
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc[mt][r] = 0.0f;
            isum[mt][r] = 0;
        }

    // Rescale (or, for the debug entry point, dump) registers 4j..4j+3 of one finished tile:
    // rows m0 + mw0 + 32 mt + 8 j + 4 h + {0..3}, column = this lane's channel.
    // `opaque0` (DUMP == 1) is a zero the compiler cannot see through: with it the store addresses
    // are computed where they are used instead of all 16 TM of them being kept in registers across
    // the K loop.
    auto finish4 = [&](const v16i &P, auto mtc, auto jc, float sw, int gp, int opaque0) {
        constexpr int mt = decltype(mtc)::value, j = decltype(jc)::value;
        if (DUMP == 1) {
            if (gp >= 0 && gp < ng && ch >= 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = m0 + mw0 + mt * 32 + 8 * j + 4 * h + i + opaque0;
                    if (m < p.M) p.P[((size_t)m * p.N + ch) * ng + gp] = P[4 * j + i];
                }
            }
        } else if (DUMP == 2) {
            // (a group past the end of K, which the linear multiplies by a zero scale, has had its
            // weights replaced by zeros: see group_step)
#pragma unroll
            for (int i = 0; i < 4; ++i) isum[mt][4 * j + i] += P[4 * j + i];
        } else if (ACT_PT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[mt][4 * j + i] = __builtin_fmaf((float)P[4 * j + i], sw, acc[mt][4 * j + i]);
        } else {
            // per-(token, group) activation scales of the tile's group, staged in LDS
            // (The offset goes through an empty asm statement so that the read stays in this MFMA
            // slot: the compiler otherwise gathers the reads of half a group at its start and runs
            // out of registers holding them.)
            uint32_t sa_off = (uint32_t)((((gp + NSTAGE) % NSTAGE) * BM + mw0 + mt * 32 + 8 * j + 4 * h) * sizeof(float));
            asm volatile("" : "+v"(sa_off));
            const v4f sa = *(const v4f *)((const uint8_t *)lds_sa + sa_off);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[mt][4 * j + i] = __builtin_fmaf((float)P[4 * j + i], sw * sa[i], acc[mt][4 * j + i]);
        }
    };

    // ---- prologue ------------------------------------------------------------------
    Meta meta_cur, meta_nxt;
    load_meta(g_lo / 4, meta_cur);
    load_b(g_lo, std::integral_constant<int, 0>{});
    if (!PART8) static_for<1, WD + 1>([&](auto gc) { load_b(g_lo + decltype(gc)::value, gc); });
    else static_for<1, L8>([&](auto gc) { load_b(g_lo + decltype(gc)::value, gc); });
    load_a(g_lo, 0);
    load_a(g_lo + 1, 1);
    load_a(g_lo + 2, 2);
    // Activation scale (fp16 bits) of (token row tid, group g+1) on its way to LDS: every thread
    // requests one (rows past the tile re-read its last row), so that all waves count the same loads.
    uint32_t sa_bits = 0;
    const uint32_t sa_voff = (uint32_t)min(m0 + min(tid, BM - 1), p.M - 1) * (uint32_t)ng * 2u;
    const uint32_t lds_sa_thread = lds_address(lds_sa) + (uint32_t)min(tid, BM - 1) * (uint32_t)sizeof(float);   // this thread's cell of stage 0
    if (!ACT_PT && DUMP != 1) {
        if (tid < BM) {
#pragma unroll
            for (int s = 1; s < NSTAGE; ++s) lds_sa[s * BM + tid] = 0.0f;   // read (times a zero scale) before first written
            lds_sa[tid] = (float)p.xscale[(size_t)min(m0 + tid, p.M - 1) * ng + g_lo];
        }
        load_reg_u16(sa_bits, sa_voff, p.xscale + min(g_lo + 1, g_hi - 1));
    }
    const float sw_row = (PART8 && DUMP != 1 && !PG8) ? (float)p.s8[rw] : 0.0f;
    // Token scales of the epilogue (one per token): all 16 TM of a lane are requested together, by
    // hand, ahead of the epilogue - in the prologue where the registers allow it (the epilogue of a
    // short launch otherwise pays a round trip to memory for them), else after the K loop and its
    // drain: one round trip for all of them.  (Written as plain loads inside the
    // epilogue they cost one round trip per token tile: the compiler does not move the next
    // tile's loads above the stores of the previous one.)
    constexpr bool HAND_SA = ACT_PT && DUMP == 0, EARLY_SA = HAND_SA && TM <= 2;
    uint32_t sa_ep[HAND_SA ? TM : 1][16];
    auto request_token_scales = [&]() {
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                load_reg_u16(sa_ep[mt][r], (uint32_t)min(m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3), p.M - 1) * 2u, p.xscale);
    };
    auto await_token_scales = [&]() {
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) await_loads<0>(sa_ep[mt][r]);
    };
    if constexpr (EARLY_SA) request_token_scales();
    // everything above has landed (registers and LDS)
    if constexpr (EARLY_SA) await_token_scales();
    await_loads<0>(meta_cur.s, meta_cur.z);
    await_loads<0>(sa_bits);
    if constexpr (PART8)
        static_for<0, L8>([&](auto sc) { await_loads<0>(b[decltype(sc)::value][0], b[decltype(sc)::value][1], b[decltype(sc)::value][2], b[decltype(sc)::value][3]); });
    else
        static_for<0, NRAW>([&](auto rc) { await_loads<0>(raw[decltype(rc)::value][0], raw[decltype(rc)::value][1]); });
    __syncthreads();
    MIXLLM_STAMP(1);
    meta_nxt = meta_cur;
    if (!PART8) {
        const uint32_t zb = zbias(meta_cur.z & 15);
        static_for<0, 8>([&](auto dc) { unpack_piece(std::integral_constant<int, 0>{}, dc, zb, 0xffffffffu); });
    }
    v4i af[RING];
    // fragment of slot t of the group held in `stage`
    auto load_frag = [&](auto stagec, auto tc) {
        constexpr int stage = decltype(stagec)::value, t = decltype(tc)::value;
        constexpr int mt = NB * (t / SB) + t % NB, j = (t % SB) / NB;
        af[t % RING] = *(const v4i *)(lds_a + a_rd[j] + stage * A_STAGE + mt * 32 * G);
    };
    static_for<0, DFRAG>([&](auto tc) { load_frag(std::integral_constant<int, 0>{}, tc); });

    // int32 accumulators of the bundle in flight (P[s]) and of the bundle being rescaled (P[s^1])
    v16i P[2][NB];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < NB; ++i) P[s][i] = zero16;
    float sw_prev = 0.0f;   // group scale of the bundle left over from the previous group

    // one group; U = g & 3 selects the register sets and the LDS stage at compile time
    auto group_step = [&](int g, auto uc) {
        constexpr int U = decltype(uc)::value;
        float sw_cur;
        if (PART8 && !per_group_s8) sw_cur = g < g_hi ? sw_row : 0.0f;
        else sw_cur = scale_of(meta_cur, U);   // zero for groups past the end (padding)
        int opaque0 = 0;
        if (DUMP == 1) asm volatile("s_mov_b32 %0, 0" : "=s"(opaque0));
        uint32_t zb_next = 0;
        const uint32_t keep_next = g + 1 < g_hi ? 0xffffffffu : 0u;
        // 8-bit weights need no unpack: group g + L8 is requested here, straight into the operand
        // registers group g-1 just vacated; this group's own request has to have landed.  It is L8
        // groups old: issued after it were the activation loads of L8 middles and the weights of
        // L8 - 1 groups (metadata and activation-scale requests of those middles are not counted:
        // the wait then asks for a few loads more than it needs, all of them older than two groups).
        if (PART8) {
            await_loads<L8 * LPW + 4 * (L8 - 1)>(b[U % NBUF][0], b[U % NBUF][1], b[U % NBUF][2], b[U % NBUF][3]);
            load_b(g + L8, std::integral_constant<int, U + L8>{});
            if (DUMP == 2 && g >= g_hi) {
#pragma unroll
                for (int j = 0; j < 4; ++j) b[U % NBUF][j] = v4i{0, 0, 0, 0};
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        static_for<0, NSLOT>([&](auto stc) {
            constexpr int st = decltype(stc)::value, q = st / SB, j = (st % SB) / NB, i = st % NB;
            constexpr int s = (U * NBG + q) & 1;                   // bundles alternate between the two accumulator sets, across groups too
            constexpr int mt = NB * q + i;
            constexpr int qp = (q + NBG - 1) % NBG;                // bundle being rescaled
            constexpr int up = NB * qp + i;                        // ... its tile handled in this slot
            const int gp = q == 0 ? g - 1 : g;                     // ... and its group
            if constexpr (st == HALF) {
                // Middle of the group.  The wait leaves at most the LPW youngest loads in flight:
                // the direct-to-LDS loads of the previous middle (activations of group g+2), which
                // are issued last in their batch.  Everything older has landed: this wave's part
                // of group g+1's activations, group g+1's packed weights and the metadata.  After
                // the barrier group g+1's activations are in LDS for every wave, and every wave is
                // done reading the stage of group g-1, which the next request overwrites.
                // (With WD = 2 the batch of the previous middle stays in flight as a whole: group
                // g+2's packed weights, in front of them the metadata request if that middle made
                // one, and the activations of group g+2.)
                // A batch is issued in the order metadata, activation scale, packed weights,
                // activations; the scale request of the previous middle (group g+1's) is older than
                // that middle's weights and activations, so with per-group activation scales the
                // WD = 2 wait does not count a metadata request as young.  An 8-bit tile requests
                // its weights at the start of a group: issued after group g+1's activations (two
                // middles ago) were the weights of two groups and the previous middle's activations;
                // with per-group activation scales the previous middle's scale request has to have
                // landed as well, and with it the older of those two weight requests.
                // (WD >= 2: the wait is bound by group g+1's activations, requested two middles ago,
                // so the whole batch of the previous middle may stay in flight, however far ahead
                // the weights run)
                constexpr int YOUNGER = PART8 ? ((!ACT_PT && DUMP != 1) || L8 == 1 ? LPW + 4 : LPW + 8) : WD == 1 ? LPW : (U == 2 && ACT_PT ? NMETA : 0) + 2 + LPW;
                if (PART8) await_loads<YOUNGER>();
                else await_loads<YOUNGER>(raw[(U + 1) % NRAW][0], raw[(U + 1) % NRAW][1]);
                if constexpr (U == 3) await_loads<YOUNGER>(meta_nxt.s, meta_nxt.z);
                if (!ACT_PT && DUMP != 1) {
                    await_loads<YOUNGER>(sa_bits);
                    // every thread stores (threads past the tile repeat its last row's value): no
                    // branch in the middle of the group, and a store the compiler does not have to
                    // order against the fragment reads it has in flight
                    const float sa_val = half_bits_to_float(sa_bits);
                    asm volatile("ds_write_b32 %0, %1" ::"v"(lds_sa_thread + (uint32_t)(((U + 1) % NSTAGE) * BM * sizeof(float))), "v"(sa_val) : "memory");
                }
                mid_group_barrier<(!ACT_PT && DUMP != 1)>();
                if constexpr (U == 1) load_meta(g / 4 + 1, meta_nxt);
                if (!ACT_PT && DUMP != 1) load_reg_u16(sa_bits, sa_voff, p.xscale + min(g + 2, g_hi - 1));
                if (!PART8) load_b(g + 1 + WD, std::integral_constant<int, U + 1 + WD>{});
                load_a(g + 3, (U + 3) % NSTAGE);
                if (!PART8) zb_next = zbias(((U == 3 ? meta_nxt.z : meta_cur.z) >> (4 * ((U + 1) % 4))) & 15);
                if (!PART8 && DUMP == 2 && !keep_next) zb_next = 0x80808080u;
                __builtin_amdgcn_sched_barrier(0);
            }
            // request the fragment DFRAG slots ahead (second half: from the next group's stage)
            if constexpr (st + DFRAG < NSLOT)
                load_frag(std::integral_constant<int, U>{}, std::integral_constant<int, st + DFRAG>{});
            else
                load_frag(std::integral_constant<int, (U + 1) % NSTAGE>{}, std::integral_constant<int, st + DFRAG - NSLOT>{});
            P[s][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[st % RING], b[U % NBUF][j], j == 0 ? zero16 : P[s][i], 0, 0, 0);
            finish4(P[s ^ 1][i], std::integral_constant<int, up>{}, std::integral_constant<int, j>{},
                    q == 0 ? sw_prev : sw_cur, gp, opaque0);
            if constexpr (!PART8 && st >= HALF) {
                static_for<0, PPS>([&](auto ec) {
                    unpack_piece(std::integral_constant<int, U + 1>{},
                                 std::integral_constant<int, PPS * (st - HALF) + decltype(ec)::value>{}, zb_next, keep_next);
                });
            }
            if (DUMP != 1) {
                // issue order: MFMA, the LDS read(s), the vector instructions in its shadow
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, ACT_PT ? 1 : 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, ACT_PT ? 16 : 20, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        sw_prev = sw_cur;
    };
    for (int g = g_lo; g < g_hi; g += 4) {
        group_step(g, std::integral_constant<int, 0>{});
        group_step(g + 1, std::integral_constant<int, 1>{});
        group_step(g + 2, std::integral_constant<int, 2>{});
        group_step(g + 3, std::integral_constant<int, 3>{});
        meta_cur = meta_nxt;
    }
    MIXLLM_STAMP(2);
    const int g_last = g_lo + ((g_hi - g_lo + 3) & ~3) - 1;   // group index the pending pair belongs to (may be a phantom one)
    // the last bundle of the last group is still waiting for its rescale
    static_for<0, SB>([&](auto tc) {
        constexpr int t = decltype(tc)::value, j = t / NB, i = t % NB, qp = NBG - 1;
        constexpr int s_last = (3 * NBG + qp) & 1;   // accumulator set of the last bundle of a group with g & 3 == 3
        finish4(P[s_last][i], std::integral_constant<int, NB * qp + i>{}, std::integral_constant<int, j>{}, sw_prev, g_last, 0);
    });
    // Drain: the last requests (clamped re-reads past the end of K) are still in flight, aimed at
    // this block's LDS and at registers nothing reads any more.  Tying those registers to the
    // wait keeps them allocated until the data has arrived; without it they could be reused
    // (say for an epilogue address) and then be overwritten by a late load.
    static_for<0, NRAW>([&](auto rc) { await_loads<0>(raw[decltype(rc)::value][0], raw[decltype(rc)::value][1]); });
    static_for<0, NBUF>([&](auto sc) { await_loads<0>(b[decltype(sc)::value][0], b[decltype(sc)::value][1], b[decltype(sc)::value][2], b[decltype(sc)::value][3]); });
    await_loads<0>(meta_nxt.s, meta_nxt.z);
    await_loads<0>(sa_bits);
    if constexpr (HAND_SA && !EARLY_SA) {   // (operand and int32 accumulator registers are free now)
        request_token_scales();
        await_token_scales();
    }
    MIXLLM_STAMP(3);
    if (DUMP == 1) return;
    if (DUMP == 2) {
        // (the channel passes through an empty asm statement so that no store address is computed,
        // and kept in registers, before the K loop)
        int ch_out = ch;
        asm volatile("" : "+v"(ch_out));
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < p.M && ch_out >= 0) p.S[(size_t)m * p.N + ch_out] = isum[mt][r];
            }
        return;
    }

    // ---- K split over several blocks: this block's fp32 sums go to the workspace, in the order of
    //      the concatenated (padded) rows; prefill_reduce_kernel adds the parts, scales and scatters
    if (p.kparts > 1) {
        const int jp = (PART8 ? 0 : p.ntiles8 * TILE_N) + rw;
        const bool valid = t16 < ntiles;
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < p.M && valid) p.partials[((size_t)kp * p.M + m) * p.np + jp] = acc[mt][r];
            }
        return;
    }
    // ---- epilogue: token scale, fp16, scatter (Sec. 3.4) ------------------------------
    // per token tile: the 16 token scales of the lane's rows are fetched together (clamped,
    // unconditional) so that the loads overlap instead of costing one round trip per row
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        float sa[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            if constexpr (HAND_SA) sa[r] = half_bits_to_float(sa_ep[mt][r]);
            else sa[r] = ACT_PT ? (float)p.xscale[min(m, p.M - 1)] : 1.0f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            if (m < p.M && ch >= 0) p.y[(size_t)m * p.N + ch] = (half_t)(acc[mt][r] * sa[r]);
        }
    }
}


// 8-bit channel tiles whose scale does not depend on the group (one scale per channel): the
// group partial sums need no float rescale in between, so the MFMA accumulators simply run
// over all of K in int32 (|sum| <= K * 127 * 127 < 2^31 for K < 133000) and are converted and
// scaled once at the end.  Same activation pipeline as prefill_block; the four token tiles are
// four independent accumulation chains issued round robin.
template <typename C, bool ACT_PT, int DUMP>
static __device__ inline void prefill_block_w8_channel_scale(const LinearParams &p, int m0, int t16_0, int g_lo, int g_hi, int kp,
                                                            uint8_t *lds_a, float *lds_sa)
{
    constexpr int TM = C::TM, WN = C::WN, BM = C::BM, A_STAGE = C::A_STAGE, LPW = C::LPW, DFRAG = C::DFRAG, RING = C::RING;
    constexpr int NSLOT = TM * 4, HALF = NSLOT / 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int n32 = lane & 31, h = lane >> 5;
    const int mw0 = wm * TM * 32;
    const int t16 = t16_0 + wn * 2 + (n32 >> 4);
    const int tile16 = min(t16, p.ntiles8 - 1);
    const int rw = tile16 * TILE_N + (n32 & 15);
    const int ch = (t16 < p.ntiles8 && rw < p.n8) ? p.perm[rw] : -1;

    uint32_t a_voff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave * LPW + i) * 8 + (lane >> 3);
        const int cs = (lane & 7) ^ ((row >> 1) & 7);
        a_voff[i] = (uint32_t)min(m0 + row, p.M - 1) * (uint32_t)p.K + cs * 16;
    }
    const uint32_t lds_a_wave = __builtin_amdgcn_readfirstlane(lds_address(lds_a) + wave * LPW * 1024);
    auto load_a = [&](int g, int stage) {
        const int8_t *src = p.xq + (size_t)min(g, g_hi - 1) * G;
#pragma unroll
        for (int i = 0; i < LPW; ++i) load_lds16(lds_a_wave + stage * A_STAGE + i * 1024, a_voff[i], src);
    };
    int a_rd[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a_rd[j] = (mw0 + n32) * G + (((2 * j + h) ^ ((n32 >> 1) & 7)) << 4);

    const uint32_t b_voff = ((uint32_t)tile16 * (uint32_t)(p.K / 64) * 64 + (n32 & 15) + 16 * h) * 16;
    // weights are requested L8 groups ahead into a ring of L8 + 1 operand sets (see prefill_block)
    constexpr int L8 = C::L8, NBUF = L8 + 1;
    static_assert(NBUF == 2 || NBUF == 4, "operand sets are indexed by the group number modulo 4");
    v4i b[NBUF][4];
    auto load_b = [&](int g, auto setc) {
        constexpr int set = decltype(setc)::value % NBUF;
        const uint8_t *base = (const uint8_t *)p.w8 + (size_t)min(g, g_hi - 1) * 2048;
        load_reg16<0>(b[set][0], b_voff, base);
        load_reg16<512>(b[set][1], b_voff, base);
        load_reg16<1024>(b[set][2], b_voff, base);
        load_reg16<1536>(b[set][3], b_voff, base);
    };

    static_for<0, L8>([&](auto gc) { load_b(g_lo + decltype(gc)::value, gc); });
    load_a(g_lo, 0);
    load_a(g_lo + 1, 1);
    load_a(g_lo + 2, 2);
    static_assert(ACT_PT, "an integer sum over groups needs an activation scale that does not depend on the group");
    static_assert(DUMP != 1, "one accumulator over all of K: there is no per-group partial to dump");
    const float sw_row = (float)p.s8[rw];
    // token scales of the epilogue, requested by hand ahead of it (see prefill_block)
    constexpr bool HAND_SA = DUMP == 0, EARLY_SA = HAND_SA && TM <= 2;
    uint32_t sa_ep[HAND_SA ? TM : 1][16];
    auto request_token_scales = [&]() {
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                load_reg_u16(sa_ep[mt][r], (uint32_t)min(m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3), p.M - 1) * 2u, p.xscale);
    };
    auto await_token_scales = [&]() {
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) await_loads<0>(sa_ep[mt][r]);
    };
    if constexpr (EARLY_SA) {
        request_token_scales();
        await_token_scales();
    }
    static_for<0, L8>([&](auto sc) { await_loads<0>(b[decltype(sc)::value][0], b[decltype(sc)::value][1], b[decltype(sc)::value][2], b[decltype(sc)::value][3]); });
    __syncthreads();
    v4i af[RING];
    // slot t: k step t / TM, token tile t % TM
    auto load_frag = [&](auto stagec, auto tc) {
        constexpr int stage = decltype(stagec)::value, t = decltype(tc)::value;
        af[t % RING] = *(const v4i *)(lds_a + a_rd[t / TM] + stage * A_STAGE + (t % TM) * 32 * G);
    };
    static_for<0, DFRAG>([&](auto tc) { load_frag(std::integral_constant<int, 0>{}, tc); });

    v16i P[TM];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) P[mt][r] = 0;

    auto group_step = [&](int g, auto uc) {
        constexpr int U = decltype(uc)::value;
        // this group's weights were requested L8 groups ago; issued after them were the activation
        // loads of L8 middles and the weights of L8 - 1 groups
        await_loads<L8 * LPW + 4 * (L8 - 1)>(b[U % NBUF][0], b[U % NBUF][1], b[U % NBUF][2], b[U % NBUF][3]);
        load_b(g + L8, std::integral_constant<int, U + L8>{});
        if (g >= g_hi) {   // a group past the end (K/128 not a multiple of 4) must add nothing
#pragma unroll
            for (int j = 0; j < 4; ++j) b[U % NBUF][j] = v4i{0, 0, 0, 0};
        }
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NSLOT>([&](auto stc) {
            constexpr int st = decltype(stc)::value;
            if constexpr (st == HALF) {
                // group g+1's activations were requested two middles ago; issued after them were
                // the weights of two groups (4 loads each; with one group of look-ahead the older
                // of the two has been waited for at the start of this group) and the activations
                // of group g+2 (LPW loads)
                await_loads<(L8 == 1 ? LPW + 4 : LPW + 8)>();
                mid_group_barrier<false>();
                load_a(g + 3, (U + 3) % NSTAGE);
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (st + DFRAG < NSLOT)
                load_frag(std::integral_constant<int, U>{}, std::integral_constant<int, st + DFRAG>{});
            else
                load_frag(std::integral_constant<int, (U + 1) % NSTAGE>{}, std::integral_constant<int, st + DFRAG - NSLOT>{});
            P[st % TM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[st % RING], b[U % NBUF][st / TM], P[st % TM], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    for (int g = g_lo; g < g_hi; g += 4) {
        group_step(g, std::integral_constant<int, 0>{});
        group_step(g + 1, std::integral_constant<int, 1>{});
        group_step(g + 2, std::integral_constant<int, 2>{});
        group_step(g + 3, std::integral_constant<int, 3>{});
    }
    // drain (see prefill_block): nothing in flight towards this block's LDS or registers
    static_for<0, NBUF>([&](auto sc) { await_loads<0>(b[decltype(sc)::value][0], b[decltype(sc)::value][1], b[decltype(sc)::value][2], b[decltype(sc)::value][3]); });
    if constexpr (HAND_SA && !EARLY_SA) {   // (the operand registers are free now)
        request_token_scales();
        await_token_scales();
    }

    if (DUMP == 0 && p.kparts > 1) {   // K split over several blocks: see prefill_block
        const bool valid = t16 < p.ntiles8;
#pragma unroll
        for (int mt = 0; mt < TM; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < p.M && valid) p.partials[((size_t)kp * p.M + m) * p.np + rw] = (float)P[mt][r] * sw_row;
            }
        return;
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        float sa[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            if constexpr (HAND_SA) sa[r] = half_bits_to_float(sa_ep[mt][r]);
            else sa[r] = (float)p.xscale[min(m, p.M - 1)];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mw0 + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            if (DUMP == 2) {
                if (m < p.M && ch >= 0) p.S[(size_t)m * p.N + ch] = P[mt][r];
            } else if (m < p.M && ch >= 0) p.y[(size_t)m * p.N + ch] = (half_t)((float)P[mt][r] * sw_row * sa[r]);
        }
    }
}

template <typename C, int MINW, int DUMP, bool ACT_PT, bool W8PC>
__global__ __launch_bounds__(C::THREADS, MINW) void linear_prefill_kernel(LinearParams p, int nbm4, int nbm8, int nb8,
                                                                         int nb4, int per4, int per8, int band4, int band8, int half8)
{
    // K split over p.kparts blocks (blockIdx.y): part kp takes 4 * p.quads_per_part groups
    MIXLLM_STAMP(0);
    const int kp = blockIdx.y;
    const int g_lo = kp * p.quads_per_part * 4, g_hi = min(p.ng, g_lo + p.quads_per_part * 4);
    // dynamic LDS (more than the 64 KB a static array may take): the activation stages, then
    // the per-(token, group) activation scales when they are in use
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    uint8_t *lds_a = smem;
    float *lds_sa = (float *)(smem + NSTAGE * C::A_STAGE);
    // Blocks are dealt round-robin to the 8 XCDs, each with its own L2.  Logical ids enumerate
    // the tile grid in bands of `band` token tiles: inside a band, channel tiles are the outer
    // index and the band's token tiles the inner one, so the ~64 blocks an XCD runs at a time
    // form a roughly square patch (band x 64/band tiles) that shares both its activation rows
    // and its weight columns through that L2.  Every XCD gets a contiguous range of the 4-bit
    // ids followed by a contiguous range of the 8-bit ids, so that every XCD ends on the cheap
    // tiles: 4-bit tiles take about twice as long as 8-bit ones (unpack, per-group rescale), and
    // the cheap ones fill the last, partly empty round of the grid.
    // Where the host says so (half8: a launch of 128 x 128 blocks at most four rounds long) the 8-bit
    // tiles are half as tall as the 4-bit ones (C::Half).  Blocks are dispatched in the order of
    // their ids, so the 8-bit blocks - the last of every XCD - are what runs while the last 4-bit
    // blocks finish, and the finer they are the less of the chip idles then: with N = 4096 and 10 %
    // 8-bit channels a launch has 33 column tiles, 2048 tokens make 528 blocks of 128 x 128 for 512
    // places, and the 16 late ones cost 15 % of the launch (58 us against 50 us for 32 column
    // tiles); as 128 blocks of 64 x 128 they fit the shadow of the 4-bit blocks.
    using C8 = typename C::Half;
    const int xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    const bool part8 = i >= per4;
    const int nb = part8 ? nb8 : nb4, nbm = part8 ? nbm8 : nbm4, band = part8 ? band8 : band4;
    const int L = part8 ? xcd * per8 + (i - per4) : xcd * per4 + i;
    if (L >= nbm * nb) return;
    const int bd = L / (band * nb);              // bands before the last one are full
    const int w = min(band, nbm - bd * band);    // token tiles in this band
    const int r = L - bd * band * nb;
    const int bn = r / w, bm = bd * band + r % w;
    constexpr int T16 = C::BN / TILE_N;
    constexpr bool ASYNC = true;   // every variant issues its loads by hand; spill free (checked by the build)
    auto tile8 = [&](auto shape) {
        using S = decltype(shape);
        if constexpr (W8PC && ACT_PT && DUMP != 1)
            prefill_block_w8_channel_scale<S, ACT_PT, DUMP>(p, bm * S::BM, bn * T16, g_lo, g_hi, kp, lds_a, lds_sa);
        else
            prefill_block<S, DUMP, ACT_PT, true, !W8PC, ASYNC>(p, bm * S::BM, bn * T16, g_lo, g_hi, kp, lds_a, lds_sa);
    };
    if (part8) {
        // (8-bit tiles of 128 rows with a weight scale per group are not built: they do not fit the
        // register file next to the ring of operand sets; that granularity always takes the half tiles)
        if constexpr (!std::is_same<C8, C>::value && W8PC) {
            if (half8) tile8(C8{});
            else tile8(C{});
        } else
            tile8(C8{});
    } else
        prefill_block<C, DUMP, ACT_PT, false, false, ASYNC>(p, bm * C::BM, bn * T16, g_lo, g_hi, kp, lds_a, lds_sa);
#ifdef MIXLLM_STAMPS
    MIXLLM_STAMP(4);                                   // stores issued
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // ... and acknowledged
    MIXLLM_STAMP(5);
#endif
}

// K split over several blocks: the parts' fp32 sums (workspace, [part][token][padded concatenated
// row]) are added in part order - a fixed order, no atomics - scaled by the token's activation
// scale where that is one per token, converted and scattered (Sec. 3.4).
constexpr int MAX_KPARTS = 8;   // K parts a launch is split into at most
__global__ __launch_bounds__(256) void prefill_reduce_kernel(LinearParams p)
{
    // four consecutive rows of the padded concatenation per thread (p.np is a multiple of 16)
    const int jp0 = (blockIdx.x * 256 + threadIdx.x) * 4, m = blockIdx.y;
    if (jp0 >= p.np) return;
    const int n8p = p.ntiles8 * TILE_N;
    // all parts are requested before the first is added (one round trip instead of one per part)
    v4f part[MAX_KPARTS];
#pragma unroll
    for (int kp = 0; kp < MAX_KPARTS; ++kp)   // (past the last part: a re-read of the last one, not added)
        part[kp] = *(const v4f *)(p.partials + ((size_t)min(kp, p.kparts - 1) * p.M + m) * p.np + jp0);
    v4f v = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int kp = 0; kp < MAX_KPARTS; ++kp)
        if (kp < p.kparts) v += part[kp];
    const float sa = p.act_per_token ? (float)p.xscale[m] : 1.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int jp = jp0 + i;
        int j;
        if (jp < n8p) {
            if (jp >= p.n8) continue;
            j = jp;
        } else {
            if (jp - n8p >= p.n4) continue;
            j = p.n8 + (jp - n8p);
        }
        p.y[(size_t)m * p.N + p.perm[j]] = (half_t)(v[i] * sa);
    }
}

#ifdef MIXLLM_STAMPS
extern "C" int mixllm_debug_set_stamps(void *stamps)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_stamps), &stamps, sizeof stamps);
}
#endif

// The kernels take more dynamic LDS than the default limit; raising the limit is a per-function
// attribute, set on the first launch of each instantiation (per device: the attribute belongs to
// the loaded code object of the current device).
template <typename C, typename K>
static int launch_variant(K kernel, bool with_sa, dim3 grid, dim3 block, hipStream_t st, const LinearParams &p, int nbm4,
                          int nbm8, int nb8, int nb4, int per4, int per8, int band4, int band8, int half8)
{
    const size_t lds_bytes = (size_t)NSTAGE * C::A_STAGE + (with_sa ? (size_t)NSTAGE * C::BM * sizeof(float) : 16);
    // (kernel, device) pairs already configured; a handful of instantiations exist
    struct Done {
        const void *fn;
        int dev;
    };
    static Done done[64];
    static int ndone = 0;
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
    {
        std::lock_guard<std::mutex> lock(mu);
        bool seen = false;
        for (int i = 0; i < ndone; ++i) seen = seen || (done[i].fn == (const void *)kernel && done[i].dev == dev);
        if (!seen) {
            hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
            if (e != hipSuccess) return (int)e;
            if (ndone < 64) done[ndone++] = Done{(const void *)kernel, dev};
        }
    }
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, p, nbm4, nbm8, nb8, nb4, per4, per8, band4, band8, half8);
    if (p.kparts > 1)
        hipLaunchKernelGGL(prefill_reduce_kernel, dim3((p.np / 4 + 255) / 256, p.M), dim3(256), 0, st, p);
    return (int)hipGetLastError();
}

// the grid of a launch: token tiles of either part (BM rows for the 4-bit part; for the 8-bit part
// half of that where a launch of 128 x 128 blocks is at most four rounds of blocks long), channel
// tiles of either part, logical block ids per XCD of either part, token tiles per band of either part
// (see linear_prefill_kernel)
struct PrefillGrid {
    int bm8, nbm4, nbm8, nb8, nb4, per4, per8, band4, band8;
};
static PrefillGrid grid_of(const LinearParams &p, int BM, int BN)
{
    PrefillGrid g;
    g.nbm4 = (p.M + BM - 1) / BM;
    g.nb8 = (p.ntiles8 * TILE_N + BN - 1) / BN;
    g.nb4 = (p.ntiles4 * TILE_N + BN - 1) / BN;
#ifndef MIXLLM_PREFILL_HALF8_ROUNDS
#define MIXLLM_PREFILL_HALF8_ROUNDS 4   // launches of up to this many rounds of 128 x 128 blocks (two per CU) run their 8-bit part in half-height blocks
#endif
    const bool half8 = MIXLLM_PREFILL_HALF8 && BM == 128 && ((long)g.nbm4 * (g.nb4 + g.nb8) <= 2L * MIXLLM_PREFILL_HALF8_ROUNDS * cu_count() || !p.w8_per_channel || p.P);
    g.bm8 = half8 ? BM / 2 : BM;
    g.nbm8 = (p.M + g.bm8 - 1) / g.bm8;
    g.per4 = (g.nbm4 * g.nb4 + 7) / 8;
    g.per8 = (g.nbm8 * g.nb8 + 7) / 8;
    g.band4 = min(MIXLLM_PREFILL_BAND, g.nbm4);   // 4 measured best on the Llama shapes (8 and 2 within 2 %, whole columns 5 % slower)
    g.band8 = min(MIXLLM_PREFILL_BAND * (BM / g.bm8), g.nbm8);   // the same token rows per band
    return g;
}

template <typename C, int MINW>
static int launch_shape(const LinearParams &p, hipStream_t st)
{
    const PrefillGrid gr = grid_of(p, C::BM, C::BN);
    static_assert(C::Half::THREADS == C::THREADS && C::Half::BN == C::BN, "both parts run in blocks of the same width");
    dim3 grid((gr.per4 + gr.per8) * 8, p.kparts), block(C::THREADS);
    auto go = [&](auto kernel, bool with_sa) {
        return launch_variant<C>(kernel, with_sa, grid, block, st, p, gr.nbm4, gr.nbm8, gr.nb8, gr.nb4, gr.per4, gr.per8, gr.band4, gr.band8,
                                 gr.bm8 != C::BM);
    };
    // per-group partials (debug entry point): every tile through the per-group pipeline
    if (p.P) return go(linear_prefill_kernel<C, MINW, 1, true, false>, false);
    // the linear, or (debug entry point) the same kernels adding the partials up as integers
    if (p.act_per_token && p.w8_per_channel)
        return p.S ? go(linear_prefill_kernel<C, MINW, 2, true, true>, false) : go(linear_prefill_kernel<C, MINW, 0, true, true>, false);
    if (p.act_per_token) {
        if (!p.S) return go(linear_prefill_kernel<C, MINW, 0, true, false>, false);
        // the sums with group-wise 8-bit scales: built for one and two token tiles per wave (with four the
        // 8-bit tiles of this variant do not fit the register file)
        if constexpr (C::TM <= 2) return go(linear_prefill_kernel<C, MINW, 2, true, false>, false);
        return (int)hipErrorInvalidValue;
    }
    // Per-(token, group) activation scales: built for one and two token tiles per wave.  With four
    // the kernel needs more than 256 registers (the scale reads from LDS and the extra multiply
    // come on top of 235), and a kernel with hand-issued loads must not spill.
    if constexpr (C::TM <= 2) {
        if (p.w8_per_channel)
            return p.S ? go(linear_prefill_kernel<C, MINW, 2, false, true>, true) : go(linear_prefill_kernel<C, MINW, 0, false, true>, true);
        return p.S ? go(linear_prefill_kernel<C, MINW, 2, false, false>, true) : go(linear_prefill_kernel<C, MINW, 0, false, false>, true);
    }
    return (int)hipErrorInvalidValue;
}

static int choose_kparts(const LinearParams &p, int tm, size_t cap_bytes, int &qpp);

// token tiles (of 32) per wave: 4 = blocks of 128 x 128, 2 = 64 x 128, 1 = 32 x 128.
// `scratch_bytes` = the scratch the launch may split K with (0 = none).
static int token_tiles_per_wave(const LinearParams &p, size_t scratch_bytes)
{
    // variants only built for one and two token tiles per wave: group-wise activation scales; the debug
    // sums with group-wise 8-bit scales
    const bool group_scaled_acts = (!p.act_per_token && !p.P) || (p.S && !p.w8_per_channel);
    if (p.prefill_tm) return (p.prefill_tm == 4 && group_scaled_acts) ? 0 : p.prefill_tm;   // the caller's choice (tests, benchmarks)
    const long nbn = (p.ntiles8 * TILE_N + 127) / 128 + (p.ntiles4 * TILE_N + 127) / 128;
    const long tiles128 = (long)((p.M + 127) / 128) * nbn, tiles64 = (long)((p.M + 63) / 64) * nbn;
    if (3 * tiles64 <= 2 * cu_count() || p.M <= 32) {                  // (never a block taller than the batch)
        // A grid this small is a race of serial chains: a block walks its quantization groups one
        // after the other, and the launch takes as long as the busiest CU.  32-row or 64-row blocks,
        // with the K split each would get, by
        //   blocks on the busiest CU (a second one half hidden behind the first)
        //     x groups of 4 per part x cost of a group of 4 in that block,
        //   + 4 where a second kernel adds the parts up, + 1.5 for the heavier start of a 64-row block
        // in units of a 32-row block's group of 4 (about 1.1 us; 1.25 for a 64-row block's).  Fitted
        // to the Llama-shaped layers with the weights read from HBM: K = 28672, N = 8192 at 33 tokens
        // 61 us in 32-row blocks of 4 parts, 41 in 64-row blocks of 7; K = 14336, N = 4096 at 256
        // tokens 46 unsplit in 32-row blocks, 39 in 64-row blocks of 3 parts, but at 64 tokens 21
        // against 25 (eight parts either way); K = N = 8192 at 96 tokens 26 unsplit in 32-row blocks,
        // 28 in 64-row blocks of 3 parts; K = 8192, N = 10240 at 128 tokens without scratch 38 in
        // 324 blocks of 32 rows, 32 in 162 of 64; K = N = 4096 at 256 tokens 15.8 in 264 blocks of 32
        // rows, 17.4 in 132 of 64.
        if (p.M > 32) {
            const long cus = cu_count(), quads = (p.ng + 3) / 4;
            auto cost = [&](int tm, long blocks) {
                int qpp = (int)quads;
                const int kp = scratch_bytes ? choose_kparts(p, tm, scratch_bytes, qpp) : 1;
                const long on_a_cu = std::max(1L, (blocks * kp + cus - 1 - cus / 10) / cus);   // (a tenth of the CUs with one more block does not count)
                return (1.0 + 0.5 * (double)(on_a_cu - 1)) * qpp * (tm == 2 ? 1.25 : 1.0) + (kp > 1 ? 4.0 : 0.0) + (tm == 2 ? 1.5 : 0.0);
            };
            if (cost(2, tiles64) < cost(1, (long)((p.M + 31) / 32) * nbn)) return 2;
        }
        return 1;
    }
    if (3 * tiles128 <= 2 * cu_count() || group_scaled_acts || p.M <= 64) return 2;
    // (a last 128-row block that is at most half full is a quarter more work than 64-row blocks have:
    // K = 4096, N = 28672 at 192 tokens 48 us in 128-row blocks, 44.5 in 64-row blocks)
    if ((long)((p.M + 127) / 128) * 128 * 4 > (long)((p.M + 63) / 64) * 64 * 5) return 2;
    return 4;
}

// Shapes the kernel takes: lanes address activations, packed weights and metadata with 32-bit byte
// offsets; a caller-chosen block shape must exist for the scale granularity.
bool prefill_covers(const LinearParams &p)
{
    const size_t lim = (size_t)1 << 31;
    if ((size_t)p.M * (size_t)p.K >= lim || (size_t)p.ntiles4 * TILE_N * (size_t)p.K / 2 >= lim ||
        (size_t)p.ntiles8 * TILE_N * (size_t)p.K >= lim)
        return false;
    return p.M >= 1 && p.N >= 1 && token_tiles_per_wave(p, 0) != 0;
}

// K split.  A block walks its K range serially, and on layers with a long K (the down projections)
// that chain, not the chip, sets the time of a launch with few output tiles: 112 groups take 55 us
// whether 32 or 256 blocks run.  Where the grid of output tiles leaves the chip short of blocks the
// K range is cut into `kparts` parts for as many blocks (whole groups of 4 quantization groups, at
// least two of them per part, at most about two blocks per CU in all); the parts' fp32 sums meet in
// the caller's scratch (prefill_reduce_kernel), which costs a second launch and 8 bytes of traffic
// per part and output, so it is kept under 16 MB of sums.  Measured (Llama-3-8B down projection,
// K = 14336, N = 4096): 58 -> 22 us at 32 tokens, 56 -> 23 at 64, 56 -> 34 at 128, 55 -> 46 at
// 256; Llama-3.1-70B (K = 28672, N = 8192): 124 -> 46 at 32, 119 -> 88 at 128.  With K <= 4096
// there is nothing to gain: of the 14 us a 32 x 128 block of 32 groups lives, 4 us do not shrink with
// K, more blocks per CU slow each other's groups down, and the adding kernel costs 4-5 us (K = N =
// 4096 at 64 tokens: 14.5 us unsplit, 11.5 + 4.7 us in two parts, 11.6 + 4.7 us in four).
// Returns the number of parts and, in qpp, their length in groups of 4 quantization groups.
static int choose_kparts(const LinearParams &p, int tm, size_t cap_bytes, int &qpp)
{
    const int quads = (p.ng + 3) / 4;
    qpp = quads;
#ifdef MIXLLM_KSPLIT_ENV
    const char *forced = getenv("MIXLLM_KPARTS");   // measurement builds only: the number of parts from the environment
#else
    const char *forced = nullptr;
#endif
    if (p.P || p.S || (p.ng < 64 && !forced)) return 1;
    const PrefillGrid g = grid_of(p, 32 * tm, tm == 4 ? 32 * MIXLLM_PREFILL_WN_LARGE : 128);
    const long blocks = (long)g.nbm4 * g.nb4 + (long)g.nbm8 * g.nb8, slots = 2L * cu_count();   // (three 32-row blocks fit a CU, but counting on that split the wide K = 8192 layers in two and cost them 10 %)
    const size_t part_bytes = (size_t)p.M * p.np * sizeof(float);
    // (blocks of 64 rows and more run two to a CU: one part too many and the launch takes a second
    // round - K = 28672, N = 8192 at 33..64 tokens is 65 blocks, 43 us in 7 parts, 49 in 8; the
    // 32-row blocks fit more to a CU and measured best with the count rounded to nearest)
    // A grid of more than 0.6 blocks per CU is not split: K = N = 8192 at 96 tokens (195 blocks) 28 us
    // unsplit, 33 in three parts; at 192 tokens 33 against 39.
    if (10 * blocks > 6L * cu_count() && !forced) return 1;
    long kp = std::min<long>(MAX_KPARTS, std::min<long>(tm >= 2 ? slots / blocks : (slots + blocks / 2) / blocks, quads / 2));
    kp = std::min<long>(kp, (long)(std::min<size_t>(cap_bytes, (size_t)16 << 20) / part_bytes));
    if (forced) kp = std::min<long>(std::min<long>(atol(forced), MAX_KPARTS), std::min<long>(quads, (long)(cap_bytes / part_bytes)));
    if (kp <= 1) return 1;
    qpp = (int)((quads + kp - 1) / kp);
    return (quads + qpp - 1) / qpp;   // parts of qpp groups of 4: never more than kp
}

// true when the kernel, given `p.partials_cap` bytes of scratch, would split K
bool prefill_would_split(const LinearParams &p)
{
    int qpp;
    return prefill_covers(p) && p.partials && choose_kparts(p, token_tiles_per_wave(p, p.partials_cap), p.partials_cap, qpp) > 1;
}

size_t prefill_scratch_bytes(const LinearParams &p)
{
    if (!prefill_covers(p)) return 0;
    int qpp;
    const int kp = choose_kparts(p, token_tiles_per_wave(p, ~(size_t)0), ~(size_t)0, qpp);
    return kp > 1 ? (size_t)kp * p.M * p.np * sizeof(float) : 0;
}

int launch_linear_prefill(const LinearParams &p0, hipStream_t st)
{
    if (p0.M == 0 || p0.N == 0) return hipSuccess;
    if (!prefill_covers(p0)) return (int)hipErrorInvalidValue;
    LinearParams p = p0;
    p.kparts = 1;
    p.quads_per_part = (p.ng + 3) / 4;
    const int tm = token_tiles_per_wave(p, p.partials ? p.partials_cap : 0);
    if (p.partials) p.kparts = choose_kparts(p, tm, p.partials_cap, p.quads_per_part);
    // 128 x 128, 4 waves, wave tile 128 x 32 (a 128 x 256 block of 8 waves measured 5 % slower).
    // Where that grid has clearly less than one block per CU the chip is short of waves, not of rate:
    // blocks of 64 x 128 (wave tile 64 x 32) or 32 x 128 (wave tile 32 x 32) double the waves and
    // halve the chain of work each one runs; their packed 4-bit weights are requested two groups
    // ahead (a group is too short to cover the latency).
    // Measured on K = 4096, N = 4096, weights read from HBM at every launch, 128 x 128 -> the shape
    // chosen here: 25.6 -> 14.1 us at M = 128, 25.7 -> 15.7 at M = 256, 26.2 -> 20.9 at M = 512; K = 14336
    // (K not split): 76 -> 43, 76 -> 48, 76 -> 62.  With 192 blocks of 128 x 128 (N = 6144, M = 512) and
    // with 224 (N = 28672, M = 128) the shapes are within 2 % of each other.
    switch (tm) {
    case 1: return launch_shape<Shape<1, 4, 1, MIXLLM_PREFILL_WD_SMALL>, 2>(p, st);
    case 2: return launch_shape<Shape<1, 4, 2, MIXLLM_PREFILL_WD_SMALL>, 2>(p, st);
    default: return launch_shape<Shape<1, MIXLLM_PREFILL_WN_LARGE, 4, MIXLLM_PREFILL_WD_LARGE>, 2>(p, st);
    }
}

// the launch plan as thirteen integers (token rows and channels of a block tile of the 4-bit part, its
// token tiles, channel tiles of the 8-bit and of the 4-bit part, blocks launched per K part, token tiles
// per band of the 4-bit part, bytes of LDS, K parts, groups per K part, then token rows, token tiles and
// token tiles per band of the 8-bit part), for the host-side test of the block -> tile mapping
bool prefill_plan(const LinearParams &p, int out[13])
{
    if (!prefill_covers(p)) return false;
    const int tm = token_tiles_per_wave(p, ~(size_t)0);   // (the plan of a launch that has the scratch to split K)
    const int BM = 32 * tm, BN = tm == 4 ? 32 * MIXLLM_PREFILL_WN_LARGE : 128;
    const PrefillGrid g = grid_of(p, BM, BN);
    out[0] = BM;
    out[1] = BN;
    out[2] = g.nbm4;
    out[3] = g.nb8;
    out[4] = g.nb4;
    out[5] = (g.per4 + g.per8) * 8;
    out[6] = g.band4;
    out[7] = NSTAGE * BM * G + ((!p.act_per_token && !p.P) ? NSTAGE * BM * (int)sizeof(float) : 16);   // (p.P is never set here)
    int qpp;
    out[8] = choose_kparts(p, tm, ~(size_t)0, qpp);   // blocks sharing a K range when the caller brings the scratch for it
    out[9] = 4 * qpp;                                 // quantization groups per part
    out[10] = g.bm8;                                  // token rows, token tiles and token tiles per band of the 8-bit part
    out[11] = g.nbm8;
    out[12] = g.band8;
    return true;
}

}  // namespace mixllm
