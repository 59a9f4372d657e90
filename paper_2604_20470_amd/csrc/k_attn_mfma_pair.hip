// Stage (c), MFMA path for bf16, d = 128 (paper Eqs. 12-13 with epsilon -> 0): the variant that walks 256 queries
// per workgroup -- PAIRS of adjacent query blocks at Bs = 128 (described here), four blocks at Bs = 64, eight at
// Bs = 32 (the differences are noted at the kernels' definitions below).  gfx950 (CDNA4) only.
//
// One workgroup = 4 wavefronts x 64 queries = query blocks 2p and 2p + 1 of one (batch, head); one wavefront per
// SIMD, so that each may use the whole register file: the 128 O^T accumulators of its 64 queries live in the
// accumulation registers, everything the vector ALU touches in the ordinary ones.  Compared with one query block
// per workgroup (k_attn_mfma) every K / V fragment read from LDS feeds two matrix instructions instead of one, and
// every K / V tile fetched from L2 serves 256 queries instead of 128: the kernel runs at the device's power limit,
// so fewer joules per chunk is what buys time.
// The workgroup walks the ascending UNION of the two CSR rows (formed beforehand by k_group_union: key block in the
// low 28 bits of an entry, the rows that list it in bits 28-29); a wavefront whose query block does not list a key
// block runs the chunk with every logit masked.  Neighbouring query blocks share most of their key blocks (the
// never-pruned zone of a frame, and, for score-based selection, similar pooled scores), so the union is only a few
// per cent longer than a row.
//
// With a single wavefront per SIMD nothing else hides a wavefront's own latencies, so the chunk is software-pipelined
// by hand: 72 matrix-instruction slots per chunk with at most one exponential and a few other instructions in the
// shadow of each (see the schedule below); the exponentials of a chunk's last logit tile and its O += V P run under
// the first slots of the next chunk.  Every instruction beside the matrix instruction costs a lone wavefront issue
// time even in that shadow (about 1.8 cycles of the slot each, scalar instructions and waits included), so the loop
// is kept as short as it can be: the normaliser is summed by the matrix pipe, waits are placed by hand once per
// batch of LDS reads, and what a chunk needs to know about the chunk after next is worked out inside slots.
// A lone wavefront also pays for every branch in full (a not-taken branch between two matrix instructions costs it
// 9 to 26 cycles), so the 72 slots of a chunk are straight-line code without any masking: the pipelined loop takes
// full 64-key chunks only, and the tile loads of the chunk after next are always issued (past the end of the list
// they re-read the last window into the stage nobody reads).  The one chunk of a sequence that can be partial (in
// its last key block) is taken before the loop, by plain code, from a 64-row window moved back to end at the last
// row, whose leading rows are masked.  A wavefront whose query block does not list a chunk's key block skips the
// chunk's arithmetic altogether (it only takes part in loads and barrier; the tile it has in flight waits).
//
// Softmax.  Q is pre-multiplied by log2(e)/sqrt(d), so the logit products are exponents of 2, and they are
// exponentiated as they are: no exponent reference is subtracted.  Softmax is invariant to a reference; one is only
// needed to keep 2^x in range, and a row whose largest exponent exceeds kExactLimit = 64 in magnitude is outside
// the accuracy range of the pre-scaled Q anyway: such rows (and any whose normaliser leaves [2^-100, 2^100]) are
// flagged and taken again by k_attn_mfma's second pass, which moves a reference and scales in fp32.  Below the
// limit nothing overflows (fp32 and bf16 share one exponent range, so large or small probabilities lose no
// precision), the logit accumulation starts from the constant 0, and the accumulators, which are out of the vector
// ALU's reach, never need rescaling.  The normaliser sums the probabilities as rounded to bf16 (by one more matrix
// instruction per P^T fragment, of half length, with a constant operand of ones and zeros).
#include "attn_mfma_common.h"
#include "dr_internal.h"


#include <type_traits>

namespace dr {
namespace {

using namespace mfma;

constexpr int kD = 128;
constexpr int kRowsPerItem = 256;                    // queries of a workgroup: 256 / Bs adjacent query blocks
constexpr int kWaves = 4, kThreads = kWaves * 64;
constexpr int kChunkKeys = 64;
constexpr int kRowBytes = kD * 2;                    // 256
constexpr int kTileBytes = kChunkKeys * kRowBytes;   // 16 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;          // K then V
constexpr int kLdsBytes = 2 * kStageBytes;           // two stages: 64 KB
constexpr float kSumMax = 1.2676506e30f, kSumMin = 7.8886091e-31f;   // 2^100, 2^-100: outside, the row is flagged

struct LoadPlan {
    uint32_t koff_i[4], voff_i[4];   // per-lane byte offset of this lane's 16 bytes in the wave's four pieces of a chunk (swizzle folded in)
    uint32_t m0_k;                   // LDS address of this wave's first K piece in stage 0
};

// Wave w moves pieces w, w+4, w+8, w+12 (1 KB = 4 rows each) of the K tile and of the V tile of the 64-row window at key0.
template <int STAGE>
__device__ __forceinline__ void issue_chunk(const LoadPlan& lp, const char* Kh, const char* Vh, int key0, int64_t row_bytes) {
    const uint64_t kbase = uniform64((uint64_t)(Kh + (int64_t)key0 * row_bytes));
    const uint64_t vbase = uniform64((uint64_t)(Vh + (int64_t)key0 * row_bytes));
    const uint32_t m0 = lp.m0_k + STAGE * kStageBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        dma16(lp.koff_i[i], kbase, m0 + i * 4096);
        dma16(lp.voff_i[i], vbase, m0 + kTileBytes + i * 4096);
    }
}

// The same for a chunk made of two 32-row windows (block size 32): tile rows 0..31 from key0_a, rows 32..63 from key0_b.
// The per-lane offsets of pieces 2, 3 already contain their 32 rows: the second base is taken 32 rows back.
template <int STAGE>
__device__ __forceinline__ void issue_chunk2(const LoadPlan& lp, const char* Kh, const char* Vh, int key0_a, int key0_b, int64_t row_bytes) {
    const uint64_t ka = uniform64((uint64_t)(Kh + (int64_t)key0_a * row_bytes)), va = uniform64((uint64_t)(Vh + (int64_t)key0_a * row_bytes));
    const uint64_t kb = uniform64((uint64_t)(Kh + ((int64_t)key0_b - 32) * row_bytes)), vb = uniform64((uint64_t)(Vh + ((int64_t)key0_b - 32) * row_bytes));
    const uint32_t m0 = lp.m0_k + STAGE * kStageBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        dma16(lp.koff_i[i], i < 2 ? ka : kb, m0 + i * 4096);
        dma16(lp.voff_i[i], i < 2 ? va : vb, m0 + kTileBytes + i * 4096);
    }
}

struct State {
    v16f o[2][4];     // [query half][channel block] O^T accumulators (accumulation registers)
    v4f lacc[2];      // [query half] normaliser: a 16x16 tile that holds the 32 queries' sums (accumulation registers)
    v8bf ones;        // A operand of the normaliser's matrix instruction: per lane all 1 or all 0 (sum_selector)
};

struct ReadPlan {
    uint32_t k_addr[8];   // LDS address for contraction step ks (stage 0, key sub-block 0)
    uint32_t v_addr[4];   // LDS address for channel block db (stage 0, mb 0, st 0, low half of the 8 keys)
};

typedef __attribute__((address_space(3))) const v8bf* lds_v8;
typedef __attribute__((address_space(3))) v4s* lds_v4;

// O^T accumulators live in the accumulation registers: in the chunk loop only matrix instructions touch them.
// The instruction goes through inline assembly so that its destination class can be chosen here (the compiler
// picks one class for all its own matrix instructions); it therefore does not know this is a matrix instruction,
// and the code that reads these accumulators with the vector ALU (epilogue) waits out the result latency by hand.
__device__ __forceinline__ void mfma_pv(v16f& acc, const v8bf& a, const v8bf& b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The normaliser's instruction: the 16x16x32 shape, half the passes of a 32x32x16.  Its B operand is a P^T fragment
// as the 32x32x16 instructions take it (lane: query lane % 32, eight keys), which the 16x16x32 shape reads as
// column lane % 16 with the four 16-lane groups as four stretches of its contraction index: groups 0 and 2 hold
// query n, groups 1 and 3 query n + 16.  An A operand that is 1 in groups 0 and 2 for rows 0..7 and in groups 1 and
// 3 for rows 8..15, 0 elsewhere (a lane's eight values are all the same), makes row m, column n of the product the
// fragment's sum for query n (m < 8) or n + 16 (m >= 8): lane L of the result holds the sum of query
// (L % 16) + 16 * (L / 32), in each of its four registers.
__device__ __forceinline__ void mfma_l(v4f& acc, const v8bf& a, const v8bf& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ bool sum_selector(int lane) { return (((lane >> 4) & 1) != 0) == ((lane & 15) >= 8); }
// the lane that holds the sum of query q (0..31) of a query half
__device__ __forceinline__ int sum_lane(int q) { return (q & 15) + 32 * (q >> 4); }
// The logit products go through inline assembly as well, so that the register classes are fixed here: logits in
// ordinary registers (the exponentials read them), Q fragments in accumulation registers.  The schedule keeps every
// reader of a logit tile at least one matrix-instruction slot behind the tile's last step.
__device__ __forceinline__ void mfma_s_first(v16f& s, const v8bf& k, const v8bf& q) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_s(v16f& s, const v8bf& k, const v8bf& q) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(k), "a"(q));
}
// Normaliser: a row's sum of probabilities is taken from the bf16-rounded values, the ones O += V P multiplies, so
// that numerator and denominator of the softmax see the same rounding and with one dominant key the quotient is
// exact.  (Summing the fp32 exponentials instead is what kernels that subtract the row maximum do, where the
// dominant probability is exactly 1 and rounds without error; here no reference is subtracted, the dominant
// probability is 2^s with any mantissa, and its rounding error, up to 2^-8 relative, would go straight into O:
// 2.2e-2 on rows with one dominant key and |V| near 5.)  The sums are formed by the matrix pipe: one more matrix
// instruction per P^T fragment (mfma_l: a selector of ones and zeros times P^T) leaves the 32 queries' sums over
// the fragment's 16 keys in lacc.  That is 72 matrix instructions per chunk instead of 64, eight of them of half
// length, but the vector ALU, whose instruction issue is what bounds a lone wavefront, loses three instructions per
// pair of probabilities (two unpacks, two additions; a lone wavefront pays 5 to 6 cycles for each).
// The accumulators are operands of the wait so that every later read of them depends on it (a plain register copy
// could otherwise be scheduled right behind the matrix instruction that produces its source).
__device__ __forceinline__ void drain_mfma(v16f (&o)[2][4], v4f (&lacc)[2]) {
    asm volatile("s_nop 15\n\ts_nop 15"
                 : "+a"(o[0][0]), "+a"(o[0][1]), "+a"(o[0][2]), "+a"(o[0][3]), "+a"(o[1][0]), "+a"(o[1][1]), "+a"(o[1][2]), "+a"(o[1][3]),
                   "+a"(lacc[0]), "+a"(lacc[1])
                 :: "memory");
}
#define DR_PIN_O() do { _Pragma("unroll") for (int qh_ = 0; qh_ < 2; ++qh_) { asm volatile("" : "+a"(st.lacc[qh_])); _Pragma("unroll") for (int db_ = 0; db_ < 4; ++db_) asm volatile("" : "+a"(st.o[qh_][db_])); } } while (0)

// ---- schedule of one chunk: 72 matrix-instruction slots, an exponential in 64 of them ----
// A wave owns 64 queries = two query halves qh; a chunk has two 32-key halves mb; tile (mb, qh) is 32 keys x 32 queries.
// "S" = the 8 steps of a logit tile; "PVL" = O += V P of a tile, 10 instructions: for each of its two P^T fragments t
// the four channel blocks of O, then the normaliser.
//   slots  0.. 7  S (0,0)      18..25  S (0,1)      26..33  S (1,0)      44..51  S (1,1)
//   slots  8..17  PVL of tile (1,1) of the PREVIOUS chunk      34..43  PVL (0,0)      52..61  PVL (0,1)      62..71  PVL (1,0)
// The exponentials are one stream, position q = 0..63, in slot q + 1 + q / 8 (every ninth slot has none): the second
// half of tile (1,1) of the previous chunk in slots 1..8, (0,0) in 10..26, (0,1) in 28..44, (1,0) in 46..62, the
// first half of (1,1) in 64..71.  A pair = two exponentials in adjacent slots and one pack to bf16 in the slot after
// (the last pair of a chunk is packed in slot 0 of the next chunk the wavefront takes part in, or after the loop).
// Every tile is read by its first exponential at least two slots after its last step, and every P^T fragment is
// complete at least four slots before the first instruction that multiplies it.
// LDS reads: K fragments of key half 1 in slots 10..17, V^T fragments of key half 0 in 18..25, of key half 1 in 44..51;
// after that the chunk's LDS stage is not read again: the barrier sits before slot 56, and slots 56..63 also fetch the K
// fragments of the next chunk's first key half and issue the tile loads of the chunk after it.
constexpr int kSlots = 72;
constexpr int kBarrierSlot = 56;
struct MfmaSlot { int kind, mb, qh, idx; };   // kind 0: S step idx of tile (mb, qh); 1: O += V P, idx = t * 4 + db; 2: normaliser, idx = t
constexpr MfmaSlot pvl_at(int mb, int qh, int i) {
    if (i == 4 || i == 9) return {2, mb, qh, i / 5};
    return {1, mb, qh, (i / 5) * 4 + i % 5};
}
constexpr MfmaSlot mfma_at(int slot) {
    if (slot < 8) return {0, 0, 0, slot};
    if (slot < 18) return pvl_at(1, 1, slot - 8);
    if (slot < 26) return {0, 0, 1, slot - 18};
    if (slot < 34) return {0, 1, 0, slot - 26};
    if (slot < 44) return pvl_at(0, 0, slot - 34);
    if (slot < 52) return {0, 1, 1, slot - 44};
    if (slot < 62) return pvl_at(0, 1, slot - 52);
    return pvl_at(1, 0, slot - 62);
}
struct ExpSlot { bool valid; int mb, qh, gi, second; };   // exponential of value 2 gi + second of tile (mb, qh)
constexpr ExpSlot exp_at(int slot) {
    if (slot % 9 == 0) return {false, 0, 0, 0, 0};
    const int q = slot - 1 - slot / 9, k = q >> 1, second = q & 1;
    if (k < 4) return {true, 1, 1, 4 + k, second};
    if (k < 12) return {true, 0, 0, k - 4, second};
    if (k < 20) return {true, 0, 1, k - 12, second};
    if (k < 28) return {true, 1, 0, k - 20, second};
    return {true, 1, 1, k - 28, second};
}

struct Frags {
    v8bf kf0[8], kf1[8];
    v8bf vf[2][2][4];      // [mb][t][db]
    v8bf pf[2][2][2];      // [mb][qh][t]
    v16f s[2][2];          // [mb][qh]
    float e_pair[2];       // the pair of exponentials in flight: packed in the slot after the second was taken
    // block size 32 only: all-ones where the wavefront's query block qh lists the key block of key half mb, else 0 (the
    // probabilities of such a tile are packed as 0); tm11_prev: the same for tile (1,1) of the chunk still in flight
    uint32_t tm[2][2], tm11_prev;
};

template <int I, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// window rows below `lo` are not keys of this chunk for this wavefront (rows before a moved-back window's own keys, or
// every row when the wavefront's query block does not list the key block): logit -inf
__device__ __forceinline__ void mask_front(v16f& s, int mb, int half, int lo) {
    int base = mb * 32 + half * 4;
    asm volatile("" : "+v"(base));
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (base + (j >> 2) * 8 + (j & 3) < lo) s[j] = -INFINITY;
}

// Where the window of the chunk after next lies, worked out in five steps of a few scalar instructions each in the
// shadow of slots 28..32: between two slots the same instructions would leave the matrix pipe idle (a lone wavefront
// issues one instruction every four to five cycles, whatever its kind).
struct Next {
    int c2, win, Sb, N, grp;          // in: chunk index, the register window over the merged list, limits, the wave's owner bit
    uint32_t row_bytes;
    const char *Kh, *Vh;
    uint32_t e;                       // the list entry
    int key0;                         // first row of the 64-row window
    uint64_t off, kbase, vbase;
    bool own;                         // the wave's query block lists the key block
    // block size 32 (a chunk = two list entries = two 32-row windows; the wave has two query blocks, bits 2 grp, 2 grp + 1)
    int n_ent;                        // entries the chunk loop walks
    uint32_t e2;                      // second entry (owner bits cleared when there is none)
    int key0_b;
    uint64_t off_b, kbase2, vbase2;   // second window, 32 rows back (see issue_chunk2)
    uint32_t own4;                    // bit mb * 2 + qh
};
template <int K, int BS>
__device__ __forceinline__ void next_step(Next& nx) {
    if constexpr (BS == 32) {
        if constexpr (K == 0) {
            nx.e = (uint32_t)__builtin_amdgcn_readlane(nx.win, (2 * nx.c2) & 63);
            const uint32_t e2 = (uint32_t)__builtin_amdgcn_readlane(nx.win, (2 * nx.c2 + 1) & 63);
            nx.e2 = (2 * nx.c2 + 1 < nx.n_ent) ? e2 : (nx.e & 0x00ffffffu);
        }
        if constexpr (K == 1) {
            // (the clamps never act on a list as k_group_union writes it; they keep any other list inside K / V)
            nx.key0 = min(min((int)(nx.e & 0x00ffffffu), nx.Sb - 1) * 32, nx.N - 32);
            nx.key0_b = min(min((int)(nx.e2 & 0x00ffffffu), nx.Sb - 1) * 32, nx.N - 32);
        }
        if constexpr (K == 2) {
            nx.own4 = ((nx.e >> (24 + 2 * nx.grp)) & 3u) | (((nx.e2 >> (24 + 2 * nx.grp)) & 3u) << 2);
            nx.own = nx.own4 != 0u;
            nx.off = (uint64_t)(uint32_t)nx.key0 * nx.row_bytes;
            nx.off_b = (uint64_t)(uint32_t)nx.key0_b * nx.row_bytes - 32ull * nx.row_bytes;
        }
        if constexpr (K == 3) nx.kbase = uniform64((uint64_t)nx.Kh + nx.off);
        if constexpr (K == 4) nx.vbase = uniform64((uint64_t)nx.Vh + nx.off);
        if constexpr (K == 5) nx.kbase2 = uniform64((uint64_t)nx.Kh + nx.off_b);
        if constexpr (K == 6) nx.vbase2 = uniform64((uint64_t)nx.Vh + nx.off_b);
        return;
    }
    if constexpr (K > 4) return;
    constexpr int kSh = BS == 128 ? 1 : 0;      // chunks per list entry, as a shift
    if constexpr (K == 0) nx.e = (uint32_t)__builtin_amdgcn_readlane(nx.win, (nx.c2 >> kSh) & 63);
    if constexpr (K == 1) {
        // (the clamp of the key block never acts on a list as k_group_union writes it; it keeps any other list inside K / V)
        const int kb = min((int)(nx.e & 0x0fffffffu), nx.Sb - 1);
        nx.key0 = min(kb * BS + (nx.c2 & kSh) * kChunkKeys, nx.N - kChunkKeys);
    }
    if constexpr (K == 2) {
        nx.own = ((nx.e >> (28 + nx.grp)) & 1u) != 0;
        nx.off = (uint64_t)(uint32_t)nx.key0 * nx.row_bytes;
    }
    if constexpr (K == 3) nx.kbase = uniform64((uint64_t)nx.Kh + nx.off);
    if constexpr (K == 4) nx.vbase = uniform64((uint64_t)nx.Vh + nx.off);
}

// A tile load in two parts, so that the matrix instruction and the exponential of the slot sit between the write of m0
// and the load that reads it (the one wait state that needs) instead of a no-op, and m0 is written by the addition itself.
template <uint32_t OFF>
__device__ __forceinline__ void set_m0(uint32_t base) {
    asm volatile("s_add_i32 m0, %0, %1" :: "s"(base), "n"(OFF) : "m0", "scc");
}
__device__ __forceinline__ void dma16_go(uint32_t voff, uint64_t base) {
    asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(voff), "s"(base) : "memory");
}
// s_waitcnt lgkmcnt(n) alone (vmcnt and expcnt fields at their maxima): placed where a whole batch of LDS reads is known
// to have had time to arrive, one wait replaces the one per fragment the compiler would otherwise put before every use.
#define DR_WAIT_LGKM(n) __builtin_amdgcn_s_waitcnt(0xC07F | ((n) << 8))

// Slots [FROM, TO) of the chunk whose tiles sit in LDS stage STAGE.  rd holds the stage-0 addresses and never
// changes: the stage is a compile-time offset of every read (the chunk loop is unrolled over the two stages).  Slots
// 56..63 issue one tile load each of the window at nx.kbase / nx.vbase into this stage, which the barrier before them
// has released; slots 60..67 read the next chunk's first K fragments from the other stage; with kSkip a wavefront
// does only that (it sits the chunk out).
template <int FROM, int TO, bool kSkip, int STAGE, int BS>
__device__ __forceinline__ void run_slots(const ReadPlan& rd, const v8bf (&qf)[2][8], State& st, Frags& fr,
                                          const LoadPlan& lp, Next& nx) {
    constexpr uint32_t kS = STAGE * kStageBytes, kV = kS + kTileBytes;
    const uint32_t m0_next = lp.m0_k;
    static_for<FROM, TO>([&](auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        constexpr MfmaSlot m = mfma_at(slot);
        if constexpr (!kSkip && slot >= 28 && slot < 35) next_step<slot - 28, BS>(nx);
        if constexpr (!kSkip) {
            // K fragments of key half 0 (read in slots 60..67 of the previous chunk); of key half 1 (slots 10..17: at most
            // the 16 V^T reads behind them are still out); V^T of key half 0 (18..25); of key half 1 (44..51: only
            // the two K reads of slots 60, 61 are younger)
            if constexpr (slot == 0) DR_WAIT_LGKM(0);
            if constexpr (slot == 26) DR_WAIT_LGKM(15);
            if constexpr (slot == 34) DR_WAIT_LGKM(0);
            if constexpr (slot == 62) DR_WAIT_LGKM(2);
        }
        if constexpr (!kSkip && slot >= 56 && slot < 64 && TO == kSlots) {
            constexpr int i = (slot - 56) >> 1;
            set_m0<kS + ((slot & 1) ? kTileBytes : 0) + i * 4096>(m0_next);
        }
        if constexpr (kSkip) {
        } else if constexpr (m.kind == 0) {
            if constexpr (m.idx == 0) mfma_s_first(fr.s[m.mb][m.qh], m.mb ? fr.kf1[0] : fr.kf0[0], qf[m.qh][0]);
            else mfma_s(fr.s[m.mb][m.qh], m.mb ? fr.kf1[m.idx] : fr.kf0[m.idx], qf[m.qh][m.idx]);
        } else if constexpr (m.kind == 1) {
            constexpr int t = m.idx >> 2, db = m.idx & 3;
            mfma_pv(st.o[m.qh][db], fr.vf[m.mb][t][db], fr.pf[m.mb][m.qh][t]);
        } else {
            mfma_l(st.lacc[m.qh], st.ones, fr.pf[m.mb][m.qh][m.idx]);
        }
        // ---- LDS reads ----
        if constexpr (slot >= 10 && slot < 18) fr.kf1[slot - 10] = *(lds_v8)(uintptr_t)(rd.k_addr[slot - 10] + kS + 32 * kRowBytes);
        if constexpr ((slot >= 18 && slot < 26) || (slot >= 44 && slot < 52)) {
            constexpr int mb = slot >= 44, f = mb ? slot - 44 : slot - 18, t = f >> 2, db = f & 3;
            union { struct { v4s a, b; } s2; v8bf v; } u;
            u.s2.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(rd.v_addr[db] + kV + (mb * 32 + t * 16) * kRowBytes));
            u.s2.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(rd.v_addr[db] + kV + (mb * 32 + t * 16 + 8) * kRowBytes));
            fr.vf[mb][t][db] = u.v;
        }
        if constexpr (slot >= 60 && slot < 68 && TO == kSlots) {
            // the next chunk's first K fragments, from the other stage (also when there is no next chunk: the address is
            // a valid LDS address)
            fr.kf0[slot - 60] = *(lds_v8)(uintptr_t)(rd.k_addr[slot - 60] + (1 - STAGE) * kStageBytes);
        }
        // ---- one exponential; the slot after a pair's second exponential packs the two (not the same slot: the
        // instruction after a transcendental may not read its result, and the wait state would be one more instruction) ----
        if constexpr (!kSkip) {
            constexpr ExpSlot e = exp_at(slot);
            constexpr ExpSlot pe = exp_at((slot + kSlots - 1) % kSlots);
            float ev = 0.f;
            if constexpr (e.valid) ev = __builtin_amdgcn_exp2f(fr.s[e.mb][e.qh][2 * e.gi + e.second]);
            if constexpr (pe.valid && pe.second) {
                constexpr int t = pe.gi >> 2, i = (2 * pe.gi) & 7;
                v2bf pk;
                pk[0] = (__bf16)fr.e_pair[0];
                pk[1] = (__bf16)fr.e_pair[1];
                if constexpr (BS == 32) {
                    // the pairs of tile (1,1) packed in slots 0..8 belong to the chunk before
                    constexpr bool prev = slot == 0 || (pe.mb == 1 && pe.qh == 1 && pe.gi >= 4);
                    union { v2bf v; uint32_t u; } b;
                    b.v = pk;
                    b.u &= prev ? fr.tm11_prev : fr.tm[pe.mb][pe.qh];
                    pk = b.v;
                }
                asm volatile("" : "+v"(pk));      // anchors the pack in this slot of the interleaved stream
                fr.pf[pe.mb][pe.qh][t][i] = pk[0];
                fr.pf[pe.mb][pe.qh][t][i + 1] = pk[1];
            }
            if constexpr (e.valid) {
                fr.e_pair[e.second] = ev;
                asm volatile("" : "+v"(fr.e_pair[e.second]));
            }
        }
        if constexpr (slot >= 56 && slot < 64 && TO == kSlots) {
            // the barrier has released the stage: one tile load each of the chunk after next
            constexpr int i = (slot - 56) >> 1;
            constexpr bool second = BS == 32 && i >= 2;      // block size 32: tile rows 32..63 come from the second window
            const uint64_t kb_i = second ? nx.kbase2 : nx.kbase, vb_i = second ? nx.vbase2 : nx.vbase;
            if constexpr (kSkip) {
                if constexpr ((slot & 1) == 0) dma16(lp.koff_i[i], kb_i, m0_next + kS + i * 4096);
                else dma16(lp.voff_i[i], vb_i, m0_next + kS + kTileBytes + i * 4096);
            } else {
                if constexpr ((slot & 1) == 0) dma16_go(lp.koff_i[i], kb_i);
                else dma16_go(lp.voff_i[i], vb_i);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
}

// Completes what the last chunk leaves in flight: the second half of its tile (1,1), then that tile's O += V P and
// normaliser (the compiler's own matrix instructions here: outside the hand-scheduled loop it looks after the wait
// states between matrix instructions and their neighbours).
template <int BS>
__device__ __forceinline__ void finish_pending(State& st, Frags& fr) {
    auto masked = [&](v2bf pk) -> v2bf {
        if constexpr (BS == 32) {
            union { v2bf v; uint32_t u; } b;
            b.v = pk;
            b.u &= fr.tm11_prev;
            return b.v;
        }
        return pk;
    };
    {   // the pair whose second exponential was taken in the last slot: values 6, 7 of the first fragment
        v2bf pk;
        pk[0] = (__bf16)fr.e_pair[0];
        pk[1] = (__bf16)fr.e_pair[1];
        pk = masked(pk);
        fr.pf[1][1][0][6] = pk[0];
        fr.pf[1][1][0][7] = pk[1];
    }
#pragma unroll
    for (int gi = 4; gi < 8; ++gi) {
        v2bf pk;
        pk[0] = (__bf16)__builtin_amdgcn_exp2f(fr.s[1][1][2 * gi]);
        pk[1] = (__bf16)__builtin_amdgcn_exp2f(fr.s[1][1][2 * gi + 1]);
        pk = masked(pk);
        fr.pf[1][1][1][(2 * gi) & 7] = pk[0];
        fr.pf[1][1][1][((2 * gi) & 7) + 1] = pk[1];
    }
#pragma unroll
    for (int idx = 0; idx < 8; ++idx)
        st.o[1][idx & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr.vf[1][idx >> 2][idx & 3], fr.pf[1][1][idx >> 2], st.o[1][idx & 3], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 2; ++t) st.lacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.ones, fr.pf[1][1][t], st.lacc[1], 0, 0, 0);
}

// One whole chunk by plain code (no pipelining), from the tiles at LDS addresses rd + stage_off: window rows below
// `lo` masked.  Used before the pipelined loop for the sequence's partial chunk.
__device__ __forceinline__ void plain_chunk(const ReadPlan& rd, uint32_t stage_off, const v8bf (&qf)[2][8], State& st,
                                            int lo, int half, uint32_t qh_mask) {
    constexpr uint32_t kV = kTileBytes;
#pragma unroll
    for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            if (!((qh_mask >> qh) & 1u)) continue;      // (block size 32: a wave's two query halves are two query blocks)
            v16f acc;
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const v8bf kf = *(lds_v8)(uintptr_t)(rd.k_addr[ks] + stage_off + mb * 32 * kRowBytes);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qh][ks], acc, 0, 0, 0);
            }
            mask_front(acc, mb, half, lo);
            v8bf pf[2];
#pragma unroll
            for (int j = 0; j < 16; j += 2) {
                v2bf pk;
                pk[0] = (__bf16)__builtin_amdgcn_exp2f(acc[j]);
                pk[1] = (__bf16)__builtin_amdgcn_exp2f(acc[j + 1]);
                pf[j >> 3][j & 7] = pk[0];
                pf[j >> 3][(j & 7) + 1] = pk[1];
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    union { struct { v4s a, b; } s2; v8bf v; } u;
                    u.s2.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(rd.v_addr[db] + stage_off + kV + (mb * 32 + t * 16) * kRowBytes));
                    u.s2.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(rd.v_addr[db] + stage_off + kV + (mb * 32 + t * 16 + 8) * kRowBytes));
                    // (the compiler's own matrix instruction here: outside the hand-scheduled loop it looks after the
                    // wait states between matrix instructions and their neighbours)
                    st.o[qh][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, pf[t], st.o[qh][db], 0, 0, 0);
                }
#pragma unroll
            for (int t = 0; t < 2; ++t) st.lacc[qh] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.ones, pf[t], st.lacc[qh], 0, 0, 0);
        }
}

// grid: (ceil(Sb / kL) * H * B) in one dimension, remapped so that one XCD walks a contiguous run of items.
// One workgroup = 4 waves of 64 queries = kL adjacent query blocks (BS = 128: waves 0-1 block 2p, waves 2-3 block
// 2p + 1; BS = 64: wave w block 4p + w).
template <int BS>
__device__ __forceinline__ void attn_pair_body(const AttnArgs& a) {
    constexpr int kL = kRowsPerItem / BS;       // query blocks per workgroup: 2 (waves 0-1, 2-3), 4 (one per wave) or 8 (two per wave)
    constexpr int kSh = BS == 128 ? 1 : 0;      // chunks per list entry, as a shift (block size 32: two entries per chunk)
    constexpr int kOwnShift = BS == 32 ? 24 : 28;               // an entry: key block below, owner bits from here
    constexpr uint32_t kKbMask = (1u << kOwnShift) - 1u;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    constexpr int kXcds = 8;
    const int n_pairs = (a.Sb + kL - 1) / kL;
    const int total_items = n_pairs * a.td.H * a.td.B;
    const int per_xcd = (total_items + kXcds - 1) / kXcds;
    const int item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (item >= total_items) return;
    const int pair = item % n_pairs, h = (item / n_pairs) % a.td.H, b = item / (n_pairs * a.td.H);
    // grp: the wave's owner bit in a list entry (block size 32: its two bits are 2 grp and 2 grp + 1)
    const int grp = BS == 128 ? wave >> 1 : wave;
    const int qb_first = BS == 32 ? kL * pair + 2 * wave : kL * pair + grp;      // the wave's (first) query block, not clamped
    const bool has_rows = qb_first < a.Sb;
    const int qb = min(qb_first, a.Sb - 1);
    const int N = a.td.N;
    const int64_t row_bytes = a.td.stride_n * 2;
    const int64_t head_off = ((int64_t)b * a.td.stride_b + (int64_t)h * a.td.stride_h) * 2;
    const char* Qh = reinterpret_cast<const char*>(a.Q) + head_off;
    const char* Kh = reinterpret_cast<const char*>(a.K) + head_off;
    const char* Vh = reinterpret_cast<const char*>(a.V) + head_off;
    const int mh = (a.mask_heads == 1) ? 0 : h;
    const int64_t mask_id = (int64_t)b * a.mask_heads + mh;
    const int32_t* rp = a.rowptr + mask_id * (a.Sb + 1);
    // the pair's merged list sits at the colidx offset of its first row (as k_group_union writes it)
    const int64_t goff = min(max((int64_t)__builtin_amdgcn_readfirstlane(rp[kL * pair]), (int64_t)0), a.colidx_stride);
    const int32_t* gl = a.gcol + mask_id * a.colidx_stride + goff;
    const int cnt = __builtin_amdgcn_readfirstlane(a.gcount[mask_id * n_pairs + pair]);

    const float cs = kExpScale;
    const int q_wave0 = BS == 128 ? qb * 128 + (wave & 1) * 64 : qb * BS;
    v8bf qf[2][8];
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
        const int qrow = min(q_wave0 + qh * 32 + l32, N - 1);
        const char* src = Qh + (int64_t)qrow * row_bytes + half * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const v8bf raw = *reinterpret_cast<const v8bf*>(src + ks * 32);
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[qh][ks][i] = (__bf16)((float)raw[i] * cs);
        }
    }

    const uint32_t lds0 = lds_addr(smem);
    LoadPlan lp;
    {
        const int piece = lane & 15, r_first = wave * 4 + (lane >> 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lp.koff_i[i] = (uint32_t)((r_first + 16 * i) * row_bytes) + ((piece ^ (r_first & 15)) << 4);
            lp.voff_i[i] = (uint32_t)((r_first + 16 * i) * row_bytes) + ((piece ^ ((r_first & 3) << 2)) << 4);
        }
    }
    lp.m0_k = __builtin_amdgcn_readfirstlane(lds0 + wave * 1024);

    ReadPlan rd;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) rd.k_addr[ks] = lds0 + l32 * kRowBytes + (((ks * 2 + half) ^ (l32 & 15)) << 4);
    {
        const int v_e = (lane & 15) >> 2, v_c = lane & 3, v_grp = (lane >> 4) & 1;
        const int r0 = half * 4 + v_e;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int piece = db * 4 + v_grp * 2 + (v_c >> 1);
            rd.v_addr[db] = lds0 + r0 * kRowBytes + ((piece ^ (v_e << 2)) << 4) + (v_c & 1) * 8;
        }
    }

    State st;
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
#pragma unroll
        for (int j = 0; j < 4; ++j) st.lacc[qh][j] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int j = 0; j < 16; ++j) st.o[qh][db][j] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) st.ones[i] = (__bf16)(sum_selector(lane) ? 1.0f : 0.0f);
    asm volatile("" : "+v"(st.ones));
    DR_PIN_O();

    // ---- the chunk sequence.  Every entry of the merged list is a key block = two chunks of 64 keys, except the
    // sequence's last key block, which holds n_last = N - (Sb - 1) * 128 keys: n_last / 64 full chunks for the loop
    // and, if n_last is no multiple of 64, one partial chunk that is taken first, from the window of the sequence's
    // last 64 rows (its leading 64 - n_last % 64 rows masked).  The list is ascending, so only its last entry can be
    // that block. ----
    const int n_last = N - (a.Sb - 1) * BS;
    const int part_keys = n_last % (BS == 32 ? 32 : kChunkKeys);
    int wbase = 0;
    int win = (cnt > 0) ? gl[min(lane, cnt - 1)] : 0;
    const uint32_t e_last = (cnt > 0) ? (uint32_t)gl[cnt - 1] : 0u;
    // The Q fragments are only ever matrix-instruction operands: they live in accumulation registers, beside O, and
    // leave the ordinary registers to what the vector ALU touches.  (The pin also marks them as arrived: the compiler,
    // which cannot see the hand-issued tile loads, would otherwise re-wait for its own loads inside the loop.)
#pragma unroll
    for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+a"(qf[qh][ks]));
    asm volatile("" : "+v"(win));
    const uint32_t e_last_s = __builtin_amdgcn_readfirstlane(e_last);
    const bool has_last = cnt > 0 && (int)(e_last_s & kKbMask) >= a.Sb - 1;
    const bool has_part = has_last && part_keys != 0;
    // Block size 32: the loop walks the entries two at a time (n_ent of them: all but a partial last key block, which
    // is taken before the loop like the partial chunk of the larger block sizes: its keys are the last part_keys rows
    // of the window of the sequence's last 64 rows).
    const int n_ent = cnt - ((BS == 32 && has_part) ? 1 : 0);
    const int n_chunks = BS == 32 ? (n_ent + 1) >> 1
                                  : (cnt << kSh) - (has_last ? (1 << kSh) - n_last / kChunkKeys : 0);     // full chunks, in list order
    // the query halves (block size 32: query blocks) of this wave that list the partial block
    const uint32_t own_part = BS == 32 ? (e_last_s >> (kOwnShift + 2 * grp)) & 3u
                                       : (((e_last_s >> (kOwnShift + grp)) & 1u) ? 3u : 0u);
    struct Desc { int key0, key0_b; uint32_t own4; bool own; };
    auto describe = [&](int c) -> Desc {          // c < n_chunks, its entries inside the register window
        // (the clamps never act on a list as k_group_union writes it; they keep any other list inside K / V)
        if constexpr (BS == 32) {
            const uint32_t e = (uint32_t)__builtin_amdgcn_readlane(win, (2 * c) & 63);
            const uint32_t e2r = (uint32_t)__builtin_amdgcn_readlane(win, (2 * c + 1) & 63);
            const uint32_t e2 = (2 * c + 1 < n_ent) ? e2r : (e & kKbMask);
            const uint32_t own4 = ((e >> (kOwnShift + 2 * grp)) & 3u) | (((e2 >> (kOwnShift + 2 * grp)) & 3u) << 2);
            return Desc{min(min((int)(e & kKbMask), a.Sb - 1) * 32, N - 32), min(min((int)(e2 & kKbMask), a.Sb - 1) * 32, N - 32),
                        own4, own4 != 0u};
        } else {
            const uint32_t e = (uint32_t)__builtin_amdgcn_readlane(win, (c >> kSh) & 63);
            const int kb = min((int)(e & kKbMask), a.Sb - 1);
            const bool own = ((e >> (kOwnShift + grp)) & 1u) != 0;
            return Desc{min(kb * BS + (c & kSh) * kChunkKeys, N - kChunkKeys), 0, own ? 15u : 0u, own};
        }
    };
    auto issue = [&](auto stage_c, const Desc& d) {
        constexpr int stage = decltype(stage_c)::value;
        if constexpr (BS == 32) issue_chunk2<stage>(lp, Kh, Vh, d.key0, d.key0_b, row_bytes);
        else issue_chunk<stage>(lp, Kh, Vh, d.key0, row_bytes);
    };
    auto tile_masks = [](Frags& fr, uint32_t own4) {          // block size 32: own4 bit mb * 2 + qh
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int qh = 0; qh < 2; ++qh) fr.tm[mb][qh] = ((own4 >> (mb * 2 + qh)) & 1u) ? ~0u : 0u;
    };

    if (n_chunks > 0 || has_part) {
        // stage 0: the first full chunk (or, without one, the partial chunk); stage 1: the partial chunk
        const Desc d0 = (n_chunks > 0) ? describe(0) : Desc{N - kChunkKeys, N - 32, 0u, false};
        issue(std::integral_constant<int, 0>{}, d0);
        if (has_part) issue_chunk<1>(lp, Kh, Vh, N - kChunkKeys, row_bytes);
        DR_WAIT_VMCNT0();
        DR_BARRIER();
        if (has_part) {
            if (own_part) plain_chunk(rd, kStageBytes, qf, st, kChunkKeys - part_keys, half, own_part);
            DR_BARRIER();          // stage 1 is free again
        }
        if (n_chunks > 0) {
            const Desc d1 = describe(min(1, n_chunks - 1));
            issue(std::integral_constant<int, 1>{}, d1);          // with a single chunk: that chunk again, never read
            Frags fr;
            // software-pipeline prologue: "previous chunk" = nothing (logits -inf, probabilities and V fragments 0)
#pragma unroll
            for (int j = 0; j < 16; ++j) fr.s[1][1][j] = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int i = 0; i < 8; ++i) fr.pf[1][1][t][i] = (__bf16)0.f;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int i = 0; i < 8; ++i) fr.vf[1][t][db][i] = (__bf16)0.f;
            }
            fr.e_pair[0] = fr.e_pair[1] = 0.f;
            fr.tm11_prev = 0u;
            uint32_t own4_cur = d0.own4, own4_nxt = d1.own4;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) fr.kf0[ks] = *(lds_v8)(uintptr_t)(rd.k_addr[ks]);
            // Loop invariant at the top of a chunk: its tiles are complete in LDS for every wave, the K fragments of
            // its first key half are on their way to registers, and the loads of the following chunk have been issued.
            asm volatile("" : "+v"(fr.s[1][1]));
            bool own_cur = d0.own, own_nxt = d1.own;
            Next nx;
            nx.Sb = a.Sb; nx.N = N; nx.grp = grp; nx.row_bytes = (uint32_t)row_bytes; nx.Kh = Kh; nx.Vh = Vh;
            nx.n_ent = n_ent; nx.own4 = 0u;
            // The loop takes two chunks per turn, one per LDS stage, so that the stage is a compile-time offset of every
            // read; an odd count is made even by a last chunk that every wavefront sits out.
            const int n_even = (n_chunks + 1) & ~1;
#define DR_CHUNK(STAGE, C)                                                                                              \
            {                                                                                                           \
                DR_PIN_O();                                                                                             \
                nx.c2 = min((C) + 2, n_chunks - 1);                                                                     \
                const bool refill = (BS == 32 ? 2 * nx.c2 : nx.c2 >> kSh) >= wbase + 64;                                \
                if (own_cur) {                                                                                          \
                    if constexpr (BS == 32) tile_masks(fr, own4_cur);                                                   \
                    run_slots<0, 27, false, STAGE, BS>(rd, qf, st, fr, lp, nx);                                             \
                    if (refill) { wbase += 64; win = gl[min(wbase + lane, cnt - 1)]; asm volatile("" : "+v"(win)); }   \
                    nx.win = win;                                                                                       \
                    run_slots<27, kBarrierSlot, false, STAGE, BS>(rd, qf, st, fr, lp, nx);                                  \
                    DR_WAIT_VMCNT0();                                                                                   \
                    DR_BARRIER();                                                                                       \
                    __builtin_amdgcn_sched_barrier(0);                                                                  \
                    run_slots<kBarrierSlot, kSlots, false, STAGE, BS>(rd, qf, st, fr, lp, nx);                              \
                    if constexpr (BS == 32) fr.tm11_prev = fr.tm[1][1];                                                 \
                } else {                                                                                                \
                    if (refill) { wbase += 64; win = gl[min(wbase + lane, cnt - 1)]; asm volatile("" : "+v"(win)); }   \
                    nx.win = win;                                                                                       \
                    next_step<0, BS>(nx); next_step<1, BS>(nx); next_step<2, BS>(nx); next_step<3, BS>(nx); next_step<4, BS>(nx);           \
                    next_step<5, BS>(nx); next_step<6, BS>(nx);                                                         \
                    DR_WAIT_VMCNT0();                                                                                   \
                    DR_BARRIER();                                                                                       \
                    __builtin_amdgcn_sched_barrier(0);                                                                  \
                    run_slots<kBarrierSlot, kSlots, true, STAGE, BS>(rd, qf, st, fr, lp, nx);                               \
                }                                                                                                       \
                DR_PIN_O();                                                                                             \
                own_cur = own_nxt && (C) + 1 < n_chunks;                                                                \
                own_nxt = nx.own;                                                                                       \
                own4_cur = own4_nxt;                                                                                    \
                own4_nxt = nx.own4;                                                                                     \
            }
            asm volatile("; chunk loop begin");      // (markers for the check of the generated code: nothing
            for (int c = 0; c < n_even; c += 2) {    // between them may touch an accumulation register except the
                DR_CHUNK(0, c)                        // matrix instructions themselves)
                DR_CHUNK(1, c + 1)
            }
            asm volatile("; chunk loop end");
#undef DR_CHUNK
            finish_pending<BS>(st, fr);
        }
        DR_WAIT_VMCNT0();          // the loads issued by the last chunks write LDS: none may outlive the workgroup
    }

    // ---- epilogue ----
    drain_mfma(st.o, st.lacc);
    char* Oh = reinterpret_cast<char*>(a.O) + head_off;
    bool out_of_range = false;
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
        const float l = __shfl(st.lacc[qh][0], sum_lane(l32));   // lane -> query l32, both halves
        const float inv = (l > 0.f) ? 1.0f / l : 0.f;
        const int qrow = q_wave0 + qh * 32 + l32;
        if (has_rows && qrow < N) {
            char* dst = Oh + (int64_t)qrow * row_bytes;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    v4bf v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (__bf16)(st.o[qh][db][g * 4 + i] * inv);
                    *reinterpret_cast<v4bf*>(dst + (db * 32 + g * 8 + half * 4) * 2) = v;
                }
            if (a.lse && half == 0)
                a.lse[((int64_t)b * a.td.H + h) * N + qrow] =
                    (l > 0.f) ? logf(l) : -INFINITY;
            // a row that lists keys has l > 0 unless every exponential underflowed; l = 0 with an empty row is exact
            const int qb_h = BS == 32 ? min(qb_first + qh, a.Sb - 1) : qb;      // the query block of this half
            const bool listed = rp[qb_h + 1] > rp[qb_h];
            if (listed && !(l >= kSumMin && l <= kSumMax && fabsf(__log2f(l)) <= kExactLimit)) out_of_range = true;
        }
    }
    // Two flag words per wave: it covers the rows of two 32-row waves of the kernels that make the second pass; they are
    // indexed by 128-row group, four words each.  A wave whose query block lies past the end of the sequence still
    // clears its words when its group exists (block size 64, odd block count): the second pass reads all four.
    const int groups128 = (N + 127) / 128;
    const int q0_own = qb_first * BS + (BS == 128 ? (wave & 1) * 64 : 0);      // the wave's first query row, not clamped
    if (a.flags && (q0_own >> 7) < groups128) {
        const int any = (has_rows && __any(out_of_range)) ? 1 : 0;
        const int64_t base = (((int64_t)b * a.td.H + h) * groups128 + (q0_own >> 7)) * 4 + ((q0_own >> 6) & 1) * 2;
        if (lane < 2) a.flags[base + lane] = any;
    }
}

// Block size 128: two query blocks per workgroup, an entry of the merged list is two chunks.  Block size 64: four
// query blocks, one per wavefront, an entry is one chunk; the same 256 queries and the same code otherwise.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_attn_mfma_pair(AttnArgs a) { attn_pair_body<128>(a); }
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_attn_mfma_quad(AttnArgs a) { attn_pair_body<64>(a); }
// Block size 32: eight query blocks, two per wavefront (one per query half); a chunk is two entries of the merged list,
// its two key halves come from two 32-row windows, and a 32 x 32 tile whose query block does not list the key block of
// its key half contributes probabilities of 0 (they are masked where they are packed to bf16).
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_attn_mfma_oct(AttnArgs a) { attn_pair_body<32>(a); }

}  // namespace

bool attn_mfma_pair_supported(const AttnArgs& a) {
    // every chunk is a full 64-row window: the sequence must hold one; the 32-bit per-lane offsets must cover it
    return a.bf16 && a.td.d == kD && (a.Bs == 128 || a.Bs == 64 || a.Bs == 32) && a.td.N >= kChunkKeys &&
           a.Sb < (a.Bs == 32 ? (1 << 24) : (1 << 28)) &&
           a.td.stride_n * 2 * kChunkKeys < (1ll << 31) && a.gcol && a.gcount && a.flags;
}

hipError_t launch_attn_mfma_pair(const AttnArgs& a, hipStream_t s) {
    if (!attn_mfma_pair_supported(a)) return hipErrorNotSupported;
    const int L = kRowsPerItem / a.Bs;
    hipError_t e = launch_group_union(L, a, s);
    if (e != hipSuccess) return e;
    auto kern = a.Bs == 128 ? k_attn_mfma_pair : a.Bs == 64 ? k_attn_mfma_quad : k_attn_mfma_oct;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int total = ((a.Sb + L - 1) / L) * a.td.H * a.td.B;
    const int grid = (total + 7) / 8 * 8;          // every XCD gets the same number of slots
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), kLdsBytes, s, a);
    return hipGetLastError();
}

}  // namespace dr
