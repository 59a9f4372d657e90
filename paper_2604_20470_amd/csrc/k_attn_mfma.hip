// Stage (c), MFMA path: block-sparse flash-attention forward for bf16, d = 128, Bs = 128
// (paper Eqs. 12-13 with epsilon -> 0).  gfx950 (CDNA4) only.
//
// One workgroup (4 wavefronts, 32 query rows each) owns one query block of one (batch, head)
// and walks the CSR row of kept key blocks in chunks of 64 keys.  K and V chunks are gathered
// L2/HBM -> LDS with direct-to-LDS 16-byte loads, double buffered, so the next chunk streams
// in while the current one is consumed; two workgroups share a CU (2 x 64 KB of LDS).
//
// The logits are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane's
// 16 accumulator values then all belong to ONE query column, so the softmax row statistics
// are plain in-register reductions plus a single exchange with the lane 32 away, and the
// exponentiated tile, packed to bf16, already sits in the B-operand layout of the second
// product O^T += V^T P^T -- no LDS round trip for P.  The contraction index of that second
// product is permuted the same way on both operands: B slot (half h, element i) of step st in
// key sub-block mb is key mb*32 + 16 st + 8 (i/4) + 4 h + i%4.  V^T fragments come from the
// row-major V chunk with the transposing LDS read ds_read_b64_tr_b16 (lane i of a 16-lane
// group receives column i of the 4 x 16 patch addressed by the group).
//
// LDS layouts (row = key, 256 bytes, sixteen 16-byte pieces per row):
//   K chunk: piece p of row r stored at piece p ^ (r & 15)       -> conflict-free ds_read_b128 A operands
//   V chunk: piece p of row r stored at piece p ^ ((r & 3) << 2) -> the 4-row patches of a transposing
//            read fall in distinct 64-byte bank groups
// All LDS read addresses are (per-lane constant) + (compile-time immediate): the chunk loop is
// unrolled over the two stages, and the swizzles are folded into twelve per-lane base registers.
//
// Softmax.  Q is pre-multiplied by log2(e)/sqrt(d) and every logit accumulation starts from -m_ref, so
// the first product delivers the exponent of 2 directly.  The exponent reference m_ref of a query is set
// to the row maximum of the first chunk and afterwards moved only when needed: softmax is invariant to
// the reference, and fp32 / bf16 share one exponent range, so a stale reference costs no accuracy as
// long as nothing overflows.  The guard is the chunk's own contribution to the normaliser (a lane's 32
// probabilities, summed with v_dot2c_f32_bf16 from the bf16-rounded values, i.e. exactly what the second
// product multiplies): while it stays below 2^10 no probability exceeds 2^10; otherwise the row maximum
// is formed, the reference is raised to it, the 64 output accumulators are rescaled and the chunk's
// exponentials are redone.  The steady state therefore has no maximum reduction at all.
#include <algorithm>

#include "attn_mfma_common.h"
#include "dr_internal.h"

namespace dr {
namespace {

using namespace mfma;

constexpr int kD = 128, kBs = 128;
constexpr int kWaves = 4, kThreads = kWaves * 64;
constexpr int kChunkKeys = 64;
constexpr int kRowBytes = kD * 2;                    // 256
constexpr int kTileBytes = kChunkKeys * kRowBytes;   // 16 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;          // K then V
constexpr int kLdsBytes = 2 * kStageBytes;           // two stages: 64 KB
constexpr float kSumLimit = 1024.0f;                 // a lane's 32 probabilities of a chunk may sum to at most this

struct LoadPlan {
    uint32_t koff, voff;     // per-lane byte offset of this lane's 16 bytes within a 16-row group (swizzle folded in)
    uint32_t m0_k;           // LDS address of this wave's first K piece in stage 0
    int64_t row_bytes;
    int r_first;             // chunk row of this lane in the wave's first piece
    int piece;
};

// Wave w moves pieces w, w+4, w+8, w+12 (1 KB = 4 rows each) of the K tile and of the V tile.
template <int STAGE>
__device__ __forceinline__ void issue_chunk(const LoadPlan& lp, const char* Kh, const char* Vh, int key0, int last_row) {
    const uint64_t kbase = uniform64((uint64_t)(Kh + (int64_t)key0 * lp.row_bytes));
    const uint64_t vbase = uniform64((uint64_t)(Vh + (int64_t)key0 * lp.row_bytes));
    const uint32_t m0 = lp.m0_k + STAGE * kStageBytes;
    if (key0 + kChunkKeys - 1 <= last_row) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint64_t step = (uint64_t)(16 * i) * (uint64_t)lp.row_bytes;
            dma16(lp.koff, kbase + step, m0 + i * 4096);
            dma16(lp.voff, vbase + step, m0 + kTileBytes + i * 4096);
        }
    } else {   // last block of the sequence: rows past the end re-read the last valid row (masked later)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = lp.r_first + 16 * i;
            const int rc = min(r, last_row - key0);
            const uint32_t ko = (uint32_t)(rc * lp.row_bytes) + ((lp.piece ^ (r & 15)) << 4);
            const uint32_t vo = (uint32_t)(rc * lp.row_bytes) + ((lp.piece ^ ((r & 3) << 2)) << 4);
            dma16(ko, kbase, m0 + i * 4096);
            dma16(vo, vbase, m0 + kTileBytes + i * 4096);
        }
    }
}

struct State {
    v16f o[4];        // O^T accumulators: channel block db, value j -> channel db*32 + (j/4)*8 + 4*half + j%4
    v16f cinit;       // -m_ref in all sixteen values: the C operand that starts every logit accumulation
    float m_ref;      // exponent reference of this lane's query column, in log2 units (0 before the first chunk)
    float l_part;     // this lane's share of the normaliser
};

struct ReadPlan {
    uint32_t k_addr[8];   // LDS address for contraction step ks (stage 0, key sub-block 0)
    uint32_t v_addr[4];   // LDS address for channel block db (stage 0, mb 0, st 0, low half of the 8 keys)
};

template <int STAGE, bool kExact, class F>
__device__ __forceinline__ void chunk_body(const ReadPlan& rd, const v8bf (&qf)[8], State& st, bool& first,
                                           int valid, int half, F&& issue) {
    typedef __attribute__((address_space(3))) const v8bf* lds_v8;
    typedef __attribute__((address_space(3))) v4s* lds_v4;
    constexpr uint32_t kK = STAGE * kStageBytes, kV = STAGE * kStageBytes + kTileBytes;

    // ---- S^T = K Q^T : [64 keys x 32 queries], two independent accumulator chains ----
    // Q is pre-scaled by log2(e)/sqrt(d) and the accumulation starts from -m_ref, so the MFMA output is directly
    // the exponent of 2: no per-element scale or subtract is left for the vector ALU.  (kExact: Q is taken as
    // stored, the accumulation starts from zero and the scale and the reference are applied in fp32 afterwards.)
    v16f s[2];
    if constexpr (kExact) {
#pragma unroll
        for (int j = 0; j < 16; ++j) s[0][j] = 0.f;
        s[1] = s[0];
    } else {
        s[0] = st.cinit;
        s[1] = st.cinit;
    }
    {
        v8bf kf[2][8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) kf[mb][ks] = *(lds_v8)(uintptr_t)(rd.k_addr[ks] + kK + mb * 32 * kRowBytes);
        __builtin_amdgcn_sched_barrier(0);   // all sixteen K reads in flight before the first MFMA waits
        issue();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][ks], qf[ks], s[mb], 0, 0, 0);
    }
    if constexpr (kExact) {
        const float cs = kExpScale, neg_ref = -st.m_ref;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) s[mb][j] = __builtin_fmaf(s[mb][j], cs, neg_ref);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- V^T fragments: issued now so that they land while the softmax runs ----
    v8bf vf[2][2][4];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                union { struct { v4s a, b; } s2; v8bf v; } u;
                u.s2.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(rd.v_addr[db] + kV + (mb * 32 + t * 16) * kRowBytes));
                u.s2.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(rd.v_addr[db] + kV + (mb * 32 + t * 16 + 8) * kRowBytes));
                vf[mb][t][db] = u.v;
            }
    __builtin_amdgcn_sched_barrier(0);

    // keys past the end of the sequence (only in the last block)
    if (valid < kChunkKeys) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (mb * 32 + (j >> 2) * 8 + half * 4 + (j & 3) >= valid) s[mb][j] = -INFINITY;
    }

    // ---- online softmax, per query column ----
    // The exponentials are taken against the current reference straight away; the chunk's share of the normaliser
    // doubles as the overflow guard (it bounds every probability of the lane), so the row maximum is only formed
    // on the rare path that moves the reference (and on the first chunk, where no reference exists yet).
    v8bf pf[2][2];
    v2bf ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;
    auto exps = [&](float& lsum) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    v2bf pk;
                    pk[0] = (__bf16)__builtin_amdgcn_exp2f(s[mb][t * 8 + i]);
                    pk[1] = (__bf16)__builtin_amdgcn_exp2f(s[mb][t * 8 + i + 1]);
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lsum, false);
                    pf[mb][t][i] = pk[0];
                    pf[mb][t][i + 1] = pk[1];
                }
            }
    };
    float lc = 0.f;
    if (!first) exps(lc);
    if (first || __any(!(lc <= kSumLimit))) {
        float mx = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[mb][j]);
        mx = max_across_halves(mx);                         // finite: every chunk holds at least one valid key
        const float delta = first ? mx : fmaxf(mx, 0.f);
        const float alpha = __builtin_amdgcn_exp2f(-delta);
        st.m_ref += delta;
        st.l_part *= alpha;
#pragma unroll
        for (int j = 0; j < 16; ++j) st.cinit[j] -= delta;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) s[mb][j] -= delta;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int j = 0; j < 16; ++j) st.o[db][j] *= alpha;
        first = false;
        lc = 0.f;
        exps(lc);
    }
    st.l_part += lc;

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < 4; ++db)
                st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mb][t][db], pf[mb][t], st.o[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);   // keep the wait that follows below the last MFMA issue
}

// One work item = one query block of one (batch, head).  kExact = false: the fast pass; each wave leaves in a.flags
// (when given) whether any of its rows lies outside the accuracy range of the pre-scaled Q (see kExactLimit).
// kExact = true: the exponent scale applied in fp32 (the caller has checked that the item is flagged).
template <bool kExact>
__device__ __forceinline__ void attn_item(const AttnArgs& a, int item, unsigned char* smem) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int qb = item % a.Sb, h = (item / a.Sb) % a.td.H, b = item / (a.Sb * a.td.H);
    const int N = a.td.N;
    const int64_t row_bytes = a.td.stride_n * 2;
    const int64_t head_off = ((int64_t)b * a.td.stride_b + (int64_t)h * a.td.stride_h) * 2;
    const char* Qh = reinterpret_cast<const char*>(a.Q) + head_off;
    const char* Kh = reinterpret_cast<const char*>(a.K) + head_off;
    const char* Vh = reinterpret_cast<const char*>(a.V) + head_off;
    const int mh = (a.mask_heads == 1) ? 0 : h;
    const int32_t* rp = a.rowptr + ((int64_t)b * a.mask_heads + mh) * (a.Sb + 1);
    const int32_t* ci = a.colidx + ((int64_t)b * a.mask_heads + mh) * a.colidx_stride;
    // row range, clipped to the colidx array of this mask (a list cut short by a too small capacity stays in bounds)
    const int lim = (int)min(a.colidx_stride, (int64_t)0x7fffffff);
    const int beg = min(max(__builtin_amdgcn_readfirstlane(rp[qb]), 0), lim);
    const int end = min(max(__builtin_amdgcn_readfirstlane(rp[qb + 1]), beg), lim);

    const float cs = kExact ? 1.0f : kExpScale;
    // Q^T fragments (B operand of S^T = K Q^T): lane holds query l32, channels ks*16 + 8*half .. +7
    const int q_wave0 = qb * kBs + wave * 32;
    v8bf qf[8];
    {
        const int qrow = min(q_wave0 + l32, N - 1);
        const char* src = Qh + (int64_t)qrow * row_bytes + half * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const v8bf raw = *reinterpret_cast<const v8bf*>(src + ks * 32);
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[ks][i] = (__bf16)((float)raw[i] * cs);     // exponent scale folded into Q
        }
    }

    const uint32_t lds0 = lds_addr(smem);
    LoadPlan lp;
    lp.row_bytes = row_bytes;
    lp.piece = lane & 15;
    lp.r_first = wave * 4 + (lane >> 4);
    lp.koff = (uint32_t)(lp.r_first * row_bytes) + ((lp.piece ^ (lp.r_first & 15)) << 4);
    lp.voff = (uint32_t)(lp.r_first * row_bytes) + ((lp.piece ^ ((lp.r_first & 3) << 2)) << 4);
    lp.m0_k = __builtin_amdgcn_readfirstlane(lds0 + wave * 1024);

    ReadPlan rd;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) rd.k_addr[ks] = lds0 + l32 * kRowBytes + (((ks * 2 + half) ^ (l32 & 15)) << 4);
    {
        const int v_e = (lane & 15) >> 2, v_c = lane & 3, v_grp = (lane >> 4) & 1;
        const int r0 = half * 4 + v_e;                   // (r0 & 3) == v_e for every (mb, st, +8) row offset
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int piece = db * 4 + v_grp * 2 + (v_c >> 1);
            rd.v_addr[db] = lds0 + r0 * kRowBytes + ((piece ^ (v_e << 2)) << 4) + (v_c & 1) * 8;
        }
    }

    State st;
    st.m_ref = 0.f;
    st.l_part = 0.f;
    bool first = true;
#pragma unroll
    for (int j = 0; j < 16; ++j) st.cinit[j] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) st.o[db][j] = 0.f;

    // The row's key-block list is walked through a 64-entry register window (lane i holds entry base + i):
    // the per-block index comes from v_readlane, so no memory access sits on the loop's critical path.
    const int n_blocks = end - beg;
    const int last_blk_chunks = (N - (a.Sb - 1) * kBs + kChunkKeys - 1) / kChunkKeys;   // 1 or 2
    auto load_window = [&](int base) { return (n_blocks > 0) ? ci[beg + min(base + lane, n_blocks - 1)] : 0; };
    auto entry = [&](int win, int blk) {      // clamped, so that a malformed list cannot address outside K/V
        return min(max(__builtin_amdgcn_readlane(win, blk & 63), 0), a.Sb - 1);
    };
    int win = load_window(0);
    // Pin the Q fragments and the window as "arrived" before the loop: otherwise the compiler, which cannot see
    // the hand-issued tile loads, re-waits for its own outstanding loads inside the loop with counts that
    // would also drain the tile prefetch.
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));
    asm volatile("" : "+v"(win));
    int kb_next = (n_blocks > 0) ? entry(win, 0) : -1;
    if (kb_next >= 0) issue_chunk<0>(lp, Kh, Vh, kb_next * kBs, N - 1);
    DR_WAIT_VMCNT0();
    // Loop invariant at each barrier: every wave has waited for its own share of the chunk about to be
    // consumed, and has finished reading the previous chunk, whose stage the next loads overwrite.
    // A block is two chunks (stage 0, then stage 1); only the sequence's last block can have one.
    for (int blk = 0; blk < n_blocks; ++blk) {
        const int kb = kb_next;
        const int key0 = kb * kBs;
        const int n_chunks = (kb == a.Sb - 1) ? last_blk_chunks : 2;
        DR_BARRIER();
        chunk_body<0, kExact>(rd, qf, st, first, N - key0, half, [&]() { if (n_chunks == 2) issue_chunk<1>(lp, Kh, Vh, key0 + kChunkKeys, N - 1); });
        DR_WAIT_VMCNT0();
        if (((blk + 1) & 63) == 0 && blk + 1 < n_blocks) win = load_window(blk + 1);
        kb_next = (blk + 1 < n_blocks) ? entry(win, blk + 1) : -1;
        if (n_chunks == 2) {
            DR_BARRIER();
            chunk_body<1, kExact>(rd, qf, st, first, N - key0 - kChunkKeys, half, [&]() { if (kb_next >= 0) issue_chunk<0>(lp, Kh, Vh, kb_next * kBs, N - 1); });
            DR_WAIT_VMCNT0();
        } else if (kb_next >= 0) {   // only for a list that is not ascending: nothing was prefetched, load serially
            DR_BARRIER();
            issue_chunk<0>(lp, Kh, Vh, kb_next * kBs, N - 1);
            DR_WAIT_VMCNT0();
        }
    }

    // ---- epilogue: normalise and store O (row = query l32, channels db*32 + (j/4)*8 + 4*half + j%4) ----
    char* Oh = reinterpret_cast<char*>(a.O) + head_off;
    const float l = st.l_part + __shfl_xor(st.l_part, 32);
    const float inv = (l > 0.f) ? 1.0f / l : 0.f;
    const int qrow = q_wave0 + l32;
    if (qrow < N) {
        char* dst = Oh + (int64_t)qrow * row_bytes;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                v4bf v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (__bf16)(st.o[db][g * 4 + i] * inv);
                *reinterpret_cast<v4bf*>(dst + (db * 32 + g * 8 + half * 4) * 2) = v;
            }
        if (a.lse && half == 0)
            a.lse[((int64_t)b * a.td.H + h) * N + qrow] =
                (l > 0.f) ? st.m_ref * 0.6931471805599453f + logf(l) : -INFINITY;
    }
    if constexpr (!kExact) {
        if (a.flags) {
            const bool out_of_range = qrow < N && l > 0.f && !(fabsf(st.m_ref + __log2f(l)) <= kExactLimit);
            const int any = __any(out_of_range) ? 1 : 0;
            if (lane == 0) a.flags[(int64_t)item * 4 + wave] = any;
        }
    }
}

// Fast pass.  grid: (Sb * H * B) in one dimension.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own
// L2; id -> work item is remapped so that one XCD walks a contiguous run of (batch, head, query block) items:
// the workgroups resident on an XCD at any time are then neighbouring query blocks of one head, whose kept key
// blocks largely coincide (the forced zone of a frame), and their K/V tiles are served from that XCD's L2.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_mfma(AttnArgs a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    constexpr int kXcds = 8;
    const int total_items = a.Sb * a.td.H * a.td.B;
    const int per_xcd = (total_items + kXcds - 1) / kXcds;
    const int item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (item >= total_items) return;
    attn_item<false>(a, item, smem);
}

// Second pass: the flagged items only.  Usually none is, so the grid is small and every workgroup looks at a
// contiguous share of the flag words, one item per thread and step (a workgroup per item would spend 28 us at 23 640
// items on starting workgroups that leave at once; one item per workgroup and step, 27 us on dependent loads).
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_mfma_second_pass(AttnArgs a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __shared__ unsigned char s_flagged[kThreads];
    const int total_items = a.Sb * a.td.H * a.td.B;
    const int per = (total_items + (int)gridDim.x - 1) / (int)gridDim.x;
    const int begin = min((int)blockIdx.x * per, total_items), end = min(begin + per, total_items);
    for (int base = begin; base < end; base += kThreads) {
        const int mine = base + (int)threadIdx.x;
        int flagged = 0;
        if (mine < end) {
            const int4 f = *reinterpret_cast<const int4*>(a.flags + (int64_t)mine * 4);
            flagged = (f.x | f.y | f.z | f.w) != 0;
        }
        if (!__syncthreads_or(flagged)) continue;
        s_flagged[threadIdx.x] = (unsigned char)flagged;
        __syncthreads();
        for (int j = 0; j < kThreads && base + j < end; ++j) {
            if (!s_flagged[j]) continue;          // the same for every thread
            attn_item<true>(a, base + j, smem);
            __syncthreads();          // the next item's tile loads overwrite LDS that slower waves may still be reading
        }
        __syncthreads();
    }
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
    // the 32-bit per-lane offsets of the tile loads must cover 64 rows
    return a.bf16 && a.td.d == kD && a.Bs == kBs && a.td.stride_n * 2 * kChunkKeys < (1ll << 31);
}

static hipError_t allow_lds() {
    for (const void* k : {reinterpret_cast<const void*>(k_attn_mfma), reinterpret_cast<const void*>(k_attn_mfma_second_pass)}) {
        hipError_t attr = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (attr != hipSuccess) return attr;
    }
    return hipSuccess;
}

static void launch_second(const AttnArgs& a, hipStream_t s) {
    const int total = a.Sb * a.td.H * a.td.B;
    hipLaunchKernelGGL(k_attn_mfma_second_pass, dim3(std::min(total, 1024)), dim3(kThreads), kLdsBytes, s, a);
}

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s) {
    if (!attn_mfma_supported(a)) return hipErrorNotSupported;
    hipError_t attr = allow_lds();
    if (attr != hipSuccess) return attr;
    const int total = a.Sb * a.td.H * a.td.B;
    const int grid = (total + 7) / 8 * 8;          // every XCD gets the same number of slots
    hipLaunchKernelGGL(k_attn_mfma, dim3(grid), dim3(kThreads), kLdsBytes, s, a);
    if (a.flags) launch_second(a, s);
    return hipGetLastError();
}

hipError_t launch_attn_mfma_second_pass(const AttnArgs& a, hipStream_t s) {
    if (!attn_mfma_supported(a) || !a.flags) return hipErrorNotSupported;
    hipError_t attr = allow_lds();
    if (attr != hipSuccess) return attr;
    launch_second(a, s);
    return hipGetLastError();
}

}  // namespace dr
