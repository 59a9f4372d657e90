// Stage (c), MFMA path for the small block sizes: block-sparse flash-attention forward for bf16, d = 128,
// Bs = 32 or 64 (paper Eqs. 12-13 with epsilon -> 0; block sizes of its hyper-parameter table).  gfx950 only.
//
// The tiling is the one of the Bs = 128 kernel (4 wavefronts x 32 query rows, 64-key chunks staged through LDS
// with direct-to-LDS loads, S^T = K Q^T and O^T += V^T P^T on v_mfma_f32_32x32x16_bf16, softmax statistics in
// registers), but a workgroup's 128 query rows now span 128 / Bs query blocks, each with its own row of the CSR.
// The workgroup walks the ascending UNION of those rows: a key block is fetched into LDS once and every wavefront
// whose query block lists it multiplies against it; the others only take part in the loads and the barrier.
// The union is formed beforehand by k_group_union (one small launch per call): per 128-row group one list of
// packed entries, key block in the low 28 bits and the set of rows listing it in the top 4, so that the attention
// kernel follows a single list through a single register window, like the Bs = 128 kernel.
// Neighbouring query blocks share most of their key blocks (the never-pruned zone of a frame), so the gather
// traffic per useful flop stays close to that of Bs = 128 instead of growing 4x or 16x.
//   Bs = 64: a chunk is one key block; wavefronts 0-1 and 2-3 follow their own row.
//   Bs = 32: a chunk is two consecutive entries of the union (keys 0..31 and 32..63 of the tile come from different
//            places); every wavefront follows its own row and may use either half, both or none (a half it does
//            not own is masked like keys past the end of the sequence).
#include "attn_mfma_common.h"
#include "dr_internal.h"

#include <type_traits>

namespace dr {
namespace {

using namespace mfma;

constexpr int kD = 128;
constexpr int kRowsPerGroup = 128;                   // query rows per workgroup
constexpr int kWaves = 4, kThreads = kWaves * 64;
constexpr int kChunkKeys = 64;
constexpr int kRowBytes = kD * 2;
constexpr int kTileBytes = kChunkKeys * kRowBytes;   // 16 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;          // K then V
constexpr int kLdsBytes = 2 * kStageBytes;
constexpr float kSumLimit = 1024.0f;                 // a lane's probabilities of a chunk may sum to at most this
constexpr int kNoBlock = 0x7fffffff;

struct LoadPlan {
    uint32_t koff, voff;     // per-lane byte offset inside a 16-row group, swizzle folded in
    uint32_t m0_k;           // LDS address of this wave's first K piece in stage 0
    int64_t row_bytes;
    int r_first;             // tile row of this lane in the wave's first piece (0..15)
    int piece;
};

// One chunk of the union walk: up to two key blocks and, per key block, the set of CSR rows (bit l = row l of the
// workgroup) that list it.
struct Chunk {
    int kb0, kb1;            // kb1 < 0: no second block (Bs = 64 always; Bs = 32 at the odd end of the union)
    uint32_t rows0, rows1;
    bool valid;
};

// Tile rows 32 * part .. 32 * part + 31 <- the 32 tokens key0 .. key0 + 31; tokens past last_row re-read last_row
// (finite values; the logits of such keys are masked).  Wave w moves pieces w, w+4, w+8, w+12 of 4 rows: its pieces
// 2 * part and 2 * part + 1 fall into this part.
template <int STAGE>
__device__ __forceinline__ void issue_part(const LoadPlan& lp, const char* Kh, const char* Vh, int key0, int part,
                                           int last_row) {
    const uint32_t m0 = lp.m0_k + STAGE * kStageBytes + part * 8192;
    if (key0 + 31 <= last_row) {
        const uint64_t kbase = uniform64((uint64_t)(Kh + (int64_t)key0 * lp.row_bytes));
        const uint64_t vbase = uniform64((uint64_t)(Vh + (int64_t)key0 * lp.row_bytes));
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint64_t step = (uint64_t)(16 * i) * (uint64_t)lp.row_bytes;
            dma16(lp.koff, kbase + step, m0 + i * 4096);
            dma16(lp.voff, vbase + step, m0 + kTileBytes + i * 4096);
        }
    } else {
        const int base_row = min(key0, last_row);
        const uint64_t kbase = uniform64((uint64_t)(Kh + (int64_t)base_row * lp.row_bytes));
        const uint64_t vbase = uniform64((uint64_t)(Vh + (int64_t)base_row * lp.row_bytes));
        int r_first = lp.r_first;
        asm volatile("" : "+v"(r_first));  // keeps the clamped offsets of this rare path from being hoisted out of the loop
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = r_first + 16 * i;                          // row inside the part
            const int rc = min(key0 + r, last_row) - base_row;       // >= 0
            const uint32_t ko = (uint32_t)(rc * lp.row_bytes) + ((lp.piece ^ (r & 15)) << 4);
            const uint32_t vo = (uint32_t)(rc * lp.row_bytes) + ((lp.piece ^ ((r & 3) << 2)) << 4);
            dma16(ko, kbase, m0 + i * 4096);
            dma16(vo, vbase, m0 + kTileBytes + i * 4096);
        }
    }
}

struct State {
    v16f o[4];
    float m_ref;
    float l_part;
};

// The swizzles are xors on the 16-byte piece index and the LDS block is 1 KB aligned, so the address of contraction
// step ks / channel block db is the base with ks << 5 / db << 6 xor-ed in: two registers instead of twelve.
struct ReadPlan {
    uint32_t k_base;      // this lane's 16 bytes of key row (lane & 31), step 0, stage 0
    uint32_t v_base;      // this lane's 8 bytes of the transposing read for channel block 0, stage 0
};

// One chunk for one wavefront.  MBM = 3: both 32-key halves of the tile are this wavefront's; MBM = 1: one half, the
// one at byte offset sel_off of the K and V tiles (0 or 32 rows).  valid0 / valid1: number of real keys in the
// (first / second) half processed (>= 32: all).
template <int STAGE, int MBM, bool kExact, class F>
__device__ __forceinline__ void chunk_body(const ReadPlan& rd, const v8bf (&qf)[8], State& st, bool& first,
                                           int valid0, int valid1, float init0, float init1, uint32_t sel_off, int half,
                                           F&& issue) {
    typedef __attribute__((address_space(3))) const v8bf* lds_v8;
    typedef __attribute__((address_space(3))) v4s* lds_v4;
    constexpr uint32_t kK = STAGE * kStageBytes, kV = STAGE * kStageBytes + kTileBytes;
    constexpr int MB0 = (MBM & 1) ? 0 : 1, MB1 = (MBM & 2) ? 2 : 1;     // active key sub-blocks: MB0 .. MB1 - 1

    uint32_t k_base = rd.k_base, v_base = rd.v_base;
    asm volatile("" : "+v"(k_base), "+v"(v_base));   // the per-step addresses are formed here, not kept in registers across chunks
    // Register budget: the logit fragments are read in two batches of four contraction steps and the V^T fragments
    // one key sub-block at a time (the second one into the registers the logits vacate), so that the variants
    // of this body and the union walk fit the 256 registers of a wave without spilling into the loop.
    auto read_v = [&](int mb, v8bf (&dst)[2][4]) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                union { struct { v4s a, b; } s2; v8bf v; } u;
                u.s2.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)((v_base ^ (db << 6)) + kV + sel_off + (mb * 32 + t * 16) * kRowBytes));
                u.s2.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)((v_base ^ (db << 6)) + kV + sel_off + (mb * 32 + t * 16 + 8) * kRowBytes));
                dst[t][db] = u.v;
            }
    };
    // init0 / init1: 0, or -inf for a half this wavefront does not own (its logits stay -inf, its probabilities 0).
    // The accumulation starts from -m_ref, so the matrix instruction delivers the logits relative to the exponent
    // reference (the accumulators have to be initialised anyway; the Bs = 128 kernel keeps this vector in registers).
    // (kExact: Q is taken as stored, the accumulation starts from zero, and the exponent scale and the reference are
    // applied in fp32 afterwards.)
    v16f s[2];
    const float c0 = kExact ? 0.f : init0 - st.m_ref, c1 = kExact ? 0.f : init1 - st.m_ref;
#pragma unroll
    for (int j = 0; j < 16; ++j) { s[0][j] = c0; s[1][j] = c1; }
#pragma unroll
    for (int batch = 0; batch < 2; ++batch) {
        v8bf kf[2][4];
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
            for (int mb = MB0; mb < MB1; ++mb)
                kf[mb][k4] = *(lds_v8)(uintptr_t)((k_base ^ ((batch * 4 + k4) << 5)) + kK + sel_off + mb * 32 * kRowBytes);
        __builtin_amdgcn_sched_barrier(0);
        if (batch == 0) {
            issue();
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
            for (int mb = MB0; mb < MB1; ++mb)
                s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][k4], qf[batch * 4 + k4], s[mb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (kExact) {
        const float cs = kExpScale, a0 = init0 - st.m_ref, a1 = init1 - st.m_ref;
#pragma unroll
        for (int mb = MB0; mb < MB1; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) s[mb][j] = __builtin_fmaf(s[mb][j], cs, mb ? a1 : a0);
    }
    v8bf vfa[2][4];
    read_v(MB0, vfa);                              // lands while the softmax runs
    __builtin_amdgcn_sched_barrier(0);

    // keys past the end of the sequence (only in the last key block)
    if (valid0 < 32 || valid1 < 32) {
        int h4 = half * 4;
        asm volatile("" : "+v"(h4));       // keeps the sixteen per-lane key indices from being hoisted out of the loop
#pragma unroll
        for (int mb = MB0; mb < MB1; ++mb) {
            const int valid = mb ? valid1 : valid0;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if ((j >> 2) * 8 + h4 + (j & 3) >= valid) s[mb][j] = -INFINITY;
        }
    }

    v8bf pf[2][2];
    v2bf ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;
    auto exps = [&](float& lsum) {
#pragma unroll
        for (int mb = MB0; mb < MB1; ++mb)
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
        for (int mb = MB0; mb < MB1; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[mb][j]);
        mx = max_across_halves(mx);        // finite: the first active sub-block of a chunk starts a key block
        const float delta = first ? mx : fmaxf(mx, 0.f);
        const float alpha = __builtin_amdgcn_exp2f(-delta);
        st.m_ref += delta;
        st.l_part *= alpha;
#pragma unroll
        for (int mb = MB0; mb < MB1; ++mb)
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

    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int db = 0; db < 4; ++db)
            st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfa[t][db], pf[MB0][t], st.o[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (MBM == 3) {
        read_v(1, vfa);                            // same registers: their first contents were consumed at issue
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < 4; ++db)
                st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfa[t][db], pf[1][t], st.o[db], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// grid: (ceil(N / 128) * H * B) in one dimension, dealt to the XCDs as contiguous runs (see the Bs = 128 kernel).
// kExact as in the Bs = 128 kernel: false = fast pass over every group, leaving per-wave range flags; true = the
// flagged groups again with the exponent scale applied in fp32.
template <int BS, bool kExact>
__device__ __forceinline__ void attn_small_body(const AttnArgs& a) {
    constexpr int L = kRowsPerGroup / BS;          // CSR rows per workgroup: 2 or 4
    constexpr int kWavesPerRow = kWaves / L;       // 2 or 1
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    constexpr int kXcds = 8;
    const int N = a.td.N;
    const int groups = (N + kRowsPerGroup - 1) / kRowsPerGroup;
    const int total_items = groups * a.td.H * a.td.B;
    const int per_xcd = (total_items + kXcds - 1) / kXcds;
    const int item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (item >= total_items) return;
    if constexpr (kExact) {
        const int4 f = *reinterpret_cast<const int4*>(a.flags + (int64_t)item * 4);
        if (__builtin_amdgcn_readfirstlane(f.x | f.y | f.z | f.w) == 0) return;
    }
    const int qg = item % groups, h = (item / groups) % a.td.H, b = item / (groups * a.td.H);
    const int64_t row_bytes = a.td.stride_n * 2;
    const int64_t head_off = ((int64_t)b * a.td.stride_b + (int64_t)h * a.td.stride_h) * 2;
    const char* Qh = reinterpret_cast<const char*>(a.Q) + head_off;
    const char* Kh = reinterpret_cast<const char*>(a.K) + head_off;
    const char* Vh = reinterpret_cast<const char*>(a.V) + head_off;
    const int mh = (a.mask_heads == 1) ? 0 : h;
    const int32_t* rp = a.rowptr + ((int64_t)b * a.mask_heads + mh) * (a.Sb + 1);
    const float cs = kExact ? 1.0f : kExpScale;
    const int q_wave0 = qg * kRowsPerGroup + wave * 32;
    v8bf qf[8];
    {
        const int qrow = min(q_wave0 + l32, N - 1);
        const char* src = Qh + (int64_t)qrow * row_bytes + half * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const v8bf raw = *reinterpret_cast<const v8bf*>(src + ks * 32);
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[ks][i] = (__bf16)((float)raw[i] * cs);
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
    rd.k_base = lds0 + l32 * kRowBytes + ((half ^ (l32 & 15)) << 4);
    {
        const int v_e = (lane & 15) >> 2, v_c = lane & 3, v_grp = (lane >> 4) & 1;
        const int r0 = half * 4 + v_e;
        const int piece = v_grp * 2 + (v_c >> 1);
        rd.v_base = lds0 + r0 * kRowBytes + ((piece ^ (v_e << 2)) << 4) + (v_c & 1) * 8;
    }

    State st;
    st.m_ref = 0.f;
    st.l_part = 0.f;
    bool first = true;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) st.o[db][j] = 0.f;

    // ---- the group's pre-merged list: entry = key block | (rows listing it) << 28, through a 64-entry register window ----
    const int gmask = (a.mask_heads == 1) ? 0 : h;
    const int64_t gid = ((int64_t)b * a.mask_heads + gmask) * groups + qg;
    const int first_row = min(qg * L, a.Sb);
    const int64_t goff = min(max((int64_t)__builtin_amdgcn_readfirstlane(rp[first_row]), (int64_t)0), a.colidx_stride);   // as in k_group_union
    const int32_t* gl = a.gcol + ((int64_t)b * a.mask_heads + gmask) * a.colidx_stride + goff;
    const int cnt = __builtin_amdgcn_readfirstlane(a.gcount[gid]);
    int pos = 0;
    int win = (cnt > 0) ? gl[min(lane, cnt - 1)] : 0;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));
    asm volatile("" : "+v"(win));
    auto next_entry = [&](int& kb, uint32_t& rows) {
        if (pos >= cnt) { kb = kNoBlock; rows = 0; return; }
        const uint32_t e = (uint32_t)__builtin_amdgcn_readlane(win, pos & 63);
        kb = min((int)(e & 0x0fffffffu), a.Sb - 1);
        rows = e >> 28;
        ++pos;
        if ((pos & 63) == 0 && pos < cnt) {
            win = gl[min(pos + lane, cnt - 1)];
            asm volatile("" : "+v"(win));
        }
    };
    auto fetch = [&]() {
        Chunk c;
        next_entry(c.kb0, c.rows0);
        c.valid = c.kb0 != kNoBlock;
        c.kb1 = -1;
        c.rows1 = 0;
        if (BS == 32 && c.valid) {
            next_entry(c.kb1, c.rows1);
            if (c.kb1 == kNoBlock) { c.kb1 = -1; c.rows1 = 0; }
        }
        if (BS == 64) c.rows1 = c.rows0;
        return c;
    };
    auto issue0 = [&](const Chunk& c) {
        if (BS == 64) { issue_part<0>(lp, Kh, Vh, c.kb0 * 64, 0, N - 1); issue_part<0>(lp, Kh, Vh, c.kb0 * 64 + 32, 1, N - 1); }
        else { issue_part<0>(lp, Kh, Vh, c.kb0 * 32, 0, N - 1); issue_part<0>(lp, Kh, Vh, (c.kb1 >= 0 ? c.kb1 : c.kb0) * 32, 1, N - 1); }
    };
    auto issue1 = [&](const Chunk& c) {
        if (BS == 64) { issue_part<1>(lp, Kh, Vh, c.kb0 * 64, 0, N - 1); issue_part<1>(lp, Kh, Vh, c.kb0 * 64 + 32, 1, N - 1); }
        else { issue_part<1>(lp, Kh, Vh, c.kb0 * 32, 0, N - 1); issue_part<1>(lp, Kh, Vh, (c.kb1 >= 0 ? c.kb1 : c.kb0) * 32, 1, N - 1); }
    };
    const int my_row = wave / kWavesPerRow;
    // A wavefront that owns only one half of a Bs = 32 chunk still runs the full body, the other half's logit
    // accumulators starting from -inf (probabilities 0, finite V): one body variant keeps the kernel inside its
    // register budget; the price is the idle half's matrix instructions.
    auto run_chunk = [&](auto stage_tag, const Chunk& c, auto&& issue) {
        constexpr int STAGE = decltype(stage_tag)::value;
        const int mbm = (int)((c.rows0 >> my_row) & 1u) | (int)(((c.rows1 >> my_row) & 1u) << 1);
        const int valid0 = N - c.kb0 * BS;
        if (BS == 64) {
            if (mbm == 3) chunk_body<STAGE, 3, kExact>(rd, qf, st, first, valid0, valid0 - 32, 0.f, 0.f, 0u, half, issue);
            else issue();
        } else {
            const int valid1 = (c.kb1 >= 0) ? N - c.kb1 * BS : 32;
            if (mbm != 0)
                chunk_body<STAGE, 3, kExact>(rd, qf, st, first, valid0, valid1, (mbm & 1) ? 0.f : -INFINITY,
                                     (mbm & 2) ? 0.f : -INFINITY, 0u, half, issue);
            else issue();
        }
    };

    Chunk cur = fetch();
    if (cur.valid) {
        issue0(cur);
        DR_WAIT_VMCNT0();
        // invariant at each barrier: every wave has waited for its share of the chunk about to be consumed and has
        // finished reading the previous one, whose stage the next loads overwrite
        while (true) {
            Chunk nxt = fetch();
            DR_BARRIER();
            run_chunk(std::integral_constant<int, 0>{}, cur, [&]() { if (nxt.valid) issue1(nxt); });
            DR_WAIT_VMCNT0();
            if (!nxt.valid) break;
            cur = nxt;
            nxt = fetch();
            DR_BARRIER();
            run_chunk(std::integral_constant<int, 1>{}, cur, [&]() { if (nxt.valid) issue0(nxt); });
            DR_WAIT_VMCNT0();
            if (!nxt.valid) break;
            cur = nxt;
        }
    }

    // ---- epilogue ----
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

// Pre-pass: the ascending union of the L consecutive CSR rows of every group (L = 128 / Bs for the kernels of this
// file, L = 256 / Bs for the kernels that walk 256 queries per workgroup), one entry per key block with the
// set of rows that list it in the top four bits (L = 8: the top eight).  A group's entries are written at the colidx offset of its first row
// (the union is never longer than the rows together), its length to gcount.  Indices are clamped to [0, Sb); an
// index listed twice in a row counts once.
// grid: (groups, mask_heads, B).  LDS: L * words presence bitmaps.
template <int L>
__global__ __launch_bounds__(256) void k_group_union(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                     int64_t colidx_stride, int Sb, int groups,
                                                     int32_t* __restrict__ gcol, int32_t* __restrict__ gcount) {
    extern __shared__ uint32_t pres[];                 // [L][words]
    __shared__ int s_wave[4];
    const int g = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
    const int masks = gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int words = (Sb + 31) / 32;
    const int64_t mask_id = (int64_t)b * masks + m;
    const int32_t* rp = rowptr + mask_id * (Sb + 1);
    const int32_t* ci = colidx + mask_id * colidx_stride;
    for (int i = tid; i < L * words; i += 256) pres[i] = 0u;
    __syncthreads();
    const int row0 = min(g * L, Sb), row1 = min(g * L + L, Sb);
    for (int l = 0; l < row1 - row0; ++l) {
        const int lim = (int)min(colidx_stride, (int64_t)0x7fffffff);       // clipped to this mask's colidx array
        const int beg = min(max(rp[row0 + l], 0), lim), end = min(max(rp[row0 + l + 1], beg), lim);
        for (int i = beg + tid; i < end; i += 256) {
            const int kb = min(max(ci[i], 0), Sb - 1);
            atomicOr(&pres[l * words + (kb >> 5)], 1u << (kb & 31));
        }
    }
    __syncthreads();
    const int64_t off0 = min(max((int64_t)rp[row0], (int64_t)0), colidx_stride);
    int32_t* out = gcol + mask_id * colidx_stride + off0;
    const int64_t room = colidx_stride - off0;             // a well-formed CSR never needs more; a malformed one is cut
    int base = 0;
    for (int w0 = 0; w0 < words; w0 += 256) {
        const int wi = w0 + tid;
        uint32_t any = 0u, r[L];
#pragma unroll
        for (int l = 0; l < L; ++l) {
            r[l] = (wi < words) ? pres[l * words + wi] : 0u;
            any |= r[l];
        }
        const int c = __popc(any);
        int incl = c;
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int wave_base = 0, total = 0;
        for (int i = 0; i < 4; ++i) {
            if (i < wave) wave_base += s_wave[i];
            total += s_wave[i];
        }
        int posn = base + wave_base + incl - c;
        uint32_t bits = any;
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            uint32_t rows = 0;
#pragma unroll
            for (int l = 0; l < L; ++l) rows |= ((r[l] >> bit) & 1u) << l;
            if (posn < room) out[posn] = (int32_t)((uint32_t)(wi * 32 + bit) | (rows << (L > 4 ? 24 : 28)));
            ++posn;
        }
        base += total;
        __syncthreads();
    }
    if (tid == 0) gcount[mask_id * groups + g] = (int)max((int64_t)0, min((int64_t)base, room));
}

// Both block sizes fit two workgroups per CU (256 registers per wave) without spilling into the loop; a spill reload
// there would wait on the tile loads in flight.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_mfma_bs64(AttnArgs a) {
    attn_small_body<64, false>(a);
}
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_mfma_bs32(AttnArgs a) {
    attn_small_body<32, false>(a);
}
// the second pass over flagged groups: rare, so its register count (and occupancy) is left to the compiler
__global__ __launch_bounds__(kThreads) void k_attn_mfma_bs64_exact(AttnArgs a) { attn_small_body<64, true>(a); }
__global__ __launch_bounds__(kThreads) void k_attn_mfma_bs32_exact(AttnArgs a) { attn_small_body<32, true>(a); }

template <class Kern>
hipError_t launch_small(Kern kern, Kern kern_exact, const AttnArgs& a, hipStream_t s) {
    for (Kern k : {kern, kern_exact}) {
        hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (attr != hipSuccess) return attr;
    }
    const int groups = (a.td.N + kRowsPerGroup - 1) / kRowsPerGroup;
    {
        hipError_t e = launch_group_union(kRowsPerGroup / a.Bs, a, s);
        if (e != hipSuccess) return e;
    }
    const int total = groups * a.td.H * a.td.B;
    const int grid = (total + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), kLdsBytes, s, a);
    if (a.flags) hipLaunchKernelGGL(kern_exact, dim3(grid), dim3(kThreads), kLdsBytes, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_group_union(int L, const AttnArgs& a, hipStream_t s) {
    if ((L != 2 && L != 4 && L != 8) || !a.gcol || !a.gcount) return hipErrorInvalidValue;
    if (a.Sb >= (L > 4 ? (1 << 24) : (1 << 28))) return hipErrorInvalidValue;      // the key block must fit below the owner bits
    const int groups = (a.Sb + L - 1) / L;
    const size_t lds = (size_t)L * ((a.Sb + 31) / 32) * 4;
    if (lds > 160 * 1024) return hipErrorInvalidValue;          // L presence bitmaps of Sb bits each must fit the LDS of a CU
    const dim3 grid(groups, a.mask_heads, a.td.B);
    auto launch = [&](auto kern) -> hipError_t {
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, a.rowptr, a.colidx, a.colidx_stride, a.Sb, groups, a.gcol, a.gcount);
        return hipGetLastError();
    };
    if (L == 8) return launch(k_group_union<8>);
    if (L == 4) return launch(k_group_union<4>);
    return launch(k_group_union<2>);
}

bool attn_mfma_small_supported(const AttnArgs& a) {
    return a.bf16 && a.td.d == kD && (a.Bs == 32 || a.Bs == 64) && a.td.stride_n * 2 * kChunkKeys < (1ll << 31);
}

// The second pass alone (the 128-row groups flagged in a.flags, with fp32 exponent scaling), behind a fast pass that
// another kernel has made: the merged lists of the groups are rebuilt first, a.gcol / a.gcount may hold others.
hipError_t launch_attn_mfma_small_second_pass(const AttnArgs& a, hipStream_t s) {
    if (!attn_mfma_small_supported(a) || !a.flags) return hipErrorNotSupported;
    hipError_t e = launch_group_union(kRowsPerGroup / a.Bs, a, s);
    if (e != hipSuccess) return e;
    auto kern = a.Bs == 32 ? k_attn_mfma_bs32_exact : k_attn_mfma_bs64_exact;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int groups = (a.td.N + kRowsPerGroup - 1) / kRowsPerGroup;
    const int total = groups * a.td.H * a.td.B;
    hipLaunchKernelGGL(kern, dim3((total + 7) / 8 * 8), dim3(kThreads), kLdsBytes, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_mfma_small(const AttnArgs& a, hipStream_t s) {
    if (!attn_mfma_small_supported(a)) return hipErrorNotSupported;
    return a.Bs == 32 ? launch_small(k_attn_mfma_bs32, k_attn_mfma_bs32_exact, a, s)
                      : launch_small(k_attn_mfma_bs64, k_attn_mfma_bs64_exact, a, s);
}

}  // namespace dr
