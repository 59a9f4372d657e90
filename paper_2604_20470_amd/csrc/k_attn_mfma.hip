// Stage (c), MFMA path: block-sparse flash-attention forward for bf16, d = 128, Bs = 128
// (paper Eqs. 12-13 with epsilon -> 0).  gfx950 (CDNA4) only.
//
// One workgroup owns one query block (128 rows) of one (batch, head) and walks the CSR row
// of kept key blocks in chunks of 64 keys.  K and V chunks are gathered HBM/L2 -> LDS with
// direct-to-LDS 16-byte loads, double buffered, so the next chunk streams in while the
// current one is consumed.
//
// The logits are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane's
// 16 accumulator values then all belong to ONE query column, so the softmax row statistics
// are plain in-register reductions plus a single exchange with the lane 32 away, and the
// exponentiated tile, packed to bf16, already sits in the B-operand layout of the second
// product O^T += V^T P^T -- no LDS round trip for P.  The contraction index of that second
// product is permuted the same way on both operands: B slot (half h, element i) of step s in
// key sub-block mb is key mb*32 + 16 s + 8 (i/4) + 4 h + i%4.  V^T fragments come from the
// row-major V chunk with the transposing LDS read ds_read_b64_tr_b16 (lane i of a 16-lane
// group receives column i of the 4 x 16 patch addressed by the group).
//
// LDS layouts (row = key, 256 bytes, sixteen 16-byte pieces per row):
//   K chunk: piece p of row r stored at piece p ^ (r & 15)     -> conflict-free ds_read_b128 A operands
//   V chunk: piece p of row r stored at piece p ^ ((r & 3) << 2) -> the 4-row patches of a transposing
//            read fall in distinct 64-byte bank groups
#include "dr_internal.h"

#include <cstdlib>

namespace dr {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kD = 128, kBs = 128;
constexpr int kChunkKeys = 64;
constexpr int kRowBytes = kD * 2;                    // 256
constexpr int kTileBytes = kChunkKeys * kRowBytes;   // 16 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;          // K then V
constexpr int kLdsBytes = 2 * kStageBytes;           // two stages: 64 KB
constexpr int kPieces = kTileBytes / 1024;           // 1 KB wave-wide load instructions per operand tile

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform).
// Issued through inline assembly so that the compiler's wait-count insertion does not see an LDS write it
// cannot disambiguate (it would drain the prefetch before every LDS read); completion is tracked by hand
// with the vmcnt waits in the main loop.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_base) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// The barrier carries no memory fence on purpose: a fence would drain the prefetch of the next
// chunk.  Ordering of the direct-to-LDS loads is enforced by the explicit vmcnt waits below.
#define DR_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// NQ = number of 32-query column blocks per wavefront (1: four waves per workgroup, 2: two waves)
template <int NQ>
struct Cfg {
    static constexpr int kWaves = 4 / NQ;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kLoadsPerChunk = 2 * kPieces / kWaves;   // per wave: K + V pieces
};

template <int NQ>
__device__ __forceinline__ void issue_chunk(const char* Kh, const char* Vh, int64_t row_bytes, int key0, int last_row,
                                            unsigned char* stage, int wave, int lane) {
    const int r_in = lane >> 4, piece = lane & 15;
    const uint32_t stage_addr = lds_addr(stage);
#pragma unroll
    for (int i = 0; i < kPieces / Cfg<NQ>::kWaves; ++i) {
        const int p = wave + i * Cfg<NQ>::kWaves;      // 1 KB piece index = rows 4p .. 4p+3
        const int r = p * 4 + r_in;
        const int row = min(key0 + r, last_row);      // rows past the end re-read the last valid row (masked later)
        const int64_t off = (int64_t)row * row_bytes;
        dma16(Kh + off + ((piece ^ (r & 15)) << 4), __builtin_amdgcn_readfirstlane(stage_addr + p * 1024));
        dma16(Vh + off + ((piece ^ ((r & 3) << 2)) << 4),
              __builtin_amdgcn_readfirstlane(stage_addr + kTileBytes + p * 1024));
    }
}

// max of a value with its copy in the lane 32 away (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ v8bf pack8(const v16f& c, int base, float cs, float mneg, float& sum) {
    v8bf out;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(c[base + i], cs, mneg));
        sum += p;
        out[i] = (__bf16)p;
    }
    return out;
}

// grid: (Sb * H * B) in one dimension.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own
// L2; id -> work item is remapped so that one XCD walks a contiguous run of (batch, head, query block) items:
// the workgroups resident on an XCD at any time are then neighbouring query blocks of one head, whose kept key
// blocks largely coincide (the forced zone of a frame), and their K/V tiles are served from that XCD's L2.
template <int NQ>
__global__ __launch_bounds__(Cfg<NQ>::kThreads) __attribute__((amdgpu_waves_per_eu(NQ == 1 ? 2 : 1, NQ == 1 ? 2 : 1))) void k_attn_mfma(AttnArgs a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    constexpr int kXcds = 8;
    const int total_items = a.Sb * a.td.H * a.td.B;
    const int per_xcd = (total_items + kXcds - 1) / kXcds;
    const int item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (item >= total_items) return;
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
    const int beg = __builtin_amdgcn_readfirstlane(rp[qb]);
    const int end = __builtin_amdgcn_readfirstlane(rp[qb + 1]);

    // Q^T fragments (B operand of S^T = K Q^T): lane holds query l32, channels ks*16 + 8*half .. +7
    const int q_wave0 = qb * kBs + wave * 32 * NQ;
    v8bf qf[NQ][8];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int qrow = min(q_wave0 + nq * 32 + l32, N - 1);
        const char* src = Qh + (int64_t)qrow * row_bytes + half * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[nq][ks] = *reinterpret_cast<const v8bf*>(src + ks * 32);
    }

    v16f o[NQ][4];
    float m_run[NQ], l_part[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_part[nq] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[nq][db][j] = 0.f;
    }
    const float cs = 1.4426950408889634f / sqrtf((float)kD);   // log2(e) / sqrt(d)

    // chunk sequence: every kept block contributes ceil(valid keys / 64) chunks
    const int n_blocks = end - beg;
    const int last_blk_chunks = (N - (a.Sb - 1) * kBs + kChunkKeys - 1) / kChunkKeys;   // 1 or 2
    int total_chunks = 2 * n_blocks;
    if (n_blocks > 0 && __builtin_amdgcn_readfirstlane(ci[end - 1]) == a.Sb - 1) total_chunks += last_blk_chunks - 2;

    auto chunk_key0 = [&](int c) { return __builtin_amdgcn_readfirstlane(ci[beg + (c >> 1)]) * kBs + (c & 1) * kChunkKeys; };

    if (total_chunks > 0) issue_chunk<NQ>(Kh, Vh, row_bytes, chunk_key0(0), N - 1, smem, wave, lane);
    wait_vmcnt<0>();

    // per-lane LDS read offsets
    const int v_e = (lane & 15) >> 2, v_c = lane & 3, v_grp = (lane >> 4) & 1;

    for (int c = 0; c < total_chunks; ++c) {
        unsigned char* stage = smem + (c & 1) * kStageBytes;
        const int key0 = chunk_key0(c);
        // One barrier per chunk: past it, every wave's share of chunk c has landed (each wave waited for its own
        // loads before arriving) and every wave has finished reading chunk c-1, whose stage the next loads reuse.
        DR_BARRIER();
        if (c + 1 < total_chunks)
            issue_chunk<NQ>(Kh, Vh, row_bytes, chunk_key0(c + 1), N - 1, smem + ((c + 1) & 1) * kStageBytes, wave, lane);

        // ---- S^T = K Q^T : [64 keys x 32*NQ queries] ----
        v16f s[NQ][2];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) s[nq][mb][j] = 0.f;
        {
            v8bf kf[2][8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    const int r = mb * 32 + l32;
                    kf[mb][ks] = *reinterpret_cast<const v8bf*>(stage + r * kRowBytes + (((ks * 2 + half) ^ (r & 15)) << 4));
                }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        s[nq][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][ks], qf[nq][ks], s[nq][mb], 0, 0, 0);
        }
        // V^T fragments for the second product: issued now so that they land while the softmax runs
        const unsigned char* vt = stage + kTileBytes;
        v8bf vf[2][2][4];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const int r_lo = mb * 32 + st * 16 + half * 4 + v_e;     // keys r_lo (i<4) and r_lo + 8 (i>=4)
                const int r_hi = r_lo + 8;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const int piece = db * 4 + v_grp * 2 + (v_c >> 1);
                    const int sub = (v_c & 1) * 8;
                    union { struct { v4s a, b; } s2; v8bf v; } u;
                    u.s2.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) v4s*)(vt + r_lo * kRowBytes + ((piece ^ ((r_lo & 3) << 2)) << 4) + sub));
                    u.s2.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) v4s*)(vt + r_hi * kRowBytes + ((piece ^ ((r_hi & 3) << 2)) << 4) + sub));
                    vf[mb][st][db] = u.v;
                }
            }
        __builtin_amdgcn_sched_barrier(0);
        // keys past the end of the sequence (only in the last block)
        const int valid = N - key0;
        if (valid < kChunkKeys) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        if (mb * 32 + (j >> 2) * 8 + half * 4 + (j & 3) >= valid) s[nq][mb][j] = -INFINITY;
        }

        // ---- online softmax, per query column ----
        v8bf pf[NQ][2][2];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            float mx = -INFINITY;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[nq][mb][j]);
            mx = max_across_halves(mx);
            const float m_new = fmaxf(m_run[nq], mx);               // finite: every chunk holds a valid key
            const float alpha = __builtin_amdgcn_exp2f((m_run[nq] - m_new) * cs);
            m_run[nq] = m_new;
            const float mneg = -m_new * cs;
            float sum = 0.f;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int st = 0; st < 2; ++st) pf[nq][mb][st] = pack8(s[nq][mb], st * 8, cs, mneg, sum);
            l_part[nq] = l_part[nq] * alpha + sum;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int j = 0; j < 16; ++j) o[nq][db][j] *= alpha;
            }
        }

        // ---- O^T += V^T P^T ----
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        o[nq][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mb][st][db], pf[nq][mb][st], o[nq][db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);   // keep the wait below the last MFMA issue
        wait_vmcnt<0>();   // this wave's share of chunk c+1 (in flight during the compute above)
    }

    // ---- epilogue: normalise and store O (row = query l32, channels db*32 + (j/4)*8 + 4*half + j%4) ----
    char* Oh = reinterpret_cast<char*>(a.O) + head_off;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float l = l_part[nq] + __shfl_xor(l_part[nq], 32);
        const float inv = (l > 0.f) ? 1.0f / l : 0.f;
        const int qrow = q_wave0 + nq * 32 + l32;
        if (qrow < N && qrow < qb * kBs + kBs) {
            char* dst = Oh + (int64_t)qrow * row_bytes;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    v4bf v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (__bf16)(o[nq][db][g * 4 + i] * inv);
                    *reinterpret_cast<v4bf*>(dst + (db * 32 + g * 8 + half * 4) * 2) = v;
                }
            if (a.lse && half == 0)
                a.lse[((int64_t)b * a.td.H + h) * N + qrow] =
                    (l > 0.f) ? m_run[nq] * (1.0f / sqrtf((float)kD)) + logf(l) : -INFINITY;
        }
    }
}

template <int NQ>
hipError_t launch_t(const AttnArgs& a, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_mfma<NQ>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int total = a.Sb * a.td.H * a.td.B;
    const int grid = (total + 7) / 8 * 8;          // every XCD gets the same number of slots
    hipLaunchKernelGGL((k_attn_mfma<NQ>), dim3(grid), dim3(Cfg<NQ>::kThreads), kLdsBytes, s, a);
    return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) { return a.bf16 && a.td.d == kD && a.Bs == kBs; }

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s) {
    if (!attn_mfma_supported(a)) return hipErrorNotSupported;
    // developer knob: DR_ATTN_NQ=2 selects two waves x 64 query columns per workgroup
    static const int nq = [] { const char* e = getenv("DR_ATTN_NQ"); return (e && e[0] == '2') ? 2 : 1; }();
    return nq == 2 ? launch_t<2>(a, s) : launch_t<1>(a, s);
}

}  // namespace dr
