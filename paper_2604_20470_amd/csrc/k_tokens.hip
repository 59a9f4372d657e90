// Algorithm 1 of the paper in its own order, for small sequences (an evaluation aid beside the block-level path):
//   k_token_scores     proxy score of every token pair (Eq. 9, fused-head mean of App. B) -> fp32 [N, N]
//   k_pair_links       per ordered frame pair (i, j): candidate window (Eq. 7), population mean / std of the scores in
//                      it (Eq. 10), z >= tau_1 / tau_2 by decay state (Eq. 11), keep-one safeguard -> link bytes [N, N]
//   k_aggregate_links  density rule per block pair ("Density control within blocks": a column is active when its
//                      kept-row ratio exceeds theta_c, the block when its active-column ratio exceeds theta_m), plus the
//                      never-pruned t <= 1 zone -> keep bitmaps, which the ordinary CSR emit turns into the mask.
// Definition of the statistics (part of the result, so that masks are bit-exact): fp64; every sum runs column by
// column (query index u ascending inside key column v), then over the column sums with v ascending, one by one, with
// no fused multiply-add.  That order is also the coalesced one: a thread owns a key column, neighbouring threads read
// neighbouring addresses.  gfx950 only.
#include "dr_internal.h"

namespace dr {
namespace {

constexpr int kTile = 64;            // token-score tile (kTile x kTile outputs per workgroup)
constexpr int kChunk = 32;           // channels staged per step
constexpr int kThreads = 256;

__device__ __forceinline__ float load_as_float(const void* base, int64_t idx, bool bf16) {
    if (bf16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx] << 16);
    return reinterpret_cast<const float*>(base)[idx];
}

// grid: (ceil(N / 64), ceil(N / 64), B * masks).  scores[b][m][p][q], fp32 accumulation.
__global__ __launch_bounds__(kThreads) void k_token_scores(const void* __restrict__ Q, const void* __restrict__ K,
                                                           TensorDesc td, int bf16, int masks, int heads_per_mask,
                                                           float scale, float* __restrict__ scores) {
    __shared__ float sq[kChunk][kTile + 1];
    __shared__ float sk[kChunk][kTile + 1];
    const int b = blockIdx.z / masks, m = blockIdx.z % masks;
    const int p0 = blockIdx.y * kTile, q0 = blockIdx.x * kTile;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int hh = 0; hh < heads_per_mask; ++hh) {
        const int h = masks == 1 ? hh : m;
        const int64_t head = (int64_t)b * td.stride_b + (int64_t)h * td.stride_h;
        for (int c0 = 0; c0 < td.d; c0 += kChunk) {
            // 64 rows x 32 channels per operand: thread -> (row = tid / 4, 8 channels)
            const int r = tid >> 2, cc = (tid & 3) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int p = p0 + r, q = q0 + r;
                sq[cc + e][r] = p < td.N ? load_as_float(Q, head + (int64_t)p * td.stride_n + c0 + cc + e, bf16) : 0.f;
                sk[cc + e][r] = q < td.N ? load_as_float(K, head + (int64_t)q * td.stride_n + c0 + cc + e, bf16) : 0.f;
            }
            __syncthreads();
#pragma unroll 8
            for (int c = 0; c < kChunk; ++c) {
                float a[4], bb[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a[i] = sq[c][ty * 4 + i];
                    bb[i] = sk[c][tx * 4 + i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * bb[j];
            }
            __syncthreads();
        }
    }
    float* out = scores + (int64_t)blockIdx.z * td.N * td.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int p = p0 + ty * 4 + i;
        if (p >= td.N) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = q0 + tx * 4 + j;
            if (q < td.N) out[(int64_t)p * td.N + q] = acc[i][j] * scale;
        }
    }
}

#pragma clang fp contract(off)

struct Best {
    float s;
    int idx;      // u * Nt + v, row-major inside the frame pair; -1: none
};
__device__ __forceinline__ Best better(Best a, Best b) {
    if (b.idx < 0) return a;
    if (a.idx < 0) return b;
    if (b.s > a.s || (b.s == a.s && b.idx < a.idx)) return b;
    return a;
}

// grid: (Nf * Nf, masks, B).  LDS: Nt doubles (column sums).
__global__ __launch_bounds__(kThreads) void k_pair_links(const float* __restrict__ scores, FrameTab tab, int N, int Nt,
                                                         int Nf, double tau_near, double tau_far,
                                                         uint8_t* __restrict__ links) {
    extern __shared__ double colsum[];
    __shared__ double s_stat[2];
    __shared__ unsigned long long s_kept;
    __shared__ float s_best_val[kThreads];
    __shared__ int s_best_idx[kThreads];
    const int i = blockIdx.x / Nf, j = blockIdx.x % Nf;
    const int tid = threadIdx.x;
    const int64_t plane = ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * N * N;
    const float* S = scores + plane + (int64_t)i * Nt * N + (int64_t)j * Nt;
    uint8_t* L = links + plane + (int64_t)i * Nt * N + (int64_t)j * Nt;
    const int t = i > j ? i - j : j - i;
    const int flags = tab.flags[t];
    if (t <= 1 || !(flags & 1)) {
        const uint8_t fill = t <= 1 ? 1 : 0;
        for (int u = 0; u < Nt; ++u)
            for (int v = tid; v < Nt; v += kThreads) L[(int64_t)u * N + v] = fill;
        return;
    }
    const int w = tab.w[t];
    const double tau = ((flags >> 1) & 3) == 1 ? tau_near : tau_far;     // class 1 = NEAR (decay length >= block size)
    // ---- mean: column sums (u ascending), then across columns (v ascending)
    for (int v = tid; v < Nt; v += kThreads) {
        const int lo = max(0, v - w), hi = min(Nt - 1, v + w);
        double acc = 0.0;
        for (int u = lo; u <= hi; ++u) acc = acc + (double)S[(int64_t)u * N + v];
        colsum[v] = acc;
    }
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        long long n = 0;
        for (int v = 0; v < Nt; ++v) {
            total = total + colsum[v];
            n += min(Nt - 1, v + w) - max(0, v - w) + 1;
        }
        s_stat[0] = total / (double)n;
        s_stat[1] = (double)n;
        s_kept = 0ull;
    }
    __syncthreads();
    const double mu = s_stat[0];
    // ---- standard deviation, same order
    for (int v = tid; v < Nt; v += kThreads) {
        const int lo = max(0, v - w), hi = min(Nt - 1, v + w);
        double acc = 0.0;
        for (int u = lo; u <= hi; ++u) {
            const double dev = (double)S[(int64_t)u * N + v] - mu;
            const double sq = dev * dev;
            acc = acc + sq;
        }
        colsum[v] = acc;
    }
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        for (int v = 0; v < Nt; ++v) total = total + colsum[v];
        s_stat[0] = sqrt(total / s_stat[1]) + 1e-6;
    }
    __syncthreads();
    const double denom = s_stat[0];
    // ---- threshold, link bytes for the whole Nt x Nt tile, and the best score for the safeguard
    unsigned long long kept = 0;
    Best best{0.f, -1};
    for (int v = tid; v < Nt; v += kThreads) {
        const int lo = max(0, v - w), hi = min(Nt - 1, v + w);
        for (int u = 0; u < Nt; ++u) {
            uint8_t keep = 0;
            if (u >= lo && u <= hi) {
                const float s = S[(int64_t)u * N + v];
                keep = (((double)s - mu) / denom >= tau) ? 1 : 0;
                kept += keep;
                best = better(best, Best{s, u * Nt + v});
            }
            L[(int64_t)u * N + v] = keep;
        }
    }
    if (kept) atomicAdd(&s_kept, kept);
    s_best_val[tid] = best.s;
    s_best_idx[tid] = best.idx;
    __syncthreads();
    if (s_kept != 0ull) return;
    // nothing passed: keep the highest score of the set (first in row-major order on ties)
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if (tid < off) {
            const Best r = better(Best{s_best_val[tid], s_best_idx[tid]}, Best{s_best_val[tid + off], s_best_idx[tid + off]});
            s_best_val[tid] = r.s;
            s_best_idx[tid] = r.idx;
        }
        __syncthreads();
    }
    if (tid == 0 && s_best_idx[0] >= 0) L[(int64_t)(s_best_idx[0] / Nt) * N + (s_best_idx[0] % Nt)] = 1;
}

// grid: (Sb, masks, B).  LDS: words uint32 (the row's keep bitmap).
__global__ __launch_bounds__(kThreads) void k_aggregate_links(const uint8_t* __restrict__ links,
                                                              const uint8_t* __restrict__ class_map, Geometry g,
                                                              uint32_t* __restrict__ keepbits, int32_t* __restrict__ counts) {
    extern __shared__ uint32_t bitmap[];
    __shared__ int s_count;
    const int qb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int words = (g.Sb + 31) / 32;
    const int64_t mask_id = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
    const uint8_t* L = links + mask_id * g.N * g.N;
    for (int i = tid; i < words; i += kThreads) bitmap[i] = 0u;
    if (tid == 0) s_count = 0;
    __syncthreads();
    const int r0 = qb * g.Bs, nr = min(g.Bs, g.N - r0);
    const int row_min = nr == g.Bs ? g.row_min_full : g.row_min_tail;
    int mine = 0;
    for (int kb = wave; kb < g.Sb; kb += kThreads / 64) {
        bool keep;
        if (class_map[(int64_t)qb * g.Sb + kb] == 3) {          // holds a token pair with t <= 1
            keep = true;
        } else {
            const int c0 = kb * g.Bs, nc = min(g.Bs, g.N - c0);
            const int col_min = nc == g.Bs ? g.col_min_full : g.col_min_tail;
            int active = 0;
            for (int c = lane; c < nc; c += 64) {
                int cnt = 0;
                for (int r = 0; r < nr; ++r) cnt += L[(int64_t)(r0 + r) * g.N + c0 + c];
                active += cnt >= row_min ? 1 : 0;
            }
            for (int off = 32; off > 0; off >>= 1) active += __shfl_down(active, off);
            active = __shfl(active, 0);
            keep = active >= col_min;
        }
        if (keep && lane == 0) {
            atomicOr(&bitmap[kb >> 5], 1u << (kb & 31));
            ++mine;
        }
    }
    if (lane == 0 && mine) atomicAdd(&s_count, mine);
    __syncthreads();
    const int64_t row = mask_id * g.Sb + qb;
    for (int i = tid; i < words; i += kThreads) keepbits[row * words + i] = bitmap[i];
    if (tid == 0) counts[row] = s_count;
}

}  // namespace

hipError_t launch_token_scores(const void* Q, const void* K, bool bf16, const TensorDesc& td, int masks,
                               int heads_per_mask, float* scores, hipStream_t s) {
    const int tiles = (td.N + kTile - 1) / kTile;
    const float scale = (float)(1.0 / ((double)heads_per_mask * sqrt((double)td.d)));
    hipLaunchKernelGGL(k_token_scores, dim3(tiles, tiles, td.B * masks), dim3(kThreads), 0, s, Q, K, td, bf16 ? 1 : 0,
                       masks, heads_per_mask, scale, scores);
    return hipGetLastError();
}

hipError_t launch_pair_links(const float* scores, const FrameTab& tab, int B, int masks, int N, int Nt, int Nf,
                             double tau_near, double tau_far, uint8_t* links, hipStream_t s) {
    hipLaunchKernelGGL(k_pair_links, dim3(Nf * Nf, masks, B), dim3(kThreads), (size_t)Nt * sizeof(double), s, scores, tab,
                       N, Nt, Nf, tau_near, tau_far, links);
    return hipGetLastError();
}

hipError_t launch_aggregate_links(const uint8_t* links, const uint8_t* class_map, const Geometry& g, int B, int masks,
                                  uint32_t* keepbits, int32_t* counts, hipStream_t s) {
    const int words = (g.Sb + 31) / 32;
    hipLaunchKernelGGL(k_aggregate_links, dim3(g.Sb, masks, B), dim3(kThreads), (size_t)words * 4, s, links, class_map, g,
                       keepbits, counts);
    return hipGetLastError();
}

}  // namespace dr
