// Stage (a): pooled Q/K block means and the block-score map (paper Eq. 9 at block
// granularity, fused-head mean of App. B).  gfx950 only.
//
// k_pool is the HBM-bound part: each workgroup streams one block of Bs token rows
// with 16-byte loads (a wavefront covers whole 256/512-byte rows, so every request
// is fully coalesced), accumulates in fp32 registers and folds the per-thread
// partials through LDS.  k_scores_mfma is an fp32 GEMM over the pooled vectors on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32: fp32 products and accumulation, as the 1e-5 score tolerance asks).
#include "dr_internal.h"

#include <hip/hip_bf16.h>

namespace dr {
namespace {

constexpr int kPoolThreads = 256;

template <bool BF16> struct Vec16;
template <> struct Vec16<true> {
    static constexpr int kElems = 8;
    __device__ static void load(const void* p, float (&f)[8]) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct Vec16<false> {
    static constexpr int kElems = 4;
    __device__ static void load(const void* p, float (&f)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
};

// grid: (Sb, Hs, 2*B); z = 2*b + which.  LDS: rows_per_pass * d floats.
template <bool BF16>
__global__ __launch_bounds__(kPoolThreads) void k_pool(const void* __restrict__ Q, const void* __restrict__ K,
                                                       TensorDesc td, int Hs, int Bs, int Sb,
                                                       float* __restrict__ pooled) {
    constexpr int VE = Vec16<BF16>::kElems;
    constexpr int ES = BF16 ? 2 : 4;
    extern __shared__ float red[];
    const int blk = blockIdx.x, h = blockIdx.y, b = blockIdx.z >> 1, which = blockIdx.z & 1;
    const int d = td.d;
    const int lanes_per_row = d / VE;
    const int rows_per_pass = kPoolThreads / lanes_per_row;
    const int tid = threadIdx.x;
    const int rr = tid / lanes_per_row, cc = (tid % lanes_per_row) * VE;
    const int row0 = blk * Bs;
    const int nrows = min(Bs, td.N - row0);
    const char* base = reinterpret_cast<const char*>(which ? K : Q) +
                       ((int64_t)b * td.stride_b + (int64_t)h * td.stride_h + (int64_t)row0 * td.stride_n + cc) * ES;
    const int64_t row_bytes = td.stride_n * ES;

    float acc[VE];
#pragma unroll
    for (int i = 0; i < VE; ++i) acc[i] = 0.f;
    int r = rr;
    // four rows in flight per thread
    for (; r + 3 * rows_per_pass < nrows; r += 4 * rows_per_pass) {
        float f0[VE], f1[VE], f2[VE], f3[VE];
        Vec16<BF16>::load(base + (int64_t)r * row_bytes, f0);
        Vec16<BF16>::load(base + (int64_t)(r + rows_per_pass) * row_bytes, f1);
        Vec16<BF16>::load(base + (int64_t)(r + 2 * rows_per_pass) * row_bytes, f2);
        Vec16<BF16>::load(base + (int64_t)(r + 3 * rows_per_pass) * row_bytes, f3);
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] += (f0[i] + f1[i]) + (f2[i] + f3[i]);
    }
    for (; r < nrows; r += rows_per_pass) {
        float f0[VE];
        Vec16<BF16>::load(base + (int64_t)r * row_bytes, f0);
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] += f0[i];
    }
#pragma unroll
    for (int i = 0; i < VE; ++i) red[rr * d + cc + i] = acc[i];
    __syncthreads();
    if (tid < d) {
        float s = 0.f;
        for (int j = 0; j < rows_per_pass; ++j) s += red[j * d + tid];
        const int64_t o = ((((int64_t)which * td.B + b) * Hs + h) * Sb + blk) * d + tid;
        pooled[o] = s / (float)nrows;
    }
}

typedef float v16f __attribute__((ext_vector_type(16)));

// scores on the fp32 matrix cores: a workgroup of 2 x 2 waves, each wave WT x WT tiles of v_mfma_f32_32x32x2_f32,
// contraction chunks of 32 staged through LDS.  The instruction contracts two k per issue (lane halves); a lane
// reads four consecutive k of its row with one 16-byte LDS load (k = 4 * half + c within a group of eight) and feeds
// component c to issue c: the k order inside a group is permuted identically for both operands, which a sum does
// not mind.  WT = 2 (128 x 128 outputs per workgroup) for rows of thousands of blocks, WT = 1 below.
constexpr int kMChunk = 32, kMPad = 36;      // row pitch 144 B keeps the 16-byte reads of 32 rows off the same banks

template <int WT>
__global__ __launch_bounds__(256) void k_scores_mfma(const float* __restrict__ pooled, int B, int Hs, int masks,
                                                     int heads_per_mask, int Sb, int d, float scale,
                                                     float* __restrict__ scores) {
    constexpr int TILE = 64 * WT;
    __shared__ __attribute__((aligned(16))) float As[TILE][kMPad];
    __shared__ __attribute__((aligned(16))) float Bs[TILE][kMPad];
    const int bm = blockIdx.z, b = bm / masks, m = bm % masks;
    const int q0 = blockIdx.y * TILE, k0 = blockIdx.x * TILE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wr = (wave >> 1) * 32 * WT, wc = (wave & 1) * 32 * WT;     // this wave's corner inside the tile
    const int h0 = (masks == 1) ? 0 : m;
    v16f acc[WT][WT];
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const int64_t plane = (int64_t)Sb * d;
    constexpr int NV = TILE * 8 / 256;             // float4 per thread and operand in one chunk (TILE rows x 32 floats)
    float4 pa[NV], pb[NV];
    const int chunks_per_head = d / kMChunk, steps = heads_per_mask * chunks_per_head;
    auto fetch = [&](int step) {                   // the next chunk travels in registers while this one is multiplied
        const int hh = step / chunks_per_head, c0 = (step % chunks_per_head) * kMChunk;
        const float* qb = pooled + ((int64_t)b * Hs + h0 + hh) * plane;
        const float* kb = pooled + (((int64_t)B + b) * Hs + h0 + hh) * plane;
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int idx = tid + it * 256;
            const int row = idx >> 3, c4 = (idx & 7) * 4;
            pa[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            pb[it] = pa[it];
            if (q0 + row < Sb) pa[it] = *reinterpret_cast<const float4*>(qb + (int64_t)(q0 + row) * d + c0 + c4);
            if (k0 + row < Sb) pb[it] = *reinterpret_cast<const float4*>(kb + (int64_t)(k0 + row) * d + c0 + c4);
        }
    };
    fetch(0);
    for (int step = 0; step < steps; ++step) {
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int idx = tid + it * 256;
            const int row = idx >> 3, c4 = (idx & 7) * 4;
            *reinterpret_cast<float4*>(&As[row][c4]) = pa[it];
            *reinterpret_cast<float4*>(&Bs[row][c4]) = pb[it];
        }
        __syncthreads();
        if (step + 1 < steps) fetch(step + 1);
#pragma unroll
        for (int g8 = 0; g8 < kMChunk; g8 += 8) {
            float4 a[WT], bb[WT];
#pragma unroll
            for (int i = 0; i < WT; ++i) {
                a[i] = *reinterpret_cast<const float4*>(&As[wr + i * 32 + l32][g8 + 4 * half]);
                bb[i] = *reinterpret_cast<const float4*>(&Bs[wc + i * 32 + l32][g8 + 4 * half]);
            }
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int i = 0; i < WT; ++i)
#pragma unroll
                    for (int j = 0; j < WT; ++j) {
                        const float av = c == 0 ? a[i].x : c == 1 ? a[i].y : c == 2 ? a[i].z : a[i].w;
                        const float bv = c == 0 ? bb[j].x : c == 1 ? bb[j].y : c == 2 ? bb[j].z : bb[j].w;
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                    }
        }
        __syncthreads();
    }
    // accumulator element e of lane (l32, half): row 8 * (e / 4) + 4 * half + e % 4, column l32
    float* out = scores + (int64_t)bm * Sb * Sb;
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            const int kc = k0 + wc + j * 32 + l32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int qr = q0 + wr + i * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                if (qr < Sb && kc < Sb) out[(int64_t)qr * Sb + kc] = acc[i][j][e] * scale;
            }
        }
}

}  // namespace

hipError_t launch_pool(const void* Q, const void* K, bool bf16, const TensorDesc& td, int Hs, int Bs, int Sb,
                       float* pooled, hipStream_t s) {
    const int ve = bf16 ? 8 : 4;
    const int rows_per_pass = kPoolThreads / (td.d / ve);
    const size_t lds = (size_t)rows_per_pass * td.d * sizeof(float);
    dim3 grid(Sb, Hs, 2 * td.B);
    if (bf16)
        hipLaunchKernelGGL(k_pool<true>, grid, dim3(kPoolThreads), lds, s, Q, K, td, Hs, Bs, Sb, pooled);
    else
        hipLaunchKernelGGL(k_pool<false>, grid, dim3(kPoolThreads), lds, s, Q, K, td, Hs, Bs, Sb, pooled);
    return hipGetLastError();
}

hipError_t launch_scores(const float* pooled, int B, int Hs, int masks, int heads_per_mask, int Sb, int d,
                         float* scores, hipStream_t s) {
    const float scale = 1.0f / (sqrtf((float)d) * (float)heads_per_mask);
    const int t128 = (Sb + 127) / 128, t64 = (Sb + 63) / 64;
    // 128 x 128 tiles pay once a row holds thousands of blocks (at 8250 blocks 0.44 against 0.47 ms); below, their
    // rounding up of Sb and the short contraction loop cost more than they save (591 blocks x 40 heads: 66 against 47 us)
    if (Sb >= 4096 && (int64_t)t128 * t128 * B * masks >= 512)
        hipLaunchKernelGGL(k_scores_mfma<2>, dim3(t128, t128, B * masks), dim3(256), 0, s, pooled, B, Hs, masks,
                           heads_per_mask, Sb, d, scale, scores);
    else
        hipLaunchKernelGGL(k_scores_mfma<1>, dim3(t64, t64, B * masks), dim3(256), 0, s, pooled, B, Hs, masks,
                           heads_per_mask, Sb, d, scale, scores);
    return hipGetLastError();
}

}  // namespace dr
