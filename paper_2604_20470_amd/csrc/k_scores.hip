// Stage (a): pooled Q/K block means and the block-score map (paper Eq. 9 at block
// granularity, fused-head mean of App. B).  gfx950 only.
//
// k_pool is the HBM-bound part: each workgroup streams one block of Bs token rows
// with 16-byte loads (a wavefront covers whole 256/512-byte rows, so every request
// is fully coalesced), accumulates in fp32 registers and folds the per-thread
// partials through LDS.  k_scores is a small fp32 GEMM over the pooled vectors.
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

// scores tile: 64 x 64 outputs per workgroup, 4 x 4 per thread, contraction chunks of 32 through LDS.
constexpr int kTile = 64, kChunk = 32;

// grid: (ceil(Sb/64), ceil(Sb/64), B*masks)
__global__ __launch_bounds__(256) void k_scores(const float* __restrict__ pooled, int B, int Hs, int masks,
                                                int heads_per_mask, int Sb, int d, float scale,
                                                float* __restrict__ scores) {
    __shared__ float As[kChunk][kTile + 4];
    __shared__ float Bt[kChunk][kTile + 4];
    const int bm = blockIdx.z, b = bm / masks, m = bm % masks;
    const int q0 = blockIdx.y * kTile, k0 = blockIdx.x * kTile;
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int h0 = (masks == 1) ? 0 : m;
    float acc[4][4] = {};
    const int64_t plane = (int64_t)Sb * d;
    for (int hh = 0; hh < heads_per_mask; ++hh) {
        const float* qb = pooled + ((int64_t)b * Hs + h0 + hh) * plane;
        const float* kb = pooled + (((int64_t)B + b) * Hs + h0 + hh) * plane;
        for (int c0 = 0; c0 < d; c0 += kChunk) {
            // 64 rows x 32 floats = 512 float4 per operand; two per thread
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int idx = tid + it * 256;
                const int row = idx / 8, c4 = (idx % 8) * 4;
                float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
                if (q0 + row < Sb) va = *reinterpret_cast<const float4*>(qb + (int64_t)(q0 + row) * d + c0 + c4);
                if (k0 + row < Sb) vb = *reinterpret_cast<const float4*>(kb + (int64_t)(k0 + row) * d + c0 + c4);
                As[c4 + 0][row] = va.x; As[c4 + 1][row] = va.y; As[c4 + 2][row] = va.z; As[c4 + 3][row] = va.w;
                Bt[c4 + 0][row] = vb.x; Bt[c4 + 1][row] = vb.y; Bt[c4 + 2][row] = vb.z; Bt[c4 + 3][row] = vb.w;
            }
            __syncthreads();
#pragma unroll
            for (int c = 0; c < kChunk; ++c) {
                const float4 a = *reinterpret_cast<const float4*>(&As[c][ty * 4]);
                const float4 bb = *reinterpret_cast<const float4*>(&Bt[c][tx * 4]);
                const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
            }
            __syncthreads();
        }
    }
    float* out = scores + (int64_t)bm * Sb * Sb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int qr = q0 + ty * 4 + i;
        if (qr >= Sb) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int kc = k0 + tx * 4 + j;
            if (kc < Sb) out[(int64_t)qr * Sb + kc] = acc[i][j] * scale;
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
    const int t = (Sb + kTile - 1) / kTile;
    const float scale = 1.0f / (sqrtf((float)d) * (float)heads_per_mask);
    hipLaunchKernelGGL(k_scores, dim3(t, t, B * masks), dim3(256), 0, s, pooled, B, Hs, masks, heads_per_mask, Sb, d,
                       scale, scores);
    return hipGetLastError();
}

}  // namespace dr
