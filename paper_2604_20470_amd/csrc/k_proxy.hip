// Objective of the paper's offline parameter search on its proxy task (App. C, Eq. 22) as a device reduction:
//   nmse = mean over (b, h) of ||A_dense - A_sparse||_F^2 / ||A_dense||_F^2,
//   loss = nmse + alpha * max(0, target - sparsity),  sparsity = 1 - mean(nnz) / Sb^2.
// Two launches: per (b, h) and slice, fp64 partial sums in a fixed order; then one workgroup folds the slices in
// order and forms the three outputs.  No atomics: the result is the same bits on every run.
#include "dr_internal.h"

namespace dr {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ void block_sum2(double& a, double& b, double* sh) {
    const int tid = threadIdx.x;
    sh[tid] = a;
    sh[kThreads + tid] = b;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (tid < s) {
            sh[tid] += sh[tid + s];
            sh[kThreads + tid] += sh[kThreads + tid + s];
        }
        __syncthreads();
    }
    a = sh[0];
    b = sh[kThreads];
}

// grid (kProxySlices, B * H): slice s of head bh covers elements [s * per, (s + 1) * per) of its N x N matrices.
__global__ __launch_bounds__(kThreads) void k_proxy_partial(const float* __restrict__ ad, const float* __restrict__ as,
                                                            long long nn, double* __restrict__ partial) {
    __shared__ double sh[2 * kThreads];
    const int bh = blockIdx.y, slice = blockIdx.x;
    const long long per = (nn + kProxySlices - 1) / kProxySlices;
    const long long lo = (long long)slice * per, hi = min(nn, lo + per);
    const float* pd = ad + (long long)bh * nn;
    const float* ps = as + (long long)bh * nn;
    double num = 0.0, den = 0.0;
    for (long long i = lo + threadIdx.x; i < hi; i += kThreads) {
        const double d = (double)pd[i], e = d - (double)ps[i];
        num += e * e;
        den += d * d;
    }
    block_sum2(num, den, sh);
    if (threadIdx.x == 0) {
        partial[((long long)bh * kProxySlices + slice) * 2 + 0] = num;
        partial[((long long)bh * kProxySlices + slice) * 2 + 1] = den;
    }
}

__global__ __launch_bounds__(kThreads) void k_proxy_final(const double* __restrict__ partial, int BH,
                                                          const int64_t* __restrict__ nnz, int n_masks, int Sb,
                                                          double target, double alpha, double* __restrict__ out) {
    __shared__ double sh[2 * kThreads];
    double ratio_sum = 0.0, nnz_sum = 0.0;
    for (int bh = threadIdx.x; bh < BH; bh += kThreads) {
        double num = 0.0, den = 0.0;
        for (int s = 0; s < kProxySlices; ++s) {
            num += partial[((long long)bh * kProxySlices + s) * 2 + 0];
            den += partial[((long long)bh * kProxySlices + s) * 2 + 1];
        }
        ratio_sum += den > 0.0 ? num / den : 0.0;
    }
    for (int m = threadIdx.x; m < n_masks; m += kThreads) nnz_sum += (double)nnz[m];
    block_sum2(ratio_sum, nnz_sum, sh);
    if (threadIdx.x == 0) {
        const double nmse = ratio_sum / (double)BH;
        const double sparsity = 1.0 - nnz_sum / (double)n_masks / ((double)Sb * (double)Sb);
        const double short_of = target - sparsity;
        out[0] = nmse + alpha * (short_of > 0.0 ? short_of : 0.0);
        out[1] = nmse;
        out[2] = sparsity;
    }
}

}  // namespace

hipError_t launch_proxy_loss(const float* A_dense, const float* A_sparse, int BH, int N, const int64_t* nnz, int n_masks,
                             int Sb, double target, double alpha, double* partial, double* out, hipStream_t s) {
    const long long nn = (long long)N * N;
    hipLaunchKernelGGL(k_proxy_partial, dim3(kProxySlices, BH), dim3(kThreads), 0, s, A_dense, A_sparse, nn, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_proxy_final, dim3(1), dim3(kThreads), 0, s, partial, BH, nnz, n_masks, Sb, target, alpha, out);
    return hipGetLastError();
}

}  // namespace dr
