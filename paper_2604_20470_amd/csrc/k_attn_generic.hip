// Stage (c), general path: block-sparse softmax attention (paper Eqs. 12-13, epsilon -> 0)
// for any supported (d, Bs) and for fp32 or bf16 storage, computed in fp32 on the vector
// ALUs.  It is the path for fp32 inputs, where the required accuracy rules out bf16 MFMA,
// and the fallback for shapes the MFMA kernel does not cover.  gfx950 only.
//
// One workgroup owns 32 query rows of one (batch, head, query block) and walks the row's
// key-block list in chunks of 64 keys staged through LDS with an online (running max /
// running sum) softmax.  Thread (r = tid / 8, g = tid % 8) owns row r: eight of the 64
// chunk logits, and d / 8 output channels.
#include "dr_internal.h"

namespace dr {
namespace {

constexpr int kRows = 32;      // query rows per workgroup
constexpr int kChunk = 64;     // keys per LDS stage
constexpr int kThreads = 256;

template <bool BF16>
__device__ __forceinline__ void load_row_to_lds(const void* src, float* dst, int d, int lane_in_row, int lanes) {
    // cooperative copy of one row of d elements by `lanes` threads
    if (BF16) {
        const uint16_t* p = reinterpret_cast<const uint16_t*>(src);
        for (int c = lane_in_row; c < d; c += lanes) dst[c] = __uint_as_float((uint32_t)p[c] << 16);
    } else {
        const float* p = reinterpret_cast<const float*>(src);
        for (int c = lane_in_row; c < d; c += lanes) dst[c] = p[c];
    }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// grid: (Sb * ceil(Bs/32), H, B).  LDS floats: Q[32][d] | K[64][d+1] | V[64][d] | P[32][64]
template <bool BF16, int D>
__global__ __launch_bounds__(kThreads) void k_attn_generic(AttnArgs a) {
    extern __shared__ float lds[];
    float* sQ = lds;
    float* sK = sQ + kRows * D;
    float* sV = sK + kChunk * (D + 1);
    float* sP = sV + kChunk * D;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int DC = D / 8;           // output channels per thread

    const int subs = (a.Bs + kRows - 1) / kRows;
    const int qb = blockIdx.x / subs, sub = blockIdx.x % subs;
    const int h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, r = tid >> 3, g = tid & 7;
    const int N = a.td.N;
    const int q_row0 = qb * a.Bs + sub * kRows;
    const int q_end = min(N, min(qb * a.Bs + a.Bs, q_row0 + kRows));
    if (q_row0 >= q_end) return;                           // partial last block: nothing in this sub-tile
    const int64_t head_off = (int64_t)b * a.td.stride_b + (int64_t)h * a.td.stride_h;
    const char* Qp = reinterpret_cast<const char*>(a.Q) + head_off * ES;
    const char* Kp = reinterpret_cast<const char*>(a.K) + head_off * ES;
    const char* Vp = reinterpret_cast<const char*>(a.V) + head_off * ES;
    const int64_t row_bytes = a.td.stride_n * ES;
    const int mh = (a.mask_heads == 1) ? 0 : h;
    const int32_t* rp = a.rowptr + ((int64_t)b * a.mask_heads + mh) * (a.Sb + 1);
    const int32_t* ci = a.colidx + ((int64_t)b * a.mask_heads + mh) * a.colidx_stride;
    // row range, clipped to the colidx array of this mask (a list cut short by a too small capacity stays in bounds)
    const int lim = (int)min(a.colidx_stride, (int64_t)0x7fffffff);
    const int beg = min(max(rp[qb], 0), lim), end = min(max(rp[qb + 1], beg), lim);

    const bool row_ok = q_row0 + r < q_end;
    if (row_ok) load_row_to_lds<BF16>(Qp + (int64_t)(q_row0 + r) * row_bytes, sQ + r * D, D, g, 8);
    else for (int c = g; c < D; c += 8) sQ[r * D + c] = 0.f;

    const float scale = 1.0f / sqrtf((float)D);
    float m_run = -INFINITY, l_run = 0.f;
    float o[DC];
#pragma unroll
    for (int i = 0; i < DC; ++i) o[i] = 0.f;

    for (int it = beg; it < end; ++it) {
        const int kb = min(max(ci[it], 0), a.Sb - 1);   // clamped: a malformed list cannot address outside K/V
        const int k_blk0 = kb * a.Bs, k_blk1 = min(N, k_blk0 + a.Bs);
        for (int k0 = k_blk0; k0 < k_blk1; k0 += kChunk) {
            const int nk = min(kChunk, k_blk1 - k0);
            __syncthreads();                   // previous chunk fully consumed (also orders the Q stores)
            for (int kr = tid >> 3; kr < kChunk; kr += kThreads / 8) {
                if (kr < nk) {
                    load_row_to_lds<BF16>(Kp + (int64_t)(k0 + kr) * row_bytes, sK + kr * (D + 1), D, g, 8);
                    load_row_to_lds<BF16>(Vp + (int64_t)(k0 + kr) * row_bytes, sV + kr * D, D, g, 8);
                } else {
                    for (int c = g; c < D; c += 8) { sK[kr * (D + 1) + c] = 0.f; sV[kr * D + c] = 0.f; }
                }
            }
            __syncthreads();
            // logits of row r against keys g, g+8, ..., g+56
            float s[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) s[j] = 0.f;
            for (int c = 0; c < D; ++c) {
                const float qv = sQ[r * D + c];
#pragma unroll
                for (int j = 0; j < 8; ++j) s[j] = fmaf(qv, sK[(g + 8 * j) * (D + 1) + c], s[j]);
            }
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                s[j] = (g + 8 * j < nk) ? s[j] * scale : -INFINITY;
                mx = fmaxf(mx, s[j]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 1));
            mx = fmaxf(mx, __shfl_xor(mx, 2));
            mx = fmaxf(mx, __shfl_xor(mx, 4));
            const float m_new = fmaxf(m_run, mx);          // finite: every chunk has at least one valid key
            const float alpha = expf(m_run - m_new);       // exp(-inf) = 0 on the first chunk
            float ps = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float p = expf(s[j] - m_new);
                sP[r * kChunk + g + 8 * j] = p;
                ps += p;
            }
            ps += __shfl_xor(ps, 1);
            ps += __shfl_xor(ps, 2);
            ps += __shfl_xor(ps, 4);
            l_run = l_run * alpha + ps;
            m_run = m_new;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < DC; ++i) o[i] *= alpha;
            for (int k = 0; k < kChunk; ++k) {
                const float p = sP[r * kChunk + k];
#pragma unroll
                for (int i = 0; i < DC; ++i) o[i] = fmaf(p, sV[k * D + g * DC + i], o[i]);
            }
        }
    }
    if (!row_ok) return;
    const float inv = (l_run > 0.f) ? 1.0f / l_run : 0.f;
    char* Op = reinterpret_cast<char*>(a.O) + (head_off + (int64_t)(q_row0 + r) * a.td.stride_n + g * DC) * ES;
#pragma unroll
    for (int i = 0; i < DC; ++i) {
        const float val = o[i] * inv;
        if (BF16) reinterpret_cast<uint16_t*>(Op)[i] = f32_to_bf16_rne(val);
        else reinterpret_cast<float*>(Op)[i] = val;
    }
    if (a.lse && g == 0)
        a.lse[((int64_t)b * a.td.H + h) * N + q_row0 + r] = (l_run > 0.f) ? m_run + logf(l_run) : -INFINITY;
}

template <bool BF16, int D>
hipError_t launch_t(const AttnArgs& a, hipStream_t s) {
    const size_t lds = sizeof(float) * (kRows * D + kChunk * (D + 1) + kChunk * D + kRows * kChunk);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_generic<BF16, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int subs = (a.Bs + kRows - 1) / kRows;
    hipLaunchKernelGGL((k_attn_generic<BF16, D>), dim3(a.Sb * subs, a.td.H, a.td.B), dim3(kThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_generic(const AttnArgs& a, hipStream_t s) {
    if (a.td.d == 64) return a.bf16 ? launch_t<true, 64>(a, s) : launch_t<false, 64>(a, s);
    if (a.td.d == 128) return a.bf16 ? launch_t<true, 128>(a, s) : launch_t<false, 128>(a, s);
    return hipErrorNotSupported;
}

}  // namespace dr
