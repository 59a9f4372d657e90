// Internal declarations shared by the host layer and the gfx950 kernels.
// Nothing here is part of the public ABI (see include/dynamicrad.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dr {

constexpr int kMaxFrames = 256;          // per-t table travels as a kernel argument
constexpr int kMaxSelectablePerRow = 8192;
constexpr int kMaxTokensTokenLevel = 16384;   // the token-level order holds [N, N] matrices
constexpr int kMaxFrameTokensTokenLevel = 4096;

// Per temporal distance t (paper Eqs. 1-6, evaluated on the host in fp64).
struct FrameTab {
    int32_t w[kMaxFrames];       // window half-width of Eq. 3
    uint8_t flags[kMaxFrames];   // bit0: frame distance retained (Eq. 6); bits 1-2: DR_CLASS_* of Eq. 8's cases
};

struct Geometry {
    int32_t N, Nt, Nf, Bs, Sb;
    // smallest integer count c with c / n > theta, for full blocks and for the partial last block
    int32_t row_min_full, row_min_tail;   // theta_c against the number of valid rows
    int32_t col_min_full, col_min_tail;   // theta_m against the number of valid columns
};

struct TensorDesc {
    int64_t stride_b, stride_h, stride_n;   // elements
    int32_t B, H, N, d;
};

// ---- stage (a) -------------------------------------------------------------------------
// pooled[which][b][hs][blk][d] = mean over the valid tokens of block blk; which 0 = Q, 1 = K.
hipError_t launch_pool(const void* Q, const void* K, bool bf16, const TensorDesc& td, int Hs, int Bs, int Sb,
                       float* pooled, hipStream_t s);
// scores[b][m][qb][kb] = (1 / (heads_per_mask * sqrt(d))) * sum_h qbar . kbar
hipError_t launch_scores(const float* pooled, int B, int Hs, int masks, int heads_per_mask, int Sb, int d,
                         float* scores, hipStream_t s);

// ---- stage (b) -------------------------------------------------------------------------
// class_map[qb][kb]; row_sel[qb] = NEAR+FAR count of the row; totals[0] += candidates, totals[1] = max row_sel.
// class_bits (may be NULL; else Sb * wave_select_slots(Sb) * 3 words, for Sb <= kWaveSelectMaxBlocks): the same classes
// as one lane mask per 64 key blocks -- selectable, FAR, forced -- which the one-wave-per-row selection reads.
constexpr int kWaveSelectMaxBlocks = 1024;
int wave_select_slots(int Sb);
hipError_t launch_class_map(const Geometry& g, const FrameTab& tab, uint8_t* class_map, uint64_t* class_bits,
                            int32_t* row_sel, unsigned long long* totals, hipStream_t s);
struct SelectArgs {
    int32_t mode;            // dr_mode: 0 static top-k, 1 cumulative mass, 2 z-score thresholds, 3 seeded uniform sample
    int32_t two_ratio;       // static / uniform: rank NEAR and FAR separately
    double ratio, ratio_far, tau;
    double tau_near, tau_far;   // z-score mode (Eq. 11's tau_1, tau_2)
    int32_t sort_cap;        // power of two >= the largest selectable count of a row
    uint32_t seed;           // uniform mode
    int32_t N, Nt, Nf, Bs;   // geometry, for the candidate sets of the z-score mode
    uint64_t near_mask[kMaxFrames / 64];   // z-score mode: bit t set when the decay length at frame distance t is >= Bs
};
// keepbits[(b*masks+m)*Sb + qb][words], counts[(b*masks+m)*Sb + qb]
hipError_t launch_select(const uint8_t* class_map, const uint64_t* class_bits, const float* scores, int B, int masks,
                         int Sb, const SelectArgs& a, uint32_t* keepbits, int32_t* counts, hipStream_t s);
// z-score mode (paper Eqs. 10-11 at block level); same outputs as launch_select.  Its kernel holds one row's scores
// in LDS as a [key blocks per frame + 1][Nf] tile beside the keep bitmap: geometries beyond the limit are refused.
constexpr size_t kSelectZscoreMaxLds = 144 * 1024;
inline size_t select_zscore_lds_bytes(int Sb, int Nt, int Nf, int Bs) {
    return (size_t)((Sb + 31) / 32) * 4 + (size_t)((Nt + Bs - 1) / Bs + 1) * (size_t)Nf * 4;
}
hipError_t launch_select_zscore(const uint8_t* class_map, const float* scores, int B, int masks, int Sb,
                                const SelectArgs& a, uint32_t* keepbits, int32_t* counts, hipStream_t s);
hipError_t launch_emit(const uint32_t* keepbits, const int32_t* counts, int B, int masks, int Sb, bool shared,
                       int32_t* rowptr, int32_t* colidx, int64_t capacity, int64_t* nnz, hipStream_t s);

// ---- Algorithm 1 in its own order (token-pair selection, then aggregation), small N -----------------
// scores[b][m][p][q] = (1 / (heads_per_mask * sqrt(d))) * sum_h Q_p . K_q
hipError_t launch_token_scores(const void* Q, const void* K, bool bf16, const TensorDesc& td, int masks,
                               int heads_per_mask, float* scores, hipStream_t s);
// links[b][m][p][q] = 1 where the token pair is kept (z-score thresholds inside every frame pair's candidate set)
hipError_t launch_pair_links(const float* scores, const FrameTab& tab, int B, int masks, int N, int Nt, int Nf,
                             double tau_near, double tau_far, uint8_t* links, hipStream_t s);
// density rule per block pair -> the keepbits / counts that launch_emit reads
hipError_t launch_aggregate_links(const uint8_t* links, const uint8_t* class_map, const Geometry& g, int B, int masks,
                                  uint32_t* keepbits, int32_t* counts, hipStream_t s);

// ---- stage (c) -------------------------------------------------------------------------
struct AttnArgs {
    const void *Q, *K, *V;
    void* O;
    float* lse;                  // nullable
    const int32_t* rowptr;       // [B, mask_heads, Sb+1]
    const int32_t* colidx;       // [B, mask_heads, colidx_stride]
    int64_t colidx_stride;
    int32_t mask_heads;
    TensorDesc td;
    int32_t Bs, Sb;
    int32_t bf16;
    // scratch of the small-block MFMA path: per 128-row group the merged key-block list (laid out like colidx) and its length
    int32_t* gcol;               // [B, mask_heads, colidx_stride]
    int32_t* gcount;             // [B, mask_heads, number of groups]
    // scratch of the bf16 MFMA paths: one word per wave of a 128-query work item, non-zero when the fast pass found
    // rows outside the accuracy range of its pre-scaled Q; those items are then taken again with fp32 scaling.
    // NULL: no second pass.
    int32_t* flags;              // [B * H * ceil(N / 128) * 4]
};
// Any d in {64,128}, Bs in {32,64,128}, f32 or bf16 storage; arithmetic in fp32 on the vector ALUs.
hipError_t launch_attn_generic(const AttnArgs& a, hipStream_t s);
// bf16 storage, d = 128, Bs = 128: MFMA path.  Returns hipErrorNotSupported for other shapes.
hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s);
bool attn_mfma_supported(const AttnArgs& a);
// The second pass of launch_attn_mfma alone: the items flagged in a.flags, with fp32 exponent scaling.
hipError_t launch_attn_mfma_second_pass(const AttnArgs& a, hipStream_t s);
// bf16 storage, d = 128, Bs = 128, N >= 64: MFMA path that walks pairs of adjacent query blocks (one wave per SIMD,
// 64 queries per wave); needs gcol / gcount / flags.  Rows it flags must be taken again by the second pass above.
hipError_t launch_attn_mfma_pair(const AttnArgs& a, hipStream_t s);
bool attn_mfma_pair_supported(const AttnArgs& a);
// Merged key-block lists of every group of L (2 or 4) consecutive CSR rows: a.gcol (laid out like colidx, a group's
// entries at the colidx offset of its first row; entry = key block | rows-that-list-it << 28) and a.gcount.
hipError_t launch_group_union(int L, const AttnArgs& a, hipStream_t s);
// bf16 storage, d = 128, Bs = 32 or 64: MFMA path that walks the union of the CSR rows of a 128-query group.
hipError_t launch_attn_mfma_small(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_mfma_small_second_pass(const AttnArgs& a, hipStream_t s);
bool attn_mfma_small_supported(const AttnArgs& a);

// ---- evaluation aid: the proxy objective of the offline search (App. C, Eq. 22) ----------------------
constexpr int kProxySlices = 64;     // partial sums per (b, h): partial is [B * H, kProxySlices, 2] doubles
hipError_t launch_proxy_loss(const float* A_dense, const float* A_sparse, int BH, int N, const int64_t* nnz, int n_masks,
                             int Sb, double target, double alpha, double* partial, double* out, hipStream_t s);

// ---- measurement aid ---------------------------------------------------------------------
// out[0] = shader-clock ticks, out[1] = 100 MHz ticks elapsed over a window of window_ticks (100 MHz units).
hipError_t launch_clock_probe(unsigned long long window_ticks, unsigned long long* out, hipStream_t s);
// MFMA-only loop: workgroups x 4 waves x iters x 8 matrix instructions; shape 32 (32x32x16) or 16 (16x16x32).
hipError_t launch_mfma_probe(int shape, int workgroups, int iters, int random_operands, float* sink, hipStream_t s);
hipError_t launch_mfma_mix_probe(int workgroups, int iters, float* sink, hipStream_t s);

}  // namespace dr
