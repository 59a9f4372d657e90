/*
 * dynamicrad.h -- C ABI of the DynamicRad attention hot path for AMD MI355X (gfx950).
 *
 * Three stages, each one call (paper: "Two-Mode Intra-Candidate Selection",
 * Algorithm 1, and the masked attention of Eq. 13):
 *
 *   dr_block_scores     pooled Q/K proxy score per (query block, key block)
 *   dr_build_mask       radial candidate geometry + per-row selection -> CSR
 *   dr_sparse_attn_fwd  softmax attention restricted to the kept key blocks
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never frees or reallocates them and keeps no reference after the call's
 *     work on the stream has finished.
 *   - Q, K, V, O are [B, H, N, d] with the innermost d contiguous; the three
 *     outer strides are given in elements and are the same for all four.
 *     Rows must be 16-byte aligned (base pointer and every stride * element
 *     size a multiple of 16).
 *   - Tokens are ordered frame-major: token p sits in frame p / (Hg*Wg) at
 *     in-frame index p % (Hg*Wg) (row-major over the Hg x Wg grid).
 *     N must equal Nf*Hg*Wg.  Blocks of Bs tokens are cut on the global token
 *     index; the last block may be partial (Sb = ceil(N / Bs)).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without a host synchronisation,
 *     except where a call says otherwise (first use of a new geometry).
 *   - After one call with a given shape and parameters (which sizes the context's
 *     scratch and builds the cached geometry) the stage calls only enqueue kernels on
 *     `stream`: no allocation, no host synchronisation, no memset; such a sequence
 *     can be captured in a HIP graph and replayed.  A replay reads the context's caches
 *     (candidate geometry, uniform-rule selection) as they are then: keep a context whose
 *     calls are captured to one geometry and one set of parameters.
 *   - Every call returns a dr_status; nothing is thrown across the boundary.
 *     dr_last_error(ctx) returns the text of the last failure on that context.
 *     Argument errors are detected on the host before anything is launched.
 *   - A dr_ctx owns device scratch and caches; it is bound to one device and
 *     must not be used from two threads at once.  Two calls on different
 *     streams that share one ctx race on its scratch.
 */
#ifndef DYNAMICRAD_H_
#define DYNAMICRAD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dr_ctx dr_ctx;

typedef enum {
    DR_OK = 0,
    DR_ERR_INVALID_ARG = 1,   /* null pointer, inconsistent shape, parameter out of range */
    DR_ERR_UNSUPPORTED = 2,   /* valid request outside what the kernels cover (d, Bs, frame count) */
    DR_ERR_CAPACITY = 3,      /* a caller-provided capacity is too small to even start */
    DR_ERR_HIP = 4,           /* a HIP runtime call failed; text in dr_last_error */
    DR_ERR_NOMEM = 5          /* scratch allocation failed */
} dr_status;

typedef enum { DR_F32 = 0, DR_BF16 = 1 } dr_dtype;

typedef enum {
    DR_MODE_STATIC_RATIO = 0,      /* keep the top max(1, floor(n*rho)) selectable blocks of a row by score */
    DR_MODE_DYNAMIC_THRESHOLD = 1, /* keep the shortest score-descending prefix holding >= tau of the softmax mass */
    DR_MODE_ZSCORE_THRESHOLD = 2,  /* the paper's own dynamic rule: scores standardised per candidate set, kept when
                                      z >= tau_1 (near) / tau_2 (far), keep-one fallback (Eqs. 10-11) */
    DR_MODE_UNIFORM_RATIO = 3      /* the paper's own static rule: a seeded, score-free uniform sample of
                                      max(1, floor(n*rho)) selectable blocks (Eq. 8) */
} dr_mode;

/* Problem shape.  Paper notation: Nf frames, Nt = Hg*Wg tokens per frame, S = N tokens, Bs block size. */
typedef struct {
    int32_t B, H, N, d;            /* batch, heads, tokens, head dim (64 or 128) */
    int32_t Nf, Hg, Wg, Bs;        /* frames, grid rows, grid cols, block size (32, 64 or 128) */
    int32_t dtype;                 /* dr_dtype of Q, K, V, O */
    int32_t reserved0;             /* must be 0 */
    int64_t stride_b, stride_h, stride_n;   /* in elements; stride of d is 1 */
} dr_shape;

/* Mask parameters beyond the per-call ones.  NULL means the defaults below. */
typedef struct {
    double gamma;        /* decay factor of Eq. 2, > 0.  Default 1.0 */
    double theta_c;      /* column density threshold, in [0, 1).  Default 0.15 */
    double theta_m;      /* block activation threshold, in [0, 1).  Default 0.60 */
    double ratio_far;    /* static mode: ratio for far-field blocks (decay length < Bs); < 0: same as ratio.  Default -1 */
    int32_t head_fuse;   /* Hf > 0: scores are the mean over heads 0..Hf-1, one mask per batch element;
                            0: one mask per head.  Default 2 (App. B, head-fusion proxy) */
    int32_t has_tau_far; /* z-score mode: 1 = `tau_far` is the threshold of far-field blocks; 0 = same as near.  Default 0 */
    double tau_far;      /* z-score mode: tau_2 of Eq. 11 (any real, -inf allowed) when has_tau_far = 1.  Default 0 */
    uint32_t seed;       /* uniform mode: seed of the counter-based sample.  Default 0 */
    int32_t reserved[3]; /* must be 0 */
} dr_mask_params;

/* Block classes written by dr_class_map. */
enum { DR_CLASS_NONE = 0, DR_CLASS_NEAR = 1, DR_CLASS_FAR = 2, DR_CLASS_FORCED = 3 };

/* Create / destroy a context on HIP device `device`.  dr_create allocates nothing on the device yet. */
dr_status dr_create(dr_ctx** out, int device);
void dr_destroy(dr_ctx* ctx);
/* Text of the last error on this context ("" if none).  Valid until the next failing call. */
const char* dr_last_error(const dr_ctx* ctx);

/*
 * Candidate geometry of one (shape, lambda, params) as a class byte per block pair.
 * Paper: window width and split rule (Eqs. 1-6), candidate set (Eq. 7), density
 * control (theta_c, theta_m), and the never-pruned t <= 1 zone (Eq. 3, Eq. 8).
 *   class_map  device, [Sb, Sb] bytes, row = query block; DR_CLASS_* values.
 * A block pair is FORCED if any of its token pairs has temporal distance <= 1.
 * Otherwise column c of the pair is active if (#rows r with |u_r - v_c| <= w(t)
 * on a retained frame distance) / (#valid rows) > theta_c, and the pair is a
 * candidate if (#active columns) / (#valid columns) > theta_m; its class is NEAR
 * or FAR by the decay length at the smallest temporal distance inside the pair.
 * Uses Nf, Hg, Wg, Bs, N of `shape` only.  Asynchronous on `stream`.
 */
dr_status dr_class_map(dr_ctx* ctx, const dr_shape* shape, double lambda, const dr_mask_params* params,
                       uint8_t* class_map, void* stream);

/*
 * Number of candidate block pairs (FORCED + NEAR + FAR) of the geometry: an upper
 * bound on nnz of any mask dr_build_mask can emit for it, i.e. a safe colidx
 * capacity per mask.  Synchronous (runs the classification and reads one count back).
 *   max_selectable_per_row  optional (may be NULL): largest NEAR+FAR count of a row.
 */
dr_status dr_mask_capacity(dr_ctx* ctx, const dr_shape* shape, double lambda, const dr_mask_params* params,
                           int64_t* candidate_blocks, int32_t* max_selectable_per_row);

/*
 * Static-ratio selection at a target effective sparsity.  Paper: k = max(1, floor(|P| rho)) of Eq. 8's keep rule;
 * the kept count of a static-ratio row depends on the geometry only (FORCED blocks + max(1, floor(n rho)) of its
 * n selectable blocks), so rho can be fixed before any score exists.  Returns the largest rho = i / 1000,
 * i = 1 .. 1000, whose mask has effective sparsity 1 - kept / Sb^2 >= target (single-ratio rule; the product
 * n * rho is taken in IEEE double).
 *   target    in (0, 1)
 *   ratio     host, receives rho
 *   achieved  host, optional (may be NULL): the effective sparsity at that rho
 * Synchronous (reads the per-row selectable counts of the cached geometry back to the host).
 * Errors: DR_ERR_INVALID_ARG for NULL / out-of-range arguments; DR_ERR_UNSUPPORTED if no rho on the grid
 * reaches the target (the never-pruned zone alone is too large).
 */
dr_status dr_static_ratio_for_sparsity(dr_ctx* ctx, const dr_shape* shape, double lambda, const dr_mask_params* params,
                                       double target, double* ratio, double* achieved);

/*
 * Stage (a).  Paper: proxy score, Eq. 9, with the fused-head mean of App. B, taken
 * at block granularity: score[b, m, qb, kb] = mean over heads of mask m of
 * mean_{p in qb}(Q_p) . mean_{q in kb}(K_q) / sqrt(d), means over valid tokens.
 *   Q, K      device, dtype/strides of `shape`
 *   head_fuse Hf in 1..H: masks = 1 (heads 0..Hf-1 averaged); 0: masks = H
 *   scores    device, float32, contiguous [B, masks, Sb, Sb]
 */
dr_status dr_block_scores(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K,
                          int32_t head_fuse, float* scores, void* stream);

/*
 * Stage (b).  Paper: Algorithm 1 restated per query-block row at block level.
 * For each (b, m, qb): kept = FORCED blocks of the row + a selection among the
 * row's NEAR/FAR blocks (n of them), ordered by score descending, ties by lower
 * key-block index, -0 equal to +0:
 *   static  : the first max(1, floor(n * ratio)) of them (Eq. 8's k rule); with
 *             params->ratio_far >= 0, NEAR and FAR are ranked separately with
 *             `ratio_or_tau` and `ratio_far`.
 *   dynamic : e_j = exp(s_j - max s) in fp64, summed one by one in that order;
 *             the shortest prefix whose sum >= tau * (total sum); at least one
 *             (the keep-one fallback of Eq. 11 / Algorithm 1).
 *   z-score : (Eqs. 10-11 at block level) the row's NEAR/FAR blocks are split into
 *             candidate sets by (smallest frame distance to the query block, side
 *             before/after it) -- the image of the paper's frame pair (i, j).  Per set, in
 *             fp64 with sums taken one by one in ascending key-block order:
 *             mu = mean, sigma = sqrt(mean (s - mu)^2), z = (s - mu) / (sigma + 1e-6);
 *             a block is kept when z >= tau, tau = `ratio_or_tau` for NEAR blocks and
 *             params->tau_far for FAR blocks (if has_tau_far); a set where nothing passes
 *             keeps its highest score (lower index on ties).  The kernel holds a row as a
 *             tile of Nf x (ceil(Hg*Wg / Bs) + 1) scores in LDS: DR_ERR_UNSUPPORTED when that
 *             exceeds 144 KB (beyond about a million tokens at block size 32).
 *   uniform : (Eq. 8 as the paper words it) scores are not read (`scores` may be NULL);
 *             every NEAR/FAR block gets the 32-bit key
 *             fmix32(fmix32(seed ^ fmix32(qb)) + kb), fmix32 = MurmurHash3's finaliser;
 *             the max(1, floor(n * ratio)) smallest keys are kept (ties by lower index);
 *             with params->ratio_far >= 0 NEAR and FAR are sampled separately.  The mask
 *             depends on the geometry, the ratios and the seed only (the same for every b
 *             and every mask head): the context keeps the selection of the last such
 *             call, and a call that repeats it only writes the CSR out.
 * Output is CSR per mask: rowptr[b, m, 0..Sb] (rowptr[..,0] = 0) and strictly
 * ascending key-block indices in colidx[b, m, rowptr[qb] .. rowptr[qb+1]).
 *   mode           dr_mode
 *   ratio_or_tau   ratio in (0, 1] (static, uniform), tau in (0, 1] (dynamic), or tau_1, any real (z-score)
 *   lambda         long-range factor of Eq. 4, > 0
 *   scores         device float32 [B, masks, Sb, Sb] (masks from params->head_fuse); must be finite;
 *                  may be NULL in uniform mode
 *   rowptr         device int32 [B, masks, Sb + 1]
 *   colidx         device int32 [B, masks, colidx_capacity]
 *   colidx_capacity  entries available per mask; > 0
 *   nnz            device int64 [B, masks]: the number of kept blocks, written even when it
 *                  exceeds the capacity.  Entries beyond the capacity are never written; the
 *                  caller must treat a mask with nnz > capacity as invalid.
 * The first call for a new (geometry, lambda, params) builds and caches the class map
 * and synchronises once; later calls are fully asynchronous.
 */
dr_status dr_build_mask(dr_ctx* ctx, const dr_shape* shape, int32_t mode, double ratio_or_tau, double lambda,
                        const dr_mask_params* params, const float* scores,
                        int32_t* rowptr, int32_t* colidx, int64_t colidx_capacity, int64_t* nnz, void* stream);

/*
 * Stage (c).  Paper: Eqs. 12-13 with epsilon -> 0: for every valid query token p of
 * query block qb, O_p = sum_q softmax_q(Q_p . K_q / sqrt(d)) V_q over the valid key
 * tokens q of the key blocks listed in row qb of the CSR; other keys have weight 0.
 * A row with no key block yields O = 0 and lse = -inf.  Non-causal.
 *   Q, K, V, O   device, dtype/strides of `shape` (O is written for valid tokens only)
 *   rowptr, colidx  device CSR as emitted by dr_build_mask; any well-formed CSR with
 *                ascending in-range indices is accepted (e.g. the full mask)
 *   mask_heads   1 (one mask per batch element shared by all heads) or H
 *   colidx_stride  distance in entries between the colidx arrays of consecutive masks
 *   lse          optional device float32 [B, H, N]: natural-log sum-exp of each row's logits
 * bf16 inputs with d = 128 use bf16 MFMA (operands Q * log2(e)/sqrt(d) re-rounded to bf16, K,
 * V and the probabilities rounded to bf16) with fp32 accumulation and fp32 softmax, for every
 * block size; fp32 inputs, and bf16 inputs with d = 64, are computed in fp32 throughout.
 * Accuracy range of the bf16 MFMA path: the second rounding of the scaled Q adds a logit error
 * that grows with |logit|, so every group of 128 query rows that holds a row whose largest
 * logit exceeds 44 in magnitude (64 in units of log2) is computed a second time, by a pass
 * that feeds Q as stored and applies the scale in fp32; that pass overwrites O (and lse) of the
 * group.  Both passes are launched by every call (the second one only steps through the flags
 * when no group was flagged); the flags live in context-owned device scratch (16 bytes per 128
 * query rows and head), grown on demand: DR_ERR_NOMEM if that allocation fails.
 * Out-of-range key-block indices are clamped to [0, Sb) and row ranges are clipped to
 * [0, colidx_stride] (memory safety: a mask that overflowed its capacity is read as far as it
 * was written), neither is reported; a row
 * whose list is not ascending is still summed correctly (softmax does not depend on the order).
 * A key block listed twice in one row is outside the contract (the paths that merge lists count
 * it once, the others once per listing).  For bf16, d = 128 and N >= 64 the call first merges
 * the rows of every two (block size 128), four (64) or eight (32) adjacent query blocks, 256
 * queries, into one key-block list, which one workgroup then walks (block size 32: fewer than
 * 2^24 blocks; environment variable DR_ATTN_PAIRS=0, read when the context is created, keeps one
 * workgroup per 128 query rows instead, which for the block sizes 64 and 32 walks the merged
 * rows of those 128 queries).  The merged lists live in
 * context-owned device scratch of the size of the colidx arrays the call is given
 * (B * mask_heads * colidx_stride entries), grown on demand: DR_ERR_NOMEM if that allocation fails.
 * The pre-pass holds one bitmap of Sb bits per merged row in LDS: DR_ERR_UNSUPPORTED when
 * (256 / Bs) * Sb bits exceed 160 KB (beyond 5 million tokens at block size 32, 84 million at 128).
 * Argument errors (NULL or misaligned pointers, strides, mask_heads) are rejected on the host
 * before any launch; the call itself is asynchronous on `stream`.
 */
dr_status dr_sparse_attn_fwd(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, const void* V,
                             const int32_t* rowptr, const int32_t* colidx, int32_t mask_heads,
                             int64_t colidx_stride, void* O, float* lse, void* stream);

/*
 * dr_sparse_attn_fwd for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the scratch the
 * kernels need beyond their inputs and outputs (range flags of the bf16 MFMA paths; merged key-block lists and
 * their lengths for block sizes 32 / 64 and for the block-size-128 kernel that walks pairs of query blocks) lies in
 * a fixed 16 MiB area of device memory that is part of the library image (one copy per GPU, held until the process
 * ends) instead of context-owned allocations.  The call allocates and frees nothing.
 *   Needed: 16 bytes per 128 query rows and head, plus, on the list-walking paths, 4 bytes per entry of the colidx
 *   arrays given (B * mask_heads * colidx_stride) and 4 bytes per group of rows.  A call that needs more than the
 *   area holds is refused with DR_ERR_UNSUPPORTED (the message gives both figures); use dr_sparse_attn_fwd then.
 * All calls on one GPU share the area, whatever their context: calls that overlap in time on one GPU race on it
 * (calls queued on one stream do not overlap).  Nothing in it has to start at zero: every word a kernel reads was
 * written earlier in the same call.
 * Other errors as dr_sparse_attn_fwd.  DR_ERR_HIP if the area's address could not be resolved when the context
 * was created.
 */
dr_status dr_sparse_attn_fwd_static(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, const void* V,
                                    const int32_t* rowptr, const int32_t* colidx, int32_t mask_heads,
                                    int64_t colidx_stride, void* O, float* lse, void* stream);

/*
 * Algorithm 1 in the paper's own order, for small sequences (an evaluation aid: it shows what the block-level
 * restatement of dr_build_mask changes).  Paper: proxy score of a token pair (Eq. 9), candidate set of a frame
 * pair (Eq. 7), score normalisation inside it (Eq. 10), decay-state thresholds with the keep-one safeguard
 * (Eq. 11), aggregation of the kept links to blocks ("Density control within blocks", last step of Algorithm 1).
 *
 * dr_token_scores: scores[b, m, p, q] = mean over the heads of mask m of Q_p . K_q / sqrt(d), fp32.
 *   Q, K       device, dtype/strides of `shape`
 *   head_fuse  as in dr_block_scores
 *   scores     device, float32, contiguous [B, masks, N, N]
 *   N <= 16384, else DR_ERR_UNSUPPORTED.
 *
 * dr_build_mask_tokens: for every ordered frame pair (i, j), t = |i - j|:
 *   t <= 1: every token pair is a link; t not retained (Eq. 6): none; otherwise over the candidate set
 *   P(i, j) = {(u, v): |u - v| <= w(t)}: mu = mean, sigma = population standard deviation of the scores,
 *   z = (s - mu) / (sigma + 1e-6), link when z >= tau, tau = `tau_near` when the decay length L(t) >= Bs, else
 *   params->tau_far (if has_tau_far, else tau_near); if no pair of the set passes, its highest score is a link
 *   (first in row-major (u, v) order on ties).  Statistics in fp64 with every sum taken column by column (u
 *   ascending inside key column v, then the column sums with v ascending), one by one, no fused multiply-add:
 *   part of the definition, so that masks are reproducible bit for bit.
 *   Then block (qb, kb) is kept when it holds a token pair with t <= 1, or when
 *   #{columns c: #links in column c / #valid rows > theta_c} / #valid columns > theta_m.
 *   token_scores  device, float32, contiguous [B, masks, N, N] (dr_token_scores' output)
 *   rowptr, colidx, colidx_capacity, nnz   as in dr_build_mask; the kept blocks are a subset of the candidate
 *                 blocks, so dr_mask_capacity bounds nnz here too
 *   links         optional device uint8 [B, masks, N, N]: receives the link matrix (1 = kept); NULL: the context
 *                 holds it in scratch of that size (DR_ERR_NOMEM if that allocation fails)
 *   params->gamma, theta_c, theta_m, head_fuse (number of masks), has_tau_far, tau_far are read.
 *   N <= 16384 and Hg * Wg <= 4096, else DR_ERR_UNSUPPORTED.  First use of a geometry synchronises once, like
 *   dr_build_mask.
 */
dr_status dr_token_scores(dr_ctx* ctx, const dr_shape* shape, const void* Q, const void* K, int32_t head_fuse,
                          float* scores, void* stream);
dr_status dr_build_mask_tokens(dr_ctx* ctx, const dr_shape* shape, double tau_near, double lambda,
                               const dr_mask_params* params, const float* token_scores, int32_t* rowptr,
                               int32_t* colidx, int64_t colidx_capacity, int64_t* nnz, uint8_t* links, void* stream);

/*
 * Objective of the paper's offline parameter search on its proxy task (App. C, Eq. 22), as a device reduction:
 *   nmse     = mean over (b, h) of ||A_dense - A_sparse||_F^2 / ||A_dense||_F^2
 *   sparsity = 1 - mean over (b, mask) of nnz / Sb^2      (effective sparsity: pruned fraction of block pairs)
 *   loss     = nmse + alpha * max(0, target - sparsity)
 * The attention matrices are inputs (the hot path does not materialise them; a caller reads them off
 * dr_sparse_attn_fwd with one-hot V columns).
 *   A_dense, A_sparse  device, float32, contiguous [B, H, N, N]
 *   nnz        device int64 [B, masks] as written by dr_build_mask / dr_build_mask_tokens
 *   Sb         number of blocks per side (> 0)
 *   target, alpha      sparsity target and penalty weight of Eq. 22 (the paper uses 0.80 and 10)
 *   out        device float64 [3]: loss, nmse, sparsity
 * All sums are taken in fp64 in a fixed order (per (b, h): one workgroup, each thread over a strided subset, then a
 * tree over the threads), so the result is reproducible run to run.  A (b, h) slice with ||A_dense||_F = 0
 * contributes 0.  Asynchronous on `stream`; allocates nothing.  Errors: DR_ERR_INVALID_ARG for NULL pointers or
 * non-positive sizes.
 */
dr_status dr_proxy_loss(dr_ctx* ctx, const float* A_dense, const float* A_sparse, int32_t B, int32_t H, int32_t N,
                        const int64_t* nnz, int32_t masks, int32_t Sb, double target, double alpha, double* out,
                        void* stream);

/* Library version string, e.g. "dynamicrad-gfx950 0.2". */
const char* dr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DYNAMICRAD_H_ */
