// Stage (b): candidate geometry, per-row selection and CSR emission.  gfx950 only.
//
//   k_class_map  integer interval arithmetic on the radial window (paper Eqs. 3, 6, 7 and the
//                density rule); one wavefront classifies one (query block, key block) pair,
//                lanes own columns, ballots count active columns.
//   k_select     one workgroup per (batch, mask, query block) row: compacts the selectable
//                blocks into LDS as 64-bit keys (score descending, key block ascending), then
//                static top-k: radix selection of the k-th smallest key, keep every key up to it
//                (paper Eq. 8 k rule); dynamic: bitonic sort and the cumulative-mass prefix
//                (keep-one fallback of Eq. 11 / Algorithm 1).
//                In the seeded uniform mode (Eq. 8 as worded in the paper) the key is a
//                counter-based hash of (seed, query block, key block) instead of the score.
//   k_select_zscore  the paper's dynamic rule (Eqs. 10-11) per row: lanes own candidate sets
//                (frame distance, side), standardise the scores of a set in fp64 and keep
//                z >= tau_1 / tau_2, with the keep-one fallback.
//   k_emit       per row: offset = sum of the previous rows' counts, bit-expansion to
//                ascending key-block indices.
#include "dr_internal.h"

namespace dr {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// grid: (Sb)   one workgroup per query block, waves stride over key blocks
__global__ __launch_bounds__(kThreads) void k_class_map(Geometry g, FrameTab tab, uint8_t* __restrict__ class_map,
                                                        int32_t* __restrict__ row_sel,
                                                        unsigned long long* __restrict__ totals) {
    __shared__ int s_sel, s_cand;
    const int qb = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = lane_id();
    if (threadIdx.x == 0) { s_sel = 0; s_cand = 0; }
    __syncthreads();
    const int r0 = qb * g.Bs, r1 = min(g.N, r0 + g.Bs);
    const int i0 = r0 / g.Nt, i1 = (r1 - 1) / g.Nt;
    const int row_min = (r1 - r0 == g.Bs) ? g.row_min_full : g.row_min_tail;
    int n_sel = 0, n_cand = 0;
    for (int kb = wave; kb < g.Sb; kb += kWaves) {
        const int c0 = kb * g.Bs, c1 = min(g.N, c0 + g.Bs);
        const int j0 = c0 / g.Nt, j1 = (c1 - 1) / g.Nt;
        const int gap = max(0, max(j0 - i1, i0 - j1));
        int cls;
        if (gap <= 1) {
            cls = 3;
        } else {
            int n_active = 0;
            for (int cbase = 0; cbase < c1 - c0; cbase += 64) {
                const int col = cbase + lane;
                bool active = false;
                if (col < c1 - c0) {
                    const int q = c0 + col;
                    const int j = q / g.Nt, v = q - j * g.Nt;
                    int cnt = 0;
                    for (int i = i0; i <= i1; ++i) {
                        const int t = abs(i - j);
                        if (tab.flags[t] & 1) {
                            const int w = tab.w[t];
                            const int u_lo = max(r0, i * g.Nt) - i * g.Nt;
                            const int u_hi = min(r1, (i + 1) * g.Nt) - 1 - i * g.Nt;
                            cnt += max(0, min(u_hi, v + w) - max(u_lo, v - w) + 1);
                        }
                    }
                    active = cnt >= row_min;
                }
                n_active += __popcll(__ballot(active));
            }
            const int col_min = (c1 - c0 == g.Bs) ? g.col_min_full : g.col_min_tail;
            cls = (n_active >= col_min) ? ((tab.flags[gap] >> 1) & 3) : 0;
        }
        if (lane == 0) class_map[(int64_t)qb * g.Sb + kb] = (uint8_t)cls;
        n_cand += (cls != 0);
        n_sel += (cls == 1 || cls == 2);
    }
    if (lane == 0) { atomicAdd(&s_sel, n_sel); atomicAdd(&s_cand, n_cand); }
    __syncthreads();
    if (threadIdx.x == 0) {
        row_sel[qb] = s_sel;
        atomicAdd(&totals[0], (unsigned long long)s_cand);
        atomicMax(&totals[1], (unsigned long long)s_sel);
    }
}

// Sort key, ascending order == (NEAR before FAR when ranked separately), score descending, kb ascending.
//   bit 63      far flag (only when the two classes are ranked separately)
//   bits 62..31 bitwise complement of the order-preserving integer image of the score
//   bits 30..0  key-block index
__device__ __forceinline__ uint64_t make_key(float s, int kb, bool far_bit) {
    s = s + 0.0f;                                  // -0 -> +0
    uint32_t u = __float_as_uint(s);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending unsigned == ascending float
    u = ~u;                                        // descending
    return ((uint64_t)(far_bit ? 1 : 0) << 63) | ((uint64_t)u << 31) | (uint64_t)(uint32_t)kb;
}
__device__ __forceinline__ float key_score(uint64_t key) {
    uint32_t u = ~(uint32_t)(key >> 31);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __uint_as_float(u);
}
__device__ __forceinline__ int key_block(uint64_t key) { return (int)(key & 0x7fffffffu); }

// MurmurHash3's 32-bit finaliser; the sample key of block pair (qb, kb) under a seed
__device__ __forceinline__ uint32_t fmix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint64_t make_sample_key(uint32_t seed, int qb, int kb, bool far_bit) {
    const uint32_t h = fmix32(fmix32(seed ^ fmix32((uint32_t)qb)) + (uint32_t)kb);
    return ((uint64_t)(far_bit ? 1 : 0) << 63) | ((uint64_t)h << 31) | (uint64_t)(uint32_t)kb;
}

// keep bitmask of one row -> global memory, and the row's count
__device__ __forceinline__ void store_row(const uint32_t* keep, int words, int64_t row, uint32_t* __restrict__ keepbits,
                                          int32_t* __restrict__ counts, int* s_cnt) {
    int c = 0;
    for (int i = threadIdx.x; i < words; i += kThreads) {
        const uint32_t wv = keep[i];
        keepbits[row * words + i] = wv;
        c += __popc(wv);
    }
    for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off);
    if (lane_id() == 0) atomicAdd(s_cnt, c);
    __syncthreads();
    if (threadIdx.x == 0) counts[row] = *s_cnt;
}

__device__ __forceinline__ int keep_count(int n, double ratio) {
    if (n == 0) return 0;
    const int k = (int)floor((double)n * ratio);
    return max(1, k);
}

// The k-th smallest (k = 1 .. n) of n distinct 64-bit keys in LDS: most-significant-digit-first radix selection,
// eight bits per pass.  A pass counts, among the keys that agree with the digits fixed so far, how many fall in each
// of the 256 values of the next digit (thread t owns bin t), scans the counts and descends into the bin that holds
// rank k.  O(n) per pass instead of the O(n log^2 n) of a full sort: the static rules only need the set of the k
// smallest keys, not their order.  All threads of the workgroup call it and all receive the key.
__device__ uint64_t kth_smallest(const uint64_t* keys, int n, int k, uint32_t* hist, int* s_wave, int* s_pick) {
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    uint64_t prefix = 0ull, mask = 0ull;
    int rank = k;
    for (int shift = 56; shift >= 0; shift -= 8) {
        hist[tid] = 0u;
        __syncthreads();
        for (int i = tid; i < n; i += kThreads) {
            const uint64_t key = keys[i];
            if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        const int h = (int)hist[tid];
        int incl = h;
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        for (int i = 0; i < wave; ++i) incl += s_wave[i];
        if (incl - h < rank && rank <= incl) { s_pick[0] = tid; s_pick[1] = rank - (incl - h); }
        __syncthreads();
        prefix |= (uint64_t)(uint32_t)s_pick[0] << shift;
        mask |= 0xffull << shift;
        rank = s_pick[1];
    }
    return prefix;
}

// grid: (Sb, masks, B).  LDS: keys[sort_cap] u64 | mass[sort_cap] f64 (dynamic mode) | keep[words] u32
__global__ __launch_bounds__(kThreads) void k_select(const uint8_t* __restrict__ class_map,
                                                     const float* __restrict__ scores, int masks, int Sb,
                                                     SelectArgs a, uint32_t* __restrict__ keepbits,
                                                     int32_t* __restrict__ counts) {
    extern __shared__ unsigned char smem[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(smem);
    double* mass = reinterpret_cast<double*>(smem + (size_t)a.sort_cap * 8);
    const int words = (Sb + 31) / 32;
    uint32_t* keep = reinterpret_cast<uint32_t*>(smem + (size_t)a.sort_cap * (a.mode == 1 ? 16 : 8));
    __shared__ int s_n, s_near, s_k, s_cnt;

    const int qb = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int64_t row = ((int64_t)b * masks + m) * Sb + qb;
    const float* srow = scores + row * Sb;
    const uint8_t* crow = class_map + (int64_t)qb * Sb;

    for (int i = tid; i < words; i += kThreads) keep[i] = 0u;
    if (tid == 0) { s_n = 0; s_near = 0; s_k = 0x7fffffff; s_cnt = 0; }
    __syncthreads();
    for (int kb = tid; kb < Sb; kb += kThreads) {
        const int c = crow[kb];
        if (c == 3) {
            atomicOr(&keep[kb >> 5], 1u << (kb & 31));
        } else if (c != 0) {
            const int pos = atomicAdd(&s_n, 1);
            const bool far_bit = a.two_ratio && c == 2;
            if (a.two_ratio && c == 1) atomicAdd(&s_near, 1);
            keys[pos] = (a.mode == 3) ? make_sample_key(a.seed, qb, kb, far_bit) : make_key(srow[kb], kb, far_bit);
        }
    }
    __syncthreads();
    const int n = s_n;
    if (n > 0 && a.mode != 1) {
        // static top-k / seeded sample: keep the k smallest keys (with two ratios: the k_near smallest NEAR keys and the
        // k_far smallest FAR keys; every NEAR key is below every FAR key)
        __shared__ uint32_t s_hist[kThreads];
        __shared__ int s_wave4[kWaves], s_pick[2];
        const int n_near = a.two_ratio ? s_near : n;
        const int k_near = keep_count(n_near, a.ratio);
        const int k_far = a.two_ratio ? keep_count(n - n_near, a.ratio_far) : 0;
        const uint64_t none = 0ull;
        const uint64_t t_near = k_near > 0 ? kth_smallest(keys, n, k_near, s_hist, s_wave4, s_pick) : none;
        const uint64_t t_far = k_far > 0 ? kth_smallest(keys, n, n_near + k_far, s_hist, s_wave4, s_pick) : none;
        for (int i = tid; i < n; i += kThreads) {
            const uint64_t key = keys[i];
            const bool far_key = (key >> 63) != 0;
            const bool sel = far_key ? (k_far > 0 && key <= t_far) : (k_near > 0 && key <= t_near);
            if (sel) { const int kb = key_block(key); atomicOr(&keep[kb >> 5], 1u << (kb & 31)); }
        }
    } else if (n > 0) {
        int P = 1;
        while (P < n) P <<= 1;
        for (int i = n + tid; i < P; i += kThreads) keys[i] = ~0ull;
        __syncthreads();
        for (int k = 2; k <= P; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = tid; i < P; i += kThreads) {
                    const int ixj = i ^ j;
                    if (ixj > i) {
                        const uint64_t x = keys[i], y = keys[ixj];
                        const bool up = (i & k) == 0;
                        if ((x > y) == up) { keys[i] = y; keys[ixj] = x; }
                    }
                }
                __syncthreads();
            }
        }
        {
            const double top = (double)key_score(keys[0]);
            for (int i = tid; i < n; i += kThreads) mass[i] = exp((double)key_score(keys[i]) - top);
            __syncthreads();
            if (tid == 0) {          // one-by-one summation in the total order: the order is part of the definition
                double cum = 0.0;
                int i = 0;
                for (; i + 8 <= n; i += 8) {          // eight loads in flight, then the dependent chain of additions
                    double v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = mass[i + e];
#pragma unroll
                    for (int e = 0; e < 8; ++e) { cum = cum + v[e]; v[e] = cum; }
#pragma unroll
                    for (int e = 0; e < 8; ++e) mass[i + e] = v[e];
                }
                for (; i < n; ++i) { cum = cum + mass[i]; mass[i] = cum; }
            }
            __syncthreads();
            const double target = a.tau * mass[n - 1];
            for (int i = tid; i < n; i += kThreads)
                if (mass[i] >= target && (i == 0 || !(mass[i - 1] >= target))) atomicMin(&s_k, i + 1);
            __syncthreads();
            const int k = max(1, min(n, s_k));
            for (int i = tid; i < k; i += kThreads) {
                const int kb = key_block(keys[i]);
                atomicOr(&keep[kb >> 5], 1u << (kb & 31));
            }
        }
    }
    __syncthreads();
    store_row(keep, words, row, keepbits, counts, &s_cnt);
}

// Static top-k / seeded sample for rows of at most 1024 key blocks: ONE wave per row, four rows per workgroup, no
// barrier.  Lane l holds the keys of key blocks l, l + 64, ... in registers, complemented (kSlots 64-bit values; 0
// where there is no key).  The classes arrive as lane masks (k_class_bits), so counting the selectable and the FAR
// keys, dropping the others and adding the forced ones are scalar operations on those masks.  The rules need the SET
// of the k smallest keys, not their order, and the keys are distinct, so any threshold that exactly k complemented
// keys reach describes it.  The threshold is built bit by bit from the top: with the bits kept so far and the next
// one set, count the keys that reach it -- per register one unsigned compare into a lane mask and a population
// count, nothing is rewritten; keep the bit when at least k do, and stop as soon as exactly k do (at the highest bit
// in which the k-th and the (k+1)-th key differ: 15 to 20 steps on real scores).  Only when keys with equal high
// words straddle rank k (equal scores) does the search go on in the low words of that group; the key-index bits
// above log2(Sb) are equal in every key and take no vote.  For a small k the search runs on a short list of one
// register instead (kth_smallest_wave_short_list).  A ballot of "selected" over the wave IS the pair of keep words
// of those 64 key blocks.  Same keys, same counts as k_select: the keep bitmaps are identical.  With one workgroup
// per row, k_select holds 8 rows per CU in flight, each waiting on its barriers; this holds up to 32.
// grid: ceil(B * masks * Sb / 4).
constexpr int kWaveSelectMaxSlots = kWaveSelectMaxBlocks / 64;
constexpr int64_t kWaveSelectMinRows = 1;
constexpr int64_t kWaveSelectPackRows = 2048;
static_assert(kWaveSelectMaxSlots <= 64, "one bit per slot in a 64-bit word");

template <int kSlots>
struct WaveKeys {
    uint64_t c[kSlots];                           // ~key; 0 = no key here
};

// selected <=> the complemented key, as a 64-bit number, is at least (hi, lo); never (0, 0)
struct WaveThreshold {
    uint32_t hi, lo;
};

template <int kSlots>
__device__ __forceinline__ WaveThreshold kth_smallest_wave(const WaveKeys<kSlots>& w, int k, int index_bits) {
    uint32_t t_hi = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t t = t_hi | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < kSlots; ++i) cnt += __popcll(__ballot((uint32_t)(w.c[i] >> 32) >= t));
        if (cnt == k) return WaveThreshold{t, 0u};    // wave-uniform
        if (cnt > k) t_hi = t;
    }
    // t_hi is the high word of the k-th largest complemented key, and more keys than rank k asks for share it
    int above = 0;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) above += __popcll(__ballot((uint32_t)(w.c[i] >> 32) > t_hi));
    const int k_low = k - above;
    uint32_t t_lo = 0x7fffffffu & ~((1u << index_bits) - 1u);   // ones in every key: the index bits no key block has
    auto vote = [&](uint32_t bit_mask) -> bool {
        const uint32_t t = t_lo | bit_mask;
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < kSlots; ++i)
            cnt += __popcll(__ballot((uint32_t)(w.c[i] >> 32) == t_hi && (uint32_t)w.c[i] >= t));
        if (cnt >= k_low) t_lo = t;
        return cnt == k_low;
    };
    if (vote(1u << 31)) return WaveThreshold{t_hi, t_lo};
    for (int bit = index_bits - 1; bit >= 0; --bit)
        if (vote(1u << bit)) break;
    return WaveThreshold{t_hi, t_lo};
}

// The same answer for a small k, by way of a short list.  The k-th largest of the 64 lanes' own maxima is a lower
// bound of the k-th largest key, so the keys that reach it hold the k largest; when they are at most 64 (a few more
// than k on real scores) they are packed one per lane through `list` (64 words of LDS that belong to this wave)
// and the search runs on one register instead of kSlots.  Only the high words take part in the bound, so keys with
// equal high words all make the list.  Returns false, with nothing decided, when the list would not fit or fewer
// than k lanes hold a key.
constexpr int kShortListMaxK = 40;

template <int kSlots>
__device__ __forceinline__ bool kth_smallest_wave_short_list(const WaveKeys<kSlots>& w, int k, int index_bits,
                                                             uint64_t* list, WaveThreshold* out) {
    uint32_t lane_max = 0u;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) lane_max = max(lane_max, (uint32_t)(w.c[i] >> 32));
    uint32_t bound = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t t = bound | (1u << bit);
        const int cnt = __popcll(__ballot(lane_max >= t));
        if (cnt >= k) bound = t;
        if (cnt == k) break;
    }
    if (bound == 0u) return false;
    uint64_t reach[kSlots];
    int listed = 0;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        reach[i] = __ballot((uint32_t)(w.c[i] >> 32) >= bound);
        listed += __popcll(reach[i]);
    }
    if (listed > 64) return false;
    if (listed == k) {                            // the list is the answer
        *out = WaveThreshold{bound, 0u};
        return true;
    }
    int at = 0;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        const int mine = at + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(reach[i] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)reach[i], 0u));
        if (__builtin_amdgcn_inverse_ballot_w64(reach[i])) list[mine] = w.c[i];
        at += __popcll(reach[i]);
    }
    // the wave's LDS operations execute in order; the fence keeps the compiler from moving the read above the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    WaveKeys<1> shortlist;
    shortlist.c[0] = (lane_id() < listed) ? list[lane_id()] : 0ull;
    __builtin_amdgcn_wave_barrier();
    // more keys than k are listed, so the threshold found lies above the bound and counts the same keys in the row
    *out = kth_smallest_wave<1>(shortlist, k, index_bits);
    return true;
}

// The class map as lane masks, for the one-wave-per-row selection: class_bits[qb][slot][3] holds, for the 64 key
// blocks of a slot, one bit per key block: selectable (NEAR or FAR), FAR, forced.  A row has `slots` entries, the
// register slots of the selection kernel that will read it; those past the row's end are 0.  Written once per
// geometry.  grid: ceil(Sb / 4); one wave per row.
__global__ __launch_bounds__(kThreads) void k_class_bits(const uint8_t* __restrict__ class_map, int Sb, int slots,
                                                         uint64_t* __restrict__ class_bits) {
    const int lane = lane_id(), qb = blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (qb >= Sb) return;
    for (int i = 0; i < slots; ++i) {
        const int kb = i * 64 + lane;
        const int c = (kb < Sb) ? class_map[(int64_t)qb * Sb + kb] : 0;
        const uint64_t sel = __ballot(c == 1 || c == 2), far = __ballot(c == 2), forced = __ballot(c == 3);
        if (lane < 3) class_bits[((int64_t)qb * slots + i) * 3 + lane] = lane == 0 ? sel : lane == 1 ? far : forced;
    }
}

// ascending unsigned == ascending float, -0 counted as +0
__device__ __forceinline__ uint32_t score_image(float s) {
    const uint32_t u = __float_as_uint(s + 0.0f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}

template <int kSlots>
__global__ __launch_bounds__(kThreads) void k_select_wave(const uint64_t* __restrict__ class_bits,
                                                          const float* __restrict__ scores, int64_t rows_total, int Sb,
                                                          SelectArgs a, uint32_t* __restrict__ keepbits,
                                                          int32_t* __restrict__ counts) {
    __shared__ uint64_t s_list[kWaves][64];                       // a wave's short list of candidate keys
    const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;   // the same in every lane, and known to be
    if (row >= rows_total) return;
    const int qb = (int)(row % Sb);
    const float* srow = scores + row * Sb;
    const int words = (Sb + 31) / 32;
    const uint64_t* cb = class_bits + (int64_t)qb * (kSlots * 3);
    int index_bits = 0;
    while ((1 << index_bits) < Sb) ++index_bits;

    // every load of the row is issued before the first is used: the scores of all kSlots * 64 positions (those past
    // the row's end read its last entry) and the lane masks of the classes
    float sc[kSlots];
    if (a.mode != 3) {
#pragma unroll
        for (int i = 0; i < kSlots; ++i) sc[i] = srow[(uint32_t)min(i * 64 + lane, Sb - 1)];
    } else {
#pragma unroll
        for (int i = 0; i < kSlots; ++i) sc[i] = 0.f;
    }
    uint64_t m_sel[kSlots], m_far[kSlots], m_forced[kSlots];
    const uint64_t ranked_apart = a.two_ratio ? ~0ull : 0ull;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        m_sel[i] = cb[i * 3 + 0];
        m_far[i] = cb[i * 3 + 1] & ranked_apart;
        m_forced[i] = cb[i * 3 + 2];
    }
    // complemented key of key block kb: (not FAR) << 63 | image << 31 | ~kb (31 bits), the image being the order-preserving
    // integer of the score (or the complement of the sample hash); 0 where the class selects nothing
    WaveKeys<kSlots> w;
    int n = 0, n_far = 0;
    const uint32_t seed_row = (a.mode == 3) ? fmix32(a.seed ^ fmix32((uint32_t)qb)) : 0u;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        const int kb = i * 64 + lane;
        const uint32_t v = (a.mode == 3) ? ~fmix32(seed_row + (uint32_t)kb) : score_image(sc[i]);
        const bool selectable = __builtin_amdgcn_inverse_ballot_w64(m_sel[i]);
        const bool far_key = __builtin_amdgcn_inverse_ballot_w64(m_far[i]);
        const uint32_t hi = (v >> 1) | (far_key ? 0u : 0x80000000u), lo = (v << 31) | (0x7fffffffu ^ (uint32_t)kb);
        w.c[i] = selectable ? (((uint64_t)hi << 32) | lo) : 0ull;
        n += __popcll(m_sel[i]);
        n_far += __popcll(m_far[i]);
    }
    WaveThreshold t_near{0u, 0u}, t_far{0u, 0u};
    int k_near = 0, k_far = 0;
    if (n > 0) {
        const int n_near = n - n_far;                               // m_far is empty unless the classes rank apart
        k_near = keep_count(n_near, a.ratio);
        k_far = a.two_ratio ? keep_count(n_far, a.ratio_far) : 0;
        uint64_t* list = s_list[wave];
        if (k_near > 0 && !(k_near <= kShortListMaxK && kth_smallest_wave_short_list<kSlots>(w, k_near, index_bits, list, &t_near)))
            t_near = kth_smallest_wave<kSlots>(w, k_near, index_bits);
        const int k_all = n_near + k_far;
        if (k_far > 0 && !(k_all <= kShortListMaxK && kth_smallest_wave_short_list<kSlots>(w, k_all, index_bits, list, &t_far)))
            t_far = kth_smallest_wave<kSlots>(w, k_all, index_bits);
    }
    // a NEAR key's complement has bit 63 set and so has every threshold of the NEAR ranking: no FAR key reaches it;
    // the FAR ranking's threshold is reached by every NEAR key and by the k_far best FAR keys.  With nothing to rank
    // the threshold is beyond every key.
    const uint64_t c_near = k_near > 0 ? (((uint64_t)t_near.hi << 32) | t_near.lo) : ~0ull;
    const uint64_t c_far = k_far > 0 ? (((uint64_t)t_far.hi << 32) | t_far.lo) : ~0ull;
    int kept = 0;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        uint64_t m = m_forced[i] | __ballot(w.c[i] >= c_near);
        if (a.two_ratio) m |= __ballot(w.c[i] >= c_far) & m_far[i];
        kept += __popcll(m);
        if (lane < 2 && 2 * i + lane < words) keepbits[row * words + 2 * i + lane] = lane ? (uint32_t)(m >> 32) : (uint32_t)m;
    }
    if (lane == 0) counts[row] = kept;
}

// grid: (Sb, masks, B).  A candidate set of the row is identified by the frame f that realises its gap: the key
// blocks whose first frame is f (f after the query block) or whose last frame is f (f before it); they lie in the
// key-block range of frame f, at most `maxlen` blocks.
// LDS: keep[words] u32 | tile[maxlen][Nf] f32.  All threads first scatter the row's selectable scores into the tile,
// position inside the set's range major, frame minor (reads of the row coalesced, the frame arithmetic once per key
// block); a lane then walks "its" frame's column: neighbouring lanes read neighbouring LDS words, and nothing in the
// serial part touches global memory.  Cells that hold no member keep a sentinel (a NaN pattern; scores are finite).
// The host refuses geometries whose tile does not fit the LDS (beyond about a million tokens at block size 32).
// The three passes over a set run in ascending key-block order, one addition at a time, with floating-point
// contraction off: the summation order and the absence of fused multiply-adds are part of the definition the
// results are compared against.  A cell outside the set adds +0.0, which leaves the running sums bit for bit as they
// are (they start at +0.0 and so are never -0.0), so the loops carry no branch.
// The threshold test is the quotient (s - mu) / (sigma + eps) >= tau in IEEE double.  A division costs about ten
// double-precision instructions, so the quotient is first estimated with a reciprocal (relative error <= 2^-52);
// only when the estimate lies within 2^-50 |tau| of tau is the division itself evaluated.
constexpr uint32_t kNoMember = 0x7fc0dead;

__global__ __launch_bounds__(kThreads) void k_select_zscore(const uint8_t* __restrict__ class_map,
                                                            const float* __restrict__ scores, int masks, int Sb,
                                                            int maxlen, SelectArgs a, uint32_t* __restrict__ keepbits,
                                                            int32_t* __restrict__ counts) {
#pragma clang fp contract(off)
    extern __shared__ unsigned char smem[];
    const int words = (Sb + 31) / 32;
    uint32_t* keep = reinterpret_cast<uint32_t*>(smem);
    uint32_t* tile = reinterpret_cast<uint32_t*>(smem + (size_t)words * 4);     // [maxlen][Nf], score bits
    __shared__ int s_cnt;
    const int qb = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int64_t row = ((int64_t)b * masks + m) * Sb + qb;
    const float* srow = scores + row * Sb;
    const uint8_t* crow = class_map + (int64_t)qb * Sb;
    for (int i = tid; i < words; i += kThreads) keep[i] = 0u;
    if (tid == 0) s_cnt = 0;
    for (int i = tid; i < maxlen * a.Nf; i += kThreads) tile[i] = kNoMember;
    __syncthreads();
    const int r0 = qb * a.Bs, r1 = min(a.N, r0 + a.Bs);
    const int i0 = r0 / a.Nt, i1 = (r1 - 1) / a.Nt;
    for (int kb = tid; kb < Sb; kb += kThreads) {
        const int c = crow[kb];
        if (c == 3) atomicOr(&keep[kb >> 5], 1u << (kb & 31));
        if (c == 1 || c == 2) {
            const uint32_t c0 = (uint32_t)kb * (uint32_t)a.Bs;                   // < N <= 2^31 - 1: 32-bit divisions
            const int j0 = (int)(c0 / (uint32_t)a.Nt);
            const int j1 = (int)((min((uint32_t)a.N, c0 + (uint32_t)a.Bs) - 1u) / (uint32_t)a.Nt);
            const int f = j0 > i1 ? j0 : j1;                                     // selectable: j0 > i1 + 1 or j1 < i0 - 1
            const int pos = kb - (int)(((uint32_t)f * (uint32_t)a.Nt) / (uint32_t)a.Bs);
            tile[pos * a.Nf + f] = __float_as_uint(srow[kb]);
        }
    }
    __syncthreads();
    for (int f = tid; f < a.Nf; f += kThreads) {
        const bool after = f > i1 + 1, before = f < i0 - 1;                      // gaps 0 and 1 are the never-pruned zone
        if (!after && !before) continue;
        const int gap = after ? f - i1 : i0 - f;
        const int64_t f_lo = (int64_t)f * a.Nt, f_hi = f_lo + a.Nt;              // tokens of frame f
        const int kb_lo = (int)(f_lo / a.Bs);
        const int len = min(Sb - 1, (int)((f_hi - 1) / a.Bs)) - kb_lo + 1;
        // cell p of the set: score bits, or kNoMember
        auto cell = [&](int p) -> uint32_t { return tile[p * a.Nf + f]; };
        int n = 0;
        double sum = 0.0;
#pragma unroll 4
        for (int p = 0; p < len; ++p) {
            const uint32_t v = cell(p);
            const bool in = v != kNoMember;
            sum = sum + (in ? (double)__uint_as_float(v) : 0.0);
            n += in ? 1 : 0;
        }
        if (n == 0) continue;
        const double mu = sum / (double)n;
        double ssq = 0.0;
#pragma unroll 4
        for (int p = 0; p < len; ++p) {
            const uint32_t v = cell(p);
            const double dlt = (double)__uint_as_float(v) - mu;
            const double sq = dlt * dlt;
            ssq = ssq + (v != kNoMember ? sq : 0.0);
        }
        const double denom = sqrt(ssq / (double)n) + 1e-6;
        const double rcp = 1.0 / denom;
        // every member of the set has the same smallest frame distance (the gap), hence the same decay state
        const double tau = ((a.near_mask[gap >> 6] >> (gap & 63)) & 1ull) ? a.tau_near : a.tau_far;
        // estimates outside [tau_lo, tau_hi] decide by themselves; an infinite tau never needs the division
        const double slack = fabs(tau) != INFINITY ? 8.9e-16 * fabs(tau) + 1e-290 : 0.0;
        const double tau_lo = tau - slack, tau_hi = tau + slack;
        bool any = false;
        int best_p = -1;
        float best_s = 0.f;
#pragma unroll 4
        for (int p = 0; p < len; ++p) {
            const uint32_t v = cell(p);
            if (v == kNoMember) continue;
            const float x = __uint_as_float(v);
            const double dev = (double)x - mu;
            const double est = dev * rcp;
            bool pass = est >= tau;
            if (est >= tau_lo && est <= tau_hi && slack != 0.0) pass = dev / denom >= tau;
            if (pass) { any = true; atomicOr(&keep[(kb_lo + p) >> 5], 1u << ((kb_lo + p) & 31)); }
            if (best_p < 0 || x > best_s) { best_p = p; best_s = x; }
        }
        if (!any) atomicOr(&keep[(kb_lo + best_p) >> 5], 1u << ((kb_lo + best_p) & 31));
    }
    __syncthreads();
    store_row(keep, words, row, keepbits, counts, &s_cnt);
}

// grid: (Sb, masks, B)
// rowptr of every mask: the exclusive prefix of its rows' kept counts, one workgroup per mask (a row used to re-sum
// all earlier counts itself: Sb^2 / 2 reads per mask).  grid: (masks, B).
__global__ __launch_bounds__(kThreads) void k_row_offsets(const int32_t* __restrict__ counts, int masks, int Sb, int shared,
                                                          int32_t* __restrict__ rowptr, int64_t* __restrict__ nnz) {
    __shared__ long long s_wave[kWaves];
    const int m = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t mask_id = (int64_t)b * masks + m;
    const int64_t src = shared ? 0 : mask_id * Sb;
    int32_t* rp = rowptr + mask_id * (Sb + 1);
    long long running = 0;
    for (int base = 0; base < Sb; base += kThreads) {
        const int i = base + tid;
        const long long c = (i < Sb) ? counts[src + i] : 0;
        long long incl = c;
        for (int o = 1; o < 64; o <<= 1) {
            const long long t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        long long wave_base = 0, total = 0;
        for (int w = 0; w < kWaves; ++w) {
            if (w < wave) wave_base += s_wave[w];
            total += s_wave[w];
        }
        if (i < Sb) rp[i] = (int32_t)(running + wave_base + incl - c);
        running += total;
        __syncthreads();
    }
    if (tid == 0) {
        rp[Sb] = (int32_t)running;
        nnz[mask_id] = running;
    }
}

// One workgroup per row: the set bits of its keep bitmap, ascending, written from the row's offset on.
__global__ __launch_bounds__(kThreads) void k_emit(const uint32_t* __restrict__ keepbits, int masks, int Sb, int shared,
                                                   const int32_t* __restrict__ rowptr, int32_t* __restrict__ colidx,
                                                   int64_t capacity) {
    __shared__ int s_wave[kWaves];
    const int qb = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t mask_id = (int64_t)b * masks + m;
    const int64_t src = shared ? 0 : mask_id * Sb;      // shared: one selection (Sb rows) serves every (b, m)
    const int64_t row = src + qb;
    const int words = (Sb + 31) / 32;
    const long long off0 = rowptr[mask_id * (Sb + 1) + qb];      // negative only if the mask outgrew 32-bit offsets
    int32_t* out = colidx + mask_id * capacity;
    long long base = off0;
    for (int w0 = 0; w0 < words; w0 += kThreads) {
        const int wi = w0 + tid;
        const uint32_t wv = (wi < words) ? keepbits[row * words + wi] : 0u;
        const int c = __popc(wv);
        // exclusive prefix of c over the workgroup
        int incl = c;
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int wave_base = 0, total = 0;
        for (int i = 0; i < kWaves; ++i) {
            if (i < wave) wave_base += s_wave[i];
            total += s_wave[i];
        }
        long long pos = base + wave_base + incl - c;
        uint32_t bits = wv;
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            if (pos >= 0 && pos < capacity) out[pos] = wi * 32 + bit;
            ++pos;
        }
        base += total;
        __syncthreads();
    }
}

}  // namespace

// register slots of the selection kernel for a row of Sb key blocks (0: too long for it)
int wave_select_slots(int Sb) {
    const int need = (Sb + 63) / 64;
    for (int s : {2, 4, 8, 12, 16})
        if (need <= s) return s;
    return 0;
}
static_assert(kWaveSelectMaxSlots == 16, "the largest instantiation");

hipError_t launch_class_map(const Geometry& g, const FrameTab& tab, uint8_t* class_map, uint64_t* class_bits,
                            int32_t* row_sel, unsigned long long* totals, hipStream_t s) {
    hipLaunchKernelGGL(k_class_map, dim3(g.Sb), dim3(kThreads), 0, s, g, tab, class_map, row_sel, totals);
    if (class_bits)
        hipLaunchKernelGGL(k_class_bits, dim3((g.Sb + kWaves - 1) / kWaves), dim3(kThreads), 0, s, class_map, g.Sb,
                           wave_select_slots(g.Sb), class_bits);
    return hipGetLastError();
}

hipError_t launch_select(const uint8_t* class_map, const uint64_t* class_bits, const float* scores, int B, int masks,
                         int Sb, const SelectArgs& a, uint32_t* keepbits, int32_t* counts, hipStream_t s) {
    // One wave per row pays when there are more rows than workgroups the chip holds at once (per-head masks), and while
    // a row's keys fit 16 register pairs per lane: measured 15 - 35 % faster than a workgroup per row there, slower
    // beyond 1024 key blocks (registers, one wave per SIMD) and on the few hundred rows of a single fused mask.
    const int64_t rows_total = (int64_t)B * masks * Sb;
    if ((a.mode == 0 || a.mode == 3) && class_bits && Sb <= kWaveSelectMaxBlocks && rows_total >= kWaveSelectMinRows) {
        // few rows: one per workgroup, so that they spread over as many CUs as there are rows
        const int waves = rows_total >= kWaveSelectPackRows ? kWaves : 1;
        const dim3 grid((unsigned)((rows_total + waves - 1) / waves)), block(64 * waves);
        const int slots = wave_select_slots(Sb);
#define DR_SELECT_WAVE(S) \
    hipLaunchKernelGGL(k_select_wave<S>, grid, block, 0, s, class_bits, scores, rows_total, Sb, a, keepbits, counts)
        if (slots == 2) DR_SELECT_WAVE(2);
        else if (slots == 4) DR_SELECT_WAVE(4);
        else if (slots == 8) DR_SELECT_WAVE(8);
        else if (slots == 12) DR_SELECT_WAVE(12);
        else DR_SELECT_WAVE(16);
#undef DR_SELECT_WAVE
        return hipGetLastError();
    }
    const size_t words = (Sb + 31) / 32;
    const size_t lds = (size_t)a.sort_cap * (a.mode == 1 ? 16 : 8) + words * 4;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_select),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_select, dim3(Sb, masks, B), dim3(kThreads), lds, s, class_map, scores, masks, Sb, a,
                       keepbits, counts);
    return hipGetLastError();
}

hipError_t launch_select_zscore(const uint8_t* class_map, const float* scores, int B, int masks, int Sb,
                                const SelectArgs& a, uint32_t* keepbits, int32_t* counts, hipStream_t s) {
    const size_t lds = select_zscore_lds_bytes(Sb, a.Nt, a.Nf, a.Bs);
    if (lds > kSelectZscoreMaxLds) return hipErrorInvalidValue;      // the host layer checks this before calling
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_select_zscore),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const int maxlen = (a.Nt + a.Bs - 1) / a.Bs + 1;          // key blocks that can touch one frame
    hipLaunchKernelGGL(k_select_zscore, dim3(Sb, masks, B), dim3(kThreads), lds, s, class_map, scores, masks, Sb, maxlen,
                       a, keepbits, counts);
    return hipGetLastError();
}

// The same for rows of at most 2048 key blocks (64 bitmap words): one wave per row, no LDS and no barrier; four rows per
// workgroup.  A lane loads one bitmap word; the wave then walks the row 64 key blocks at a time: the two words of that
// stretch are read back as a wave-uniform lane mask, a lane whose bit is set stores its key block at the running
// offset plus the number of set bits below it (v_mbcnt), so that each store instruction writes one contiguous run.
// grid: ceil(B * masks * Sb / 4).
__global__ __launch_bounds__(kThreads) void k_emit_wave(const uint32_t* __restrict__ keepbits, int64_t rows_total, int Sb,
                                                        int shared, const int32_t* __restrict__ rowptr,
                                                        int32_t* __restrict__ colidx, int64_t capacity) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;      // (mask_id, qb) flattened
    if (r >= rows_total) return;
    const int64_t mask_id = r / Sb;
    const int qb = (int)(r - mask_id * Sb);
    const int64_t row = shared ? qb : r;
    const int words = (Sb + 31) / 32;
    const uint32_t wv = (lane < words) ? keepbits[row * words + lane] : 0u;
    long long pos = (long long)rowptr[mask_id * (Sb + 1) + qb];            // negative only past 32-bit offsets
    int32_t* out = colidx + mask_id * capacity;
    const int stretches = (Sb + 63) / 64;
    for (int i = 0; i < stretches; ++i) {                                  // wave-uniform
        const uint32_t lo = __builtin_amdgcn_readlane(wv, 2 * i), hi = __builtin_amdgcn_readlane(wv, 2 * i + 1);
        const uint32_t mine = (lane < 32) ? (lo >> lane) : (hi >> (lane - 32));
        const long long p = pos + (int)__builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
        if ((mine & 1u) && p >= 0 && p < capacity) out[p] = i * 64 + lane;
        pos += __popc(lo) + __popc(hi);
    }
}

hipError_t launch_emit(const uint32_t* keepbits, const int32_t* counts, int B, int masks, int Sb, bool shared,
                       int32_t* rowptr, int32_t* colidx, int64_t capacity, int64_t* nnz, hipStream_t s) {
    hipLaunchKernelGGL(k_row_offsets, dim3(masks, B), dim3(kThreads), 0, s, counts, masks, Sb, shared ? 1 : 0, rowptr, nnz);
    if (Sb <= 64 * 32) {
        const int64_t rows_total = (int64_t)B * masks * Sb;
        const int waves = rows_total >= kWaveSelectPackRows ? kWaves : 1;
        hipLaunchKernelGGL(k_emit_wave, dim3((unsigned)((rows_total + waves - 1) / waves)), dim3(64 * waves), 0, s, keepbits,
                           rows_total, Sb, shared ? 1 : 0, rowptr, colidx, capacity);
    } else {
        hipLaunchKernelGGL(k_emit, dim3(Sb, masks, B), dim3(kThreads), 0, s, keepbits, masks, Sb, shared ? 1 : 0, rowptr,
                           colidx, capacity);
    }
    return hipGetLastError();
}

}  // namespace dr
