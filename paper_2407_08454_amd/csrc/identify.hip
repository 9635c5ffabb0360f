// Merging-set identification (Section 3.2; Section 4.1 Def. 4.1 and Algorithm 1;
// conserved states: Section 4.1 last paragraph, Section 5.1; pivot: Section 4.2 Eq. (7)).
//
// Kernels:
//   cosine_scan_kernel  streams K once and writes sim[j] = cos(k_{j-1}, k_j) (Eq. (2)) and the
//                       inverse norm of every key; HBM-bound, 16 lanes per 128-wide row,
//                       16 B per lane.
//   anchor_run_kernel   (anchor reading of Algorithm 1 only) for every free token i, how many
//                       free tokens directly below it are similar enough to k_i.
//   segment_kernel      one workgroup per slice: exact top-k of the aggregated scores by
//                       radix select, boundary flags, prefix scan to set ids, the budget
//                       fallback, and a segmented arg-max scan for the pivots.  All integer
//                       outputs are deterministic.
//   segment_reg_kernel  the same for the adjacent rule and up to 16384 tokens with the slice held
//                       in registers (16 tokens per thread)
//   sim_append_kernel   decode time: the one new similarity
//   evict_select_kernel, gather_rows_kernel, gather_merge_values_kernel
//                       comparison workloads (eviction by score; evicted values averaged into the
//                       nearest kept token)
#include "kvm_common.h"

namespace kvm {

// ------------------------------------------------------------------------------------------
// cosine scan
// ------------------------------------------------------------------------------------------

constexpr int COS_BLOCK = 256;
constexpr int COS_GROUPS = COS_BLOCK / 16;                  // 16-lane groups per workgroup
constexpr int COS_ROWS_PER_GROUP = 16;                      // consecutive rows per 16-lane group
constexpr int COS_ROWS_PER_BLOCK = COS_GROUPS * COS_ROWS_PER_GROUP;



template <typename T>
__global__ __launch_bounds__(COS_BLOCK) void cosine_scan_kernel(const T *__restrict__ K, float *__restrict__ sim,
                                                                 float *__restrict__ inv_norm_out,
                                                                 const int32_t *__restrict__ seq_lens, int H, int N,
                                                                 int tiles_per_slice)
{
    typedef typename Elem<T>::Raw Raw;
    __shared__ Raw last_row[COS_GROUPS][16];                // the last row of every group, for its successor

    const int slice = blockIdx.x / tiles_per_slice;
    const int tile = blockIdx.x - slice * tiles_per_slice;
    const int n = clamp_len(seq_lens, slice / H, N);
    const int c = threadIdx.x & 15, group = threadIdx.x >> 4;
    const int j_block = tile * COS_ROWS_PER_BLOCK;
    const int j0 = j_block + group * COS_ROWS_PER_GROUP;
    float *sims = sim + (size_t)slice * N;
    if (j_block >= n) {                                      // padding only: defined zeros, nothing read
        if (c == 0)
            for (int i = 0; i < COS_ROWS_PER_GROUP; ++i)
                if (j0 + i < N) {
                    sims[j0 + i] = 0.f;
                    if (inv_norm_out) inv_norm_out[(size_t)slice * N + j0 + i] = 0.f;
                }
        return;
    }
    const T *Ks = K + (size_t)slice * N * HEAD_DIM;

    // every row of the group at once (rows past the end are replaced by the last valid one and
    // never used), plus the row before the workgroup's first for group 0
    Raw raw[COS_ROWS_PER_GROUP];
#pragma unroll
    for (int i = 0; i < COS_ROWS_PER_GROUP; ++i) raw[i] = Elem<T>::load(Ks + (size_t)min(j0 + i, n - 1) * HEAD_DIM, c);
    Raw prev = raw[0];
    if (group == 0 && j0 >= 1) prev = Elem<T>::load(Ks + (size_t)(j0 - 1) * HEAD_DIM, c);
    last_row[group][c] = raw[COS_ROWS_PER_GROUP - 1];
    __syncthreads();
    if (group > 0) prev = last_row[group - 1][c];

    float r_prev = inv_norm(row16_sum(RowDot<T>::dot(prev, prev)));
#pragma unroll
    for (int i = 0; i < COS_ROWS_PER_GROUP; ++i) {
        const int j = j0 + i;
        const float dot = row16_sum(RowDot<T>::dot(raw[i], prev));
        const float r = inv_norm(row16_sum(RowDot<T>::dot(raw[i], raw[i])));
        // zero norm, first token of the sequence or padding: similarity 0
        const float s = (j > 0 && j < n) ? (dot * r) * r_prev : 0.f;
        if (c == (i & 15) && j < N) {
            sims[j] = s;
            if (inv_norm_out) inv_norm_out[(size_t)slice * N + j] = j < n ? r : 0.f;
        }
        prev = raw[i];
        r_prev = r;
    }
}

// Decode time: only the similarity of the newest token to its predecessor is new.  One 16-lane
// group per slice; nothing but sim[n-1] is written.
template <typename T>
__global__ __launch_bounds__(256) void sim_append_kernel(const T *__restrict__ K, float *__restrict__ sim,
                                                         const int32_t *__restrict__ seq_lens, int H, int N, int slices)
{
    const int slice = blockIdx.x * 16 + (threadIdx.x >> 4);
    if (slice >= slices) return;
    const int c = threadIdx.x & 15;
    const int n = clamp_len(seq_lens, slice / H, N);
    if (n == 0) return;
    float s = 0.f;
    if (n >= 2) {                                            // uniform over the 16 lanes of the group
        const T *Ks = K + (size_t)slice * N * HEAD_DIM;
        const typename Elem<T>::Raw a = Elem<T>::load(Ks + (size_t)(n - 2) * HEAD_DIM, c);
        const typename Elem<T>::Raw b = Elem<T>::load(Ks + (size_t)(n - 1) * HEAD_DIM, c);
        const float dot = row16_sum(RowDot<T>::dot(b, a));
        const float ra = inv_norm(row16_sum(RowDot<T>::dot(a, a))), rb = inv_norm(row16_sum(RowDot<T>::dot(b, b)));
        s = (dot * rb) * ra;                                 // the order of the scan kernel: same bits
    }
    if (c == 0) sim[(size_t)slice * N + n - 1] = s;
}

// ------------------------------------------------------------------------------------------
// anchor rule: run lengths
// ------------------------------------------------------------------------------------------

constexpr int RUN_BLOCK = 256;
constexpr int RUN_ANCHORS_PER_GROUP = 4;                    // anchors a 16-lane group handles in turn
constexpr int RUN_TILE = (RUN_BLOCK / 16) * RUN_ANCHORS_PER_GROUP;
constexpr int RUN_BATCH = 4;                                 // candidate rows in flight per group

// run[i] = number of tokens i-1, i-2, ... directly below the free token i that are free and
// whose cosine similarity to k_i exceeds eps, up to the first one that is not (0 for a
// conserved token).  One 16-lane group per anchor; the rows come from L2, which the
// neighbouring anchors keep warm.  flags bit 0 = conserved.
template <typename T>
__global__ __launch_bounds__(RUN_BLOCK) void anchor_run_kernel(const T *__restrict__ K, const float *__restrict__ inv_norm,
                                                                const uint8_t *__restrict__ flags, int32_t *__restrict__ run,
                                                                const int32_t *__restrict__ seq_lens, int H, int N,
                                                                int tiles_per_slice, float eps)
{
    typedef typename Elem<T>::Raw Raw;
    const int slice = blockIdx.x / tiles_per_slice;
    const int tile = blockIdx.x - slice * tiles_per_slice;
    const int n = clamp_len(seq_lens, slice / H, N);
    const int c = threadIdx.x & 15, group = threadIdx.x >> 4;
    const T *Ks = K + (size_t)slice * N * HEAD_DIM;
    const float *rn = inv_norm + (size_t)slice * N;
    const uint8_t *fl = flags + (size_t)slice * N;
    int32_t *runs = run + (size_t)slice * N;
    for (int a = 0; a < RUN_ANCHORS_PER_GROUP; ++a) {
        const int i = tile * RUN_TILE + a * (RUN_BLOCK / 16) + group;
        if (i >= n) continue;                                // (uniform within the group)
        int count = 0;
        if (!(fl[i] & 1)) {
            const Raw anchor = Elem<T>::load(Ks + (size_t)i * HEAD_DIM, c);
            const float ri = rn[i];
            bool open = true;
            for (int base = i - 1; base >= 0 && open; base -= RUN_BATCH) {
                Raw row[RUN_BATCH];
                float rj[RUN_BATCH];
                bool free_j[RUN_BATCH];
#pragma unroll
                for (int u = 0; u < RUN_BATCH; ++u) {
                    const int j = max(base - u, 0);
                    row[u] = Elem<T>::load(Ks + (size_t)j * HEAD_DIM, c);
                    rj[u] = rn[j];
                    free_j[u] = base - u >= 0 && !(fl[j] & 1);
                }
#pragma unroll
                for (int u = 0; u < RUN_BATCH; ++u) {
                    const float cosv = (row16_sum(RowDot<T>::dot(anchor, row[u])) * ri) * rj[u];
                    open = open && free_j[u] && cosv > eps;
                    count += open ? 1 : 0;
                }
            }
        }
        if (c == 0) runs[i] = count;
    }
}

// ------------------------------------------------------------------------------------------
// segmentation: one workgroup per slice
// ------------------------------------------------------------------------------------------

constexpr int SEG_BLOCK = 1024;
constexpr int SEG_WAVES = SEG_BLOCK / WAVE;
constexpr int SEG_ITEMS = 4;
constexpr int SEG_TILE = SEG_BLOCK * SEG_ITEMS;

struct SegShared {
    int hist[256];
    int wave_i[SEG_WAVES];
    int wave_i2[SEG_WAVES];
    unsigned long long wave_k[SEG_WAVES];
    int wave_f[SEG_WAVES];
    int bc[4];
    unsigned long long bck;
};

__device__ __forceinline__ unsigned long long shfl_up_u64(unsigned long long v, int off) {
    uint32_t lo = __shfl_up((uint32_t)v, off, WAVE), hi = __shfl_up((uint32_t)(v >> 32), off, WAVE);
    return ((unsigned long long)hi << 32) | lo;
}

// Exclusive prefix sum of one int per thread over the block; total returned to all threads.
__device__ __forceinline__ int block_exclusive_sum(int v, int &total, int *wave_slots) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        int t = __shfl_up(inc, off, WAVE);
        if (lane >= off) inc += t;
    }
    __syncthreads();                                         // wave_slots may still be read from a previous use
    if (lane == WAVE - 1) wave_slots[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < SEG_WAVES; ++i) {
        int a = wave_slots[i];
        if (i < w) before += a;
        all += a;
    }
    total = all;
    return before + inc - v;
}

__device__ __forceinline__ int block_sum(int v, int *wave_slots) {
    int total;
    (void)block_exclusive_sum(v, total, wave_slots);
    return total;
}

// k-th largest (k >= 1) of the keys that `key_at(j, key)` accepts for j in [0, count).
// Needs k <= number of accepted keys.  Returns the key value T and the number of accepted
// keys strictly greater than T.  MSB-first radix select, 8 bits per pass.
template <typename KeyFn>
__device__ void block_select_kth_largest(KeyFn key_at, int count, int k, uint32_t &T, int &greater, SegShared &sh)
{
    uint32_t prefix = 0, mask = 0;
    int remaining = k, gt = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = threadIdx.x; i < 256; i += SEG_BLOCK) sh.hist[i] = 0;
        __syncthreads();
        for (int j = threadIdx.x; j < count; j += SEG_BLOCK) {
            uint32_t key;
            if (key_at(j, key) && (key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (threadIdx.x < WAVE) {
            const int lane = threadIdx.x;
            int h[4], s = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { h[i] = sh.hist[lane * 4 + i]; s += h[i]; }
            int suf = s;                                     // inclusive suffix sum over lanes
#pragma unroll
            for (int off = 1; off < WAVE; off <<= 1) {
                int t = __shfl_down(suf, off, WAVE);
                if (lane + off < WAVE) suf += t;
            }
            int above = suf - s;                             // keys in higher-numbered lanes' bins
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                if (above < remaining && remaining <= above + h[i]) { sh.bc[0] = lane * 4 + i; sh.bc[1] = above; }
                above += h[i];
            }
        }
        __syncthreads();
        const int digit = sh.bc[0], above = sh.bc[1];
        gt += above;
        remaining -= above;
        prefix |= (uint32_t)digit << shift;
        mask |= 255u << shift;
        __syncthreads();
    }
    T = prefix;
    greater = gt;
}

// flags[j] := 1 for the conserved tokens of a slice -- positions [pre, n) (the recent window)
// and the n_heavy largest masses among [0, pre) (exact top-k, ties to the lower index) -- and 0
// for the others.  Whole workgroup; no barrier after the last store.
__device__ void mark_conserved(const float *mass, uint8_t *flags, int n, int pre, int n_heavy, SegShared &sh)
{
    const int tid = threadIdx.x;
    uint32_t T1 = 0;
    int take_eq1 = 0;
    if (n_heavy > 0) {
        int gt1;
        block_select_kth_largest([&](int j, uint32_t &key) { key = sortable_key(mass[j]); return true; }, pre,
                                 n_heavy, T1, gt1, sh);
        take_eq1 = n_heavy - gt1;
    }
    int carry = 0;
    for (int t0 = 0; t0 < n; t0 += SEG_TILE) {
        const int jb = t0 + tid * SEG_ITEMS;
        uint32_t key[SEG_ITEMS];
        int eq_cnt = 0;
#pragma unroll
        for (int i = 0; i < SEG_ITEMS; ++i) {
            const int j = jb + i;
            key[i] = (j < pre && n_heavy > 0) ? sortable_key(mass[j]) : 0u;
            if (j < pre && n_heavy > 0 && key[i] == T1) ++eq_cnt;
        }
        int total;
        int rank = carry + block_exclusive_sum(eq_cnt, total, sh.wave_i);
#pragma unroll
        for (int i = 0; i < SEG_ITEMS; ++i) {
            const int j = jb + i;
            if (j >= n) break;
            bool prot = j >= pre;
            if (!prot && n_heavy > 0) {
                if (key[i] > T1) prot = true;
                else if (key[i] == T1) { prot = rank < take_eq1; ++rank; }
            }
            flags[j] = prot ? 1 : 0;
        }
        carry += total;
    }
}

// Random member of a set of m tokens that starts at token lo of a slice: the SplitMix64
// output function (Steele, Lea, Flood 2014) at the counter seed + slice * 2^32 + lo, upper
// 32 bits scaled to [0, m).
__device__ __forceinline__ int random_member(uint64_t seed, int slice, int lo, int m) {
    uint64_t z = seed + (((uint64_t)(uint32_t)slice << 32) | (uint32_t)lo) + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (int)(((z >> 32) * (uint64_t)m) >> 32);
}

struct SegArgs {
    const float *mass;
    const float *sim;
    uint8_t *flags;
    int32_t *set_id, *set_start, *pivot, *n_sets, *slice_status;
    const int32_t *seq_lens;
    int H, N, cap_rows, enforce;
    double budget, recent_ratio, heavy_ratio;
    float threshold;
    int pivot_rule;
    uint64_t pivot_seed;
    const int32_t *run;       // anchor rule: run lengths
    int set_rule;
    int phase;                // SEG_ALL, or the two halves the anchor rule runs its own kernel between
    int walk_in_lds;          // anchor rule: 3 N bytes of dynamic LDS hold the walk's inputs
};
enum { SEG_ALL = 0, SEG_FLAGS_ONLY = 1, SEG_AFTER_FLAGS = 2 };

__global__ __launch_bounds__(SEG_BLOCK) void segment_kernel(SegArgs a)
{
    __shared__ SegShared sh;
    const int slice = blockIdx.x;
    const int tid = threadIdx.x;
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    const float *mass = a.mass + (size_t)slice * a.N;
    const float *sim = a.sim + (size_t)slice * a.N;
    uint8_t *flags = a.flags + (size_t)slice * a.N;
    int32_t *set_id = a.set_id + (size_t)slice * a.N;
    int32_t *set_start = a.set_start + (size_t)slice * (a.cap_rows + 1);
    int32_t *pivot = a.pivot + (size_t)slice * a.cap_rows;
    const float eps = a.threshold;

    int n_recent = (int)floor(a.recent_ratio * (double)n);
    if (n_recent > n) n_recent = n;
    int n_heavy = (int)floor(a.heavy_ratio * (double)n);
    const int pre = n - n_recent;                            // the top-k is taken over [0, pre)
    if (n_heavy > pre) n_heavy = pre;
    const int cap = (int)floor(a.budget * (double)n);

    if (a.phase != SEG_AFTER_FLAGS) {
    for (int j = n + tid; j < a.N; j += SEG_BLOCK) set_id[j] = -1;

    mark_conserved(mass, flags, n, pre, n_heavy, sh);
    }
    if (a.phase == SEG_FLAGS_ONLY) return;
    __syncthreads();

    const bool anchor_rule = a.set_rule == KVM_SETS_ANCHOR;
    if (anchor_rule) {
        // Walk every stretch of free tokens down from its last token: the set of token i reaches
        // run[i] tokens down, and the token below it is the next i.  Bit 2 marks a set's first
        // token.  (One thread per stretch; a stretch costs one dependent load per set.)
        const int32_t *run = a.run + (size_t)slice * a.N;
        extern __shared__ uint16_t walk_lds[];               // run lengths, then the conserved bits
        if (a.walk_in_lds) {
            // a copy in LDS: the walk is a chain of dependent reads (a run length fits 16 bits
            // whenever the copy fits LDS)
            uint16_t *lrun = walk_lds;
            uint8_t *lprot = reinterpret_cast<uint8_t *>(walk_lds + a.N);
            for (int j = tid; j < n; j += SEG_BLOCK) {
                lrun[j] = (uint16_t)min(max(run[j], 0), 65535);
                lprot[j] = flags[j] & 1;
            }
            __syncthreads();
            for (int e = tid; e < n; e += SEG_BLOCK) {
                if (lprot[e] || (e + 1 < n && !lprot[e + 1])) continue;       // not the last token of a stretch
                int i = e;
                while (i >= 0 && !lprot[i]) {
                    const int first = max(i - (int)lrun[i], 0);
                    flags[first] = 4;                         // a free token: no other bit is set
                    i = first - 1;
                }
            }
        } else {
            for (int e = tid; e < n; e += SEG_BLOCK) {
                if ((flags[e] & 1) || (e + 1 < n && !(flags[e + 1] & 1))) continue;
                int i = e;
                while (i >= 0 && !(flags[i] & 1)) {
                    const int first = max(i - max(run[i], 0), 0);
                    flags[first] = 4;                         // a free token: no other bit is set
                    i = first - 1;
                }
            }
        }
        __syncthreads();
    }

    // j-1 and j may share a set (before the budget rule); "natural" boundary = both free, sim <= eps
    auto joins = [&](int j) -> bool {
        if (anchor_rule) return j >= 1 && !(flags[j] & 5);   // neither conserved nor a set's first token
        return j >= 1 && !(flags[j] & 1) && !(flags[j - 1] & 1) && sim[j] > eps;
    };
    auto natural = [&](int j) -> bool { return j >= 1 && !(flags[j] & 1) && !(flags[j - 1] & 1) && !(sim[j] > eps); };

    // ---- count sets and natural boundaries ----------------------------------------------------
    int m0 = 0, nat = 0;
    for (int j = tid; j < n; j += SEG_BLOCK) {
        m0 += joins(j) ? 0 : 1;
        nat += natural(j) ? 1 : 0;
    }
    const int M0 = block_sum(m0, sh.wave_i);
    const int n_nat = block_sum(nat, sh.wave_i2);
    int status = 0;

    // ---- budget fallback: remove the most similar natural boundaries (ties: higher index) -----
    if (anchor_rule && a.enforce && M0 > cap) status |= KVM_SLICE_INFEASIBLE;   // no fallback for this rule
    if (!anchor_rule && a.enforce && M0 > cap) {
        const int r = M0 - cap;
        bool all = n_nat <= r;
        uint32_t T2 = 0;
        int take_eq2 = 0, total_eq2 = 0;
        if (n_nat < r) status |= KVM_SLICE_INFEASIBLE;
        if (n_nat > 0) status |= KVM_SLICE_FALLBACK;
        if (!all) {
            int gt2;
            block_select_kth_largest([&](int j, uint32_t &key) { key = sortable_key(sim[j]); return natural(j); }, n, r,
                                     T2, gt2, sh);
            take_eq2 = r - gt2;
            int eqc = 0;
            for (int j = tid; j < n; j += SEG_BLOCK) eqc += (natural(j) && sortable_key(sim[j]) == T2) ? 1 : 0;
            total_eq2 = block_sum(eqc, sh.wave_i);
        }
        if (n_nat > 0) {
            int carry = 0;
            for (int t0 = 0; t0 < n; t0 += SEG_TILE) {
                const int jb = t0 + tid * SEG_ITEMS;
                bool isnat[SEG_ITEMS];
                uint32_t key[SEG_ITEMS];
                int eq_cnt = 0;
#pragma unroll
                for (int i = 0; i < SEG_ITEMS; ++i) {
                    const int j = jb + i;
                    isnat[i] = j < n && natural(j);
                    key[i] = isnat[i] ? sortable_key(sim[j]) : 0u;
                    if (isnat[i] && !all && key[i] == T2) ++eq_cnt;
                }
                int total;
                int rank = carry + block_exclusive_sum(eq_cnt, total, sh.wave_i2);
#pragma unroll
                for (int i = 0; i < SEG_ITEMS; ++i) {
                    const int j = jb + i;
                    if (!isnat[i]) continue;
                    bool rem = all || key[i] > T2;
                    if (!rem && key[i] == T2) { rem = (total_eq2 - 1 - rank) < take_eq2; ++rank; }
                    if (rem) flags[j] |= 2;
                }
                carry += total;
            }
        }
        __syncthreads();
    }

    // ---- set ids, set starts, pivots -------------------------------------------------------------
    auto head = [&](int j) -> bool { return !(joins(j) || (flags[j] & 2)); };   // j starts a set
    int set_carry = 0;
    unsigned long long key_carry = 0;                        // running max of the set that crosses the tile edge
    for (int t0 = 0; t0 < n; t0 += SEG_TILE) {
        const int jb = t0 + tid * SEG_ITEMS;
        bool hd[SEG_ITEMS + 1];
        unsigned long long key[SEG_ITEMS];
        int heads = 0;
#pragma unroll
        for (int i = 0; i <= SEG_ITEMS; ++i) {
            const int j = jb + i;
            hd[i] = j < n ? head(j) : true;                  // the position after the last token closes a set
            if (i < SEG_ITEMS && j < n) {
                heads += hd[i] ? 1 : 0;
                key[i] = ((unsigned long long)sortable_key(mass[j]) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)j);
            }
        }
        // thread summary for the segmented max scan: (any head, max of the trailing open segment)
        int f = 0;
        unsigned long long k = 0;
#pragma unroll
        for (int i = 0; i < SEG_ITEMS; ++i) {
            if (jb + i >= n) break;
            if (hd[i]) { f = 1; k = key[i]; }
            else k = k > key[i] ? k : key[i];
        }
        int total_heads;
        const int sets_before = set_carry + block_exclusive_sum(heads, total_heads, sh.wave_i);
        // inclusive segmented scan over thread summaries within the wave
        const int lane = tid & 63, w = tid >> 6;
        int fi = f;
        unsigned long long ki = k;
#pragma unroll
        for (int off = 1; off < WAVE; off <<= 1) {
            int f2 = __shfl_up(fi, off, WAVE);
            unsigned long long k2 = shfl_up_u64(ki, off);
            if (lane >= off) {
                if (!fi) ki = ki > k2 ? ki : k2;
                fi |= f2;
            }
        }
        if (lane == WAVE - 1) { sh.wave_f[w] = fi; sh.wave_k[w] = ki; }
        int fe = __shfl_up(fi, 1, WAVE);                     // exclusive within the wave
        unsigned long long ke = shfl_up_u64(ki, 1);
        if (lane == 0) { fe = 0; ke = 0; }
        __syncthreads();
        int fp = 0;                                          // everything before this wave, tile carry included
        unsigned long long kp = key_carry;
        for (int i = 0; i < w; ++i) {
            if (sh.wave_f[i]) { fp = 1; kp = sh.wave_k[i]; }
            else kp = kp > sh.wave_k[i] ? kp : sh.wave_k[i];
        }
        unsigned long long incoming = fe ? ke : (kp > ke ? kp : ke);
        // walk the thread's items
        int s = sets_before - 1;
        unsigned long long cur = incoming;
#pragma unroll
        for (int i = 0; i < SEG_ITEMS; ++i) {
            const int j = jb + i;
            if (j >= n) break;
            if (hd[i]) {
                ++s;
                cur = key[i];
                if (s <= a.cap_rows) set_start[s] = j;
            } else {
                cur = cur > key[i] ? cur : key[i];
            }
            set_id[j] = s;
            if (hd[i + 1] && s < a.cap_rows) pivot[s] = (int32_t)(0xFFFFFFFFu - (uint32_t)cur);
        }
        // carry to the next tile: the inclusive value of the last thread
        __syncthreads();
        if (tid == SEG_BLOCK - 1) sh.bck = cur;
        __syncthreads();
        key_carry = sh.bck;
        set_carry += total_heads;
        (void)fp;
    }
    const int M = set_carry;
    for (int s = M + tid; s <= a.cap_rows; s += SEG_BLOCK) {
        set_start[s] = n;
        if (s < a.cap_rows) pivot[s] = -1;
    }
    if (a.pivot_rule != KVM_PIVOT_MAX_SCORE) {
        // the other pivot rules need only the sets' extents, which are complete now
        __syncthreads();
        for (int s = tid; s < min(M, a.cap_rows); s += SEG_BLOCK) {
            const int lo = set_start[s], hi = set_start[s + 1];
            pivot[s] = a.pivot_rule == KVM_PIVOT_LAST ? hi - 1 : lo + random_member(a.pivot_seed, slice, lo, hi - lo);
        }
    }
    if (M > a.cap_rows) status |= KVM_SLICE_TRUNCATED;
    if (tid == 0) {
        a.n_sets[slice] = M;
        a.slice_status[slice] = status;
    }
}

// ------------------------------------------------------------------------------------------
// segmentation of slices of up to 16384 tokens (adjacent rule): everything in registers
// ------------------------------------------------------------------------------------------
//
// segment_kernel above walks a slice in tiles and goes back to memory for the scores, the
// similarities and the flag bytes in every one of its passes; with 1024 threads per slice each of
// its ~40 barriers is expensive and only two slices fit a CU.  Here a thread owns 16 consecutive
// tokens and keeps their score keys, similarities and flag bits in registers from one coalesced
// read to the final write; a workgroup has just enough threads for the slice (256 for 4096
// tokens: four slices per CU, the whole headline workload resident at once), and the same steps
// -- exact top-k by radix select, boundary test, budget rule, set numbering, segmented arg-max --
// run on the registers.  Same results bit for bit.

constexpr int SR_ITEMS = 16;

template <int BLOCK> struct SegRegShared {
    int hist[256];
    int wave_i[BLOCK / WAVE];
    int wave_i2[BLOCK / WAVE];
    unsigned long long wave_k[BLOCK / WAVE];
    int wave_f[BLOCK / WAVE];
    int bc[2];
    unsigned long long bck;
    uint32_t bits[BLOCK + 1];            // one 16-bit mask per thread, handed to the neighbour
};

template <int WAVES>
__device__ __forceinline__ int block_exclusive_sum_w(int v, int &total, int *wave_slots) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        int t = __shfl_up(inc, off, WAVE);
        if (lane >= off) inc += t;
    }
    __syncthreads();                                         // wave_slots may still be read from a previous use
    if (lane == WAVE - 1) wave_slots[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        int a = wave_slots[i];
        if (i < w) before += a;
        all += a;
    }
    total = all;
    return before + inc - v;
}

// k-th largest (k >= 1) of the keys whose bit is set in `valid` (16 keys per thread).  Needs
// k <= number of valid keys.  Returns the key value T and the number of valid keys greater than T.
template <int BLOCK>
__device__ void select_kth_largest_reg(const uint32_t *key, uint32_t valid, int k, uint32_t &T, int &greater,
                                       SegRegShared<BLOCK> &sh)
{
    uint32_t prefix = 0, mask = 0;
    int remaining = k, gt = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = threadIdx.x; i < 256; i += BLOCK) sh.hist[i] = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < SR_ITEMS; ++i)
            if (((valid >> i) & 1u) && (key[i] & mask) == prefix) atomicAdd(&sh.hist[(key[i] >> shift) & 255u], 1);
        __syncthreads();
        if (threadIdx.x < WAVE) {
            const int lane = threadIdx.x;
            int h[4], s = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { h[i] = sh.hist[lane * 4 + i]; s += h[i]; }
            int suf = s;                                     // inclusive suffix sum over lanes
#pragma unroll
            for (int off = 1; off < WAVE; off <<= 1) {
                int t = __shfl_down(suf, off, WAVE);
                if (lane + off < WAVE) suf += t;
            }
            int above = suf - s;                             // keys in higher-numbered lanes' bins
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                if (above < remaining && remaining <= above + h[i]) { sh.bc[0] = lane * 4 + i; sh.bc[1] = above; }
                above += h[i];
            }
        }
        __syncthreads();
        const int digit = sh.bc[0], above = sh.bc[1];
        gt += above;
        remaining -= above;
        prefix |= (uint32_t)digit << shift;
        mask |= 255u << shift;
    }
    T = prefix;
    greater = gt;
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void segment_reg_kernel(SegArgs a)
{
    constexpr int WAVES = BLOCK / WAVE;
    __shared__ SegRegShared<BLOCK> sh;
    const int slice = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    const float *mass = a.mass + (size_t)slice * a.N;
    const float *sim = a.sim + (size_t)slice * a.N;
    int32_t *set_id = a.set_id + (size_t)slice * a.N;
    int32_t *set_start = a.set_start + (size_t)slice * (a.cap_rows + 1);
    int32_t *pivot = a.pivot + (size_t)slice * a.cap_rows;
    const float eps = a.threshold;

    int n_recent = (int)floor(a.recent_ratio * (double)n);
    if (n_recent > n) n_recent = n;
    int n_heavy = (int)floor(a.heavy_ratio * (double)n);
    const int pre = n - n_recent;                            // the top-k is taken over [0, pre)
    if (n_heavy > pre) n_heavy = pre;
    const int cap = (int)floor(a.budget * (double)n);

    // this thread's tokens jb .. jb+15: score keys and similarities, read once (16 bytes at a time
    // where the rows are aligned for it)
    const int jb = tid * SR_ITEMS;
    const bool vec = (a.N & 3) == 0 && ((reinterpret_cast<uintptr_t>(a.mass) | reinterpret_cast<uintptr_t>(a.sim) |
                                         reinterpret_cast<uintptr_t>(a.set_id)) & 15) == 0;
    uint32_t key[SR_ITEMS];
    float sm[SR_ITEMS];
#pragma unroll
    for (int v = 0; v < SR_ITEMS / 4; ++v) {
        f32x4 m4 = {0.f, 0.f, 0.f, 0.f}, s4 = {0.f, 0.f, 0.f, 0.f};
        if (vec && jb + 4 * v + 3 < a.N) {                   // (N is the row stride: whole vectors stay inside the row)
            m4 = *reinterpret_cast<const f32x4 *>(mass + jb + 4 * v);
            s4 = *reinterpret_cast<const f32x4 *>(sim + jb + 4 * v);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (jb + 4 * v + e < a.N) { m4[e] = mass[jb + 4 * v + e]; s4[e] = sim[jb + 4 * v + e]; }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float me = m4[e];
            key[4 * v + e] = sortable_key(me);
            sm[4 * v + e] = s4[e];
        }
    }
    uint32_t in_n = 0, in_pre = 0;                           // bit i: token jb+i < n, < pre
#pragma unroll
    for (int i = 0; i < SR_ITEMS; ++i) {
        in_n |= (jb + i < n ? 1u : 0u) << i;
        in_pre |= (jb + i < pre ? 1u : 0u) << i;
    }
    for (int j = n + tid; j < a.N; j += BLOCK) set_id[j] = -1;

    // ---- conserved tokens: the recent window and the exact top-k of the scores before it --------
    uint32_t prot = in_n & ~in_pre;
    if (n_heavy > 0) {
        uint32_t T1;
        int gt1;
        select_kth_largest_reg<BLOCK>(key, in_pre, n_heavy, T1, gt1, sh);
        const int take_eq1 = n_heavy - gt1;
        int eq_cnt = 0;
#pragma unroll
        for (int i = 0; i < SR_ITEMS; ++i) eq_cnt += (((in_pre >> i) & 1u) && key[i] == T1) ? 1 : 0;
        int total;
        int rank = block_exclusive_sum_w<WAVES>(eq_cnt, total, sh.wave_i);
#pragma unroll
        for (int i = 0; i < SR_ITEMS; ++i) {
            if (!((in_pre >> i) & 1u)) continue;
            if (key[i] > T1) prot |= 1u << i;
            else if (key[i] == T1) { if (rank < take_eq1) prot |= 1u << i; ++rank; }
        }
    }
    // the neighbour's last token
    __syncthreads();
    sh.bits[tid + 1] = prot;
    if (tid == 0) sh.bits[0] = 0;
    __syncthreads();
    const uint32_t prot_prev = (prot << 1) | ((sh.bits[tid] >> (SR_ITEMS - 1)) & 1u);   // bit i: token jb+i-1 is conserved

    // j-1 and j may share a set (before the budget rule); "natural" boundary = both free, sim <= eps
    uint32_t joins = 0, natural = 0;
#pragma unroll
    for (int i = 0; i < SR_ITEMS; ++i) {
        const bool both_free = jb + i >= 1 && jb + i < n && !((prot >> i) & 1u) && !((prot_prev >> i) & 1u);
        const bool above = sm[i] > eps;
        joins |= (both_free && above ? 1u : 0u) << i;
        natural |= (both_free && !above ? 1u : 0u) << i;
    }
    int M0, n_nat;
    (void)block_exclusive_sum_w<WAVES>(__popc(in_n & ~joins), M0, sh.wave_i);
    (void)block_exclusive_sum_w<WAVES>(__popc(natural), n_nat, sh.wave_i2);
    int status = 0;

    // ---- budget rule: remove the most similar natural boundaries (ties: higher index first) ------
    uint32_t removed = 0;
    if (a.enforce && M0 > cap) {
        const int r = M0 - cap;
        const bool all = n_nat <= r;
        if (n_nat < r) status |= KVM_SLICE_INFEASIBLE;
        if (n_nat > 0) status |= KVM_SLICE_FALLBACK;
        if (all) {
            removed = natural;
        } else {
            uint32_t skey[SR_ITEMS];
#pragma unroll
            for (int i = 0; i < SR_ITEMS; ++i) skey[i] = sortable_key(sm[i]);
            uint32_t T2;
            int gt2;
            select_kth_largest_reg<BLOCK>(skey, natural, r, T2, gt2, sh);
            const int take_eq2 = r - gt2;
            int eq_cnt = 0;
#pragma unroll
            for (int i = 0; i < SR_ITEMS; ++i) eq_cnt += (((natural >> i) & 1u) && skey[i] == T2) ? 1 : 0;
            int total_eq2;
            int rank = block_exclusive_sum_w<WAVES>(eq_cnt, total_eq2, sh.wave_i);
#pragma unroll
            for (int i = 0; i < SR_ITEMS; ++i) {
                if (!((natural >> i) & 1u)) continue;
                if (skey[i] > T2) removed |= 1u << i;
                else if (skey[i] == T2) { if (total_eq2 - 1 - rank < take_eq2) removed |= 1u << i; ++rank; }
            }
        }
    }

    // ---- set ids, set starts, pivots -----------------------------------------------------------
    // token j starts a set unless it joins its predecessor or its boundary was removed; the position
    // after the last token closes the last set
    const uint32_t head = (in_n & ~(joins | removed)) | (~in_n & 0xFFFFu);
    __syncthreads();
    sh.bits[tid] = head;
    if (tid == 0) sh.bits[BLOCK] = 0xFFFFu;
    __syncthreads();
    const uint32_t head_next = (head >> 1) | ((sh.bits[tid + 1] & 1u) << (SR_ITEMS - 1));   // bit i: token jb+i+1 starts a set
    const int heads = __popc(head & in_n);
    unsigned long long mkey[SR_ITEMS];
#pragma unroll
    for (int i = 0; i < SR_ITEMS; ++i) mkey[i] = ((unsigned long long)key[i] << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)(jb + i));
    // thread summary for the segmented max scan: (any head, max of the trailing open segment)
    int f = 0;
    unsigned long long k = 0;
#pragma unroll
    for (int i = 0; i < SR_ITEMS; ++i) {
        if (!((in_n >> i) & 1u)) break;
        if ((head >> i) & 1u) { f = 1; k = mkey[i]; }
        else k = k > mkey[i] ? k : mkey[i];
    }
    int M;
    const int sets_before = block_exclusive_sum_w<WAVES>(heads, M, sh.wave_i);
    int fi = f;
    unsigned long long ki = k;
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        int f2 = __shfl_up(fi, off, WAVE);
        unsigned long long k2 = shfl_up_u64(ki, off);
        if (lane >= off) {
            if (!fi) ki = ki > k2 ? ki : k2;
            fi |= f2;
        }
    }
    if (lane == WAVE - 1) { sh.wave_f[w] = fi; sh.wave_k[w] = ki; }
    int fe = __shfl_up(fi, 1, WAVE);                         // exclusive within the wave
    unsigned long long ke = shfl_up_u64(ki, 1);
    if (lane == 0) { fe = 0; ke = 0; }
    __syncthreads();
    unsigned long long kp = 0;                               // everything before this wave
    for (int i = 0; i < w; ++i) {
        if (sh.wave_f[i]) kp = sh.wave_k[i];
        else kp = kp > sh.wave_k[i] ? kp : sh.wave_k[i];
    }
    unsigned long long cur = fe ? ke : (kp > ke ? kp : ke);
    int s = sets_before - 1;
    int32_t ids[SR_ITEMS];
#pragma unroll
    for (int i = 0; i < SR_ITEMS; ++i) {
        const int j = jb + i;
        if ((in_n >> i) & 1u) {
            if ((head >> i) & 1u) {
                ++s;
                cur = mkey[i];
                if (s <= a.cap_rows) set_start[s] = j;
            } else {
                cur = cur > mkey[i] ? cur : mkey[i];
            }
            if (((head_next >> i) & 1u) && s < a.cap_rows) pivot[s] = (int32_t)(0xFFFFFFFFu - (uint32_t)cur);
        }
        ids[i] = s;
    }
#pragma unroll
    for (int v = 0; v < SR_ITEMS / 4; ++v) {
        if (vec && jb + 4 * v + 3 < n) {
            int4 o = {ids[4 * v], ids[4 * v + 1], ids[4 * v + 2], ids[4 * v + 3]};
            *reinterpret_cast<int4 *>(set_id + jb + 4 * v) = o;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (jb + 4 * v + e < n) set_id[jb + 4 * v + e] = ids[4 * v + e];
        }
    }
    for (int t = M + tid; t <= a.cap_rows; t += BLOCK) {
        set_start[t] = n;
        if (t < a.cap_rows) pivot[t] = -1;
    }
    if (a.pivot_rule != KVM_PIVOT_MAX_SCORE) {
        // the other pivot rules need only the sets' extents, which are complete now
        __syncthreads();
        for (int t = tid; t < min(M, a.cap_rows); t += BLOCK) {
            const int lo = set_start[t], hi = set_start[t + 1];
            pivot[t] = a.pivot_rule == KVM_PIVOT_LAST ? hi - 1 : lo + random_member(a.pivot_seed, slice, lo, hi - lo);
        }
    }
    if (M > a.cap_rows) status |= KVM_SLICE_TRUNCATED;
    if (tid == 0) {
        a.n_sets[slice] = M;
        a.slice_status[slice] = status;
    }
}

// ------------------------------------------------------------------------------------------
// comparison workload: eviction by aggregated attention score
// ------------------------------------------------------------------------------------------

struct EvictArgs {
    const float *mass;
    uint8_t *flags;
    int32_t *kept, *n_kept;
    const int32_t *seq_lens;
    int H, N, cap_rows;
    double budget, recent_ratio;
};

// Per slice: keep the recent window and the tokens with the largest masses among the others,
// floor(budget n) in all; write their positions in ascending order.
__global__ __launch_bounds__(SEG_BLOCK) void evict_select_kernel(EvictArgs a)
{
    __shared__ SegShared sh;
    const int slice = blockIdx.x;
    const int tid = threadIdx.x;
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    const float *mass = a.mass + (size_t)slice * a.N;
    uint8_t *flags = a.flags + (size_t)slice * a.N;
    int32_t *kept = a.kept + (size_t)slice * a.cap_rows;
    const int cap = min((int)floor(a.budget * (double)n), a.cap_rows);
    int n_recent = (int)floor(a.recent_ratio * (double)n);
    if (n_recent > cap) n_recent = cap;                      // a window wider than the budget is cut to it
    const int pre = n - n_recent;
    const int n_heavy = min(cap - n_recent, pre);
    mark_conserved(mass, flags, n, pre, n_heavy, sh);
    __syncthreads();
    int carry = 0;
    for (int t0 = 0; t0 < n; t0 += SEG_TILE) {
        const int jb = t0 + tid * SEG_ITEMS;
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < SEG_ITEMS; ++i) cnt += (jb + i < n && flags[jb + i]) ? 1 : 0;
        int total;
        int pos = carry + block_exclusive_sum(cnt, total, sh.wave_i);
#pragma unroll
        for (int i = 0; i < SEG_ITEMS; ++i)
            if (jb + i < n && flags[jb + i]) kept[pos++] = jb + i;
        carry += total;
    }
    for (int s = carry + tid; s < a.cap_rows; s += SEG_BLOCK) kept[s] = -1;
    if (tid == 0) a.n_kept[slice] = carry;
}

// out[s] = in[kept[s]] for the kept rows of K and V; 16 lanes per row.
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                           T *__restrict__ K_out, T *__restrict__ V_out,
                                                           const int32_t *__restrict__ kept, const int32_t *__restrict__ n_kept,
                                                           int N, int cap_rows, int tiles_per_slice)
{
    const int slice = blockIdx.x / tiles_per_slice;
    const int tile = blockIdx.x - slice * tiles_per_slice;
    const int c = threadIdx.x & 15, group = threadIdx.x >> 4;
    const int m = min(max(n_kept[slice], 0), cap_rows);
    const int32_t *kp = kept + (size_t)slice * cap_rows;
    constexpr int ROWS = 4;                                  // rows per group, loads in flight together
    const int s0 = (tile * 16 + group) * ROWS;
    typename Elem<T>::Raw rk[ROWS], rv[ROWS];
    int src[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        src[r] = s0 + r < m ? min(max(kp[s0 + r], 0), N - 1) : -1;
        if (src[r] >= 0) {
            rk[r] = Elem<T>::load(K + ((size_t)slice * N + src[r]) * HEAD_DIM, c);
            rv[r] = Elem<T>::load(V + ((size_t)slice * N + src[r]) * HEAD_DIM, c);
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        if (src[r] >= 0) {
            Elem<T>::store(K_out + ((size_t)slice * cap_rows + s0 + r) * HEAD_DIM, c, rk[r]);
            Elem<T>::store(V_out + ((size_t)slice * cap_rows + s0 + r) * HEAD_DIM, c, rv[r]);
        }
}

template <typename T>
static void launch_gather(const kvm_shape &sh, int cap_rows, const void *K, const void *V, void *K_out, void *V_out,
                          const int32_t *kept, const int32_t *n_kept, hipStream_t st)
{
    const int tiles = (cap_rows + 63) / 64;
    const long long blocks = (long long)sh.B * sh.H_kv * tiles;
    ProfScope prof("gather_rows_kernel", st);
    hipLaunchKernelGGL(gather_rows_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, (const T *)K, (const T *)V, (T *)K_out,
                       (T *)V_out, kept, n_kept, sh.N, cap_rows, tiles);
}

// Second comparison workload (value-only merging): K_out[s] = K[kept[s]]; V_out[s] = mean of the
// values of the tokens that are nearest to kept[s] among the kept positions (equal distances: the
// later one), i.e. of the range that ends half-way to either neighbour.  One 16-lane group per kept
// row for the first 32 rows of its range (4 loads in flight); what a longer range has left is summed
// by the whole workgroup, one range after the other (64 rows in flight, partial sums through LDS in
// a fixed order): scores that fall with the position leave one gap of thousands of tokens between
// the heavy tokens and the recent window, and half of all values sit in it.
// fp32 sums, one division, one rounding.
constexpr int VM_OWN_ROWS = 32;

template <typename T>
__global__ __launch_bounds__(256) void gather_merge_values_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                                   T *__restrict__ K_out, T *__restrict__ V_out,
                                                                   const int32_t *__restrict__ kept,
                                                                   const int32_t *__restrict__ n_kept,
                                                                   const int32_t *__restrict__ seq_lens, int H, int N,
                                                                   int cap_rows, int tiles_per_slice)
{
    using E = Elem<T>;
    using Raw = typename E::Raw;
    __shared__ int rest_lo[16], rest_hi[16];
    __shared__ float red[4][16][9];                          // per wave and 8-element chunk (padded)
    const int slice = blockIdx.x / tiles_per_slice;
    // Consecutive workgroups go to consecutive XCDs, and the long ranges sit at the same tiles in
    // every slice: the tiles are rotated by the slice index so that they do not all meet on the
    // same one or two XCDs.
    const int tile = (blockIdx.x - slice * tiles_per_slice + slice) % tiles_per_slice;
    const int c = threadIdx.x & 15, group = threadIdx.x >> 4, wave = threadIdx.x >> 6;
    const int n = clamp_len(seq_lens, slice / H, N);
    const int m = min(max(n_kept[slice], 0), cap_rows);
    if (tile * 16 >= m) return;                              // (the whole workgroup)
    const int s = tile * 16 + group;
    const int32_t *kp = kept + (size_t)slice * cap_rows;
    const T *Ks = K + (size_t)slice * N * HEAD_DIM;
    const T *Vs = V + (size_t)slice * N * HEAD_DIM;
    // the range of this group's kept token (positions are clamped into the slice: the list may
    // hold anything when the caller's buffers are inconsistent)
    int lo = 0, hi = 0, p = 0;
    if (s < m) {
        p = min(max(kp[s], 0), n - 1);
        lo = s == 0 ? 0 : (min(max(kp[s - 1], 0), n - 1) + p + 1) >> 1;
        hi = s == m - 1 ? n : (p + min(max(kp[s + 1], 0), n - 1) + 1) >> 1;
        lo = min(lo, p);
        hi = max(hi, p + 1);
    }
    const int cnt = hi - lo;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    Raw kr;
    if (s < m) kr = E::load(Ks + (size_t)p * HEAD_DIM, c);
    // the group's own part
    const int own_hi = min(hi, lo + VM_OWN_ROWS);
    if (c == 0) { rest_lo[group] = own_hi; rest_hi[group] = hi; }
    for (int j0 = lo; j0 < own_hi; j0 += 4) {
        Raw r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (j0 + u < own_hi) r[u] = E::load(Vs + (size_t)(j0 + u) * HEAD_DIM, c);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (j0 + u < own_hi) {
                float x[8];
                E::to_float(r[u], x);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += x[e];
            }
    }
    __syncthreads();
    // what longer ranges have left, by the whole workgroup
    for (int g = 0; g < 16; ++g) {
        const int r_lo = rest_lo[g], r_hi = rest_hi[g];
        if (r_hi <= r_lo) continue;                          // (the same for the whole workgroup)
        float part[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) part[e] = 0.f;
        for (int j0 = r_lo; j0 < r_hi; j0 += 64) {
            Raw r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + 16 * u + group < r_hi) r[u] = E::load(Vs + (size_t)(j0 + 16 * u + group) * HEAD_DIM, c);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + 16 * u + group < r_hi) {
                    float x[8];
                    E::to_float(r[u], x);
#pragma unroll
                    for (int e = 0; e < 8; ++e) part[e] += x[e];
                }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) part[e] = rows4_sum(part[e]);
        if ((threadIdx.x & 48) == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) red[wave][c][e] = part[e];
        }
        __syncthreads();
        if (group == g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (red[0][c][e] + red[1][c][e]) + (red[2][c][e] + red[3][c][e]);
        }
        __syncthreads();                                     // red is written again for the next long range
    }
    if (s < m) {
        const float cf = (float)cnt;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] / cf;
        E::store(K_out + ((size_t)slice * cap_rows + s) * HEAD_DIM, c, kr);
        E::store(V_out + ((size_t)slice * cap_rows + s) * HEAD_DIM, c, E::from_float(acc));   // a lone value comes back bit for bit
    }
}

template <typename T>
static void launch_gather_merge_values(const kvm_shape &sh, int cap_rows, const void *K, const void *V, void *K_out,
                                       void *V_out, const int32_t *kept, const int32_t *n_kept, hipStream_t st)
{
    const int tiles = (cap_rows + 15) / 16;
    const long long blocks = (long long)sh.B * sh.H_kv * tiles;
    ProfScope prof("gather_merge_values_kernel", st);
    hipLaunchKernelGGL(gather_merge_values_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, (const T *)K, (const T *)V,
                       (T *)K_out, (T *)V_out, kept, n_kept, sh.seq_lens, sh.H_kv, sh.N, cap_rows, tiles);
}

kvm_status launch_evict(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                        const float *mass, int32_t *kept, int32_t *n_kept, void *K_out, void *V_out, uint8_t *flags,
                        bool merge_values, hipStream_t st)
{
    const long long slices = (long long)sh.B * sh.H_kv;
    if (slices == 0) return KVM_OK;
    EvictArgs a;
    a.mass = mass;
    a.flags = flags;
    a.kept = kept;
    a.n_kept = n_kept;
    a.seq_lens = sh.seq_lens;
    a.H = sh.H_kv;
    a.N = sh.N;
    a.cap_rows = cap_rows;
    a.budget = pr.budget;
    a.recent_ratio = pr.recent_ratio;
    {
        ProfScope prof("evict_select_kernel", st);
        hipLaunchKernelGGL(evict_select_kernel, dim3((unsigned)slices), dim3(SEG_BLOCK), 0, st, a);
    }
    kvm_status rc = check_launch("evict_select_kernel");
    if (rc != KVM_OK || cap_rows == 0 || sh.N == 0) return rc;
    if (merge_values) {
        switch (sh.dtype) {
        case KVM_F32: launch_gather_merge_values<float>(sh, cap_rows, K, V, K_out, V_out, kept, n_kept, st); break;
        case KVM_F16: launch_gather_merge_values<half_t>(sh, cap_rows, K, V, K_out, V_out, kept, n_kept, st); break;
        default: launch_gather_merge_values<bf16_t>(sh, cap_rows, K, V, K_out, V_out, kept, n_kept, st); break;
        }
        return check_launch("gather_merge_values_kernel");
    }
    switch (sh.dtype) {
    case KVM_F32: launch_gather<float>(sh, cap_rows, K, V, K_out, V_out, kept, n_kept, st); break;
    case KVM_F16: launch_gather<half_t>(sh, cap_rows, K, V, K_out, V_out, kept, n_kept, st); break;
    default: launch_gather<bf16_t>(sh, cap_rows, K, V, K_out, V_out, kept, n_kept, st); break;
    }
    return check_launch("gather_rows_kernel");
}

// ------------------------------------------------------------------------------------------
// host launcher
// ------------------------------------------------------------------------------------------

template <typename T>
static void launch_cosine(const kvm_shape &sh, const void *K, float *sim, float *inv_norm, hipStream_t st)
{
    const int tiles = (sh.N + COS_ROWS_PER_BLOCK - 1) / COS_ROWS_PER_BLOCK;
    const long long blocks = (long long)sh.B * sh.H_kv * tiles;
    ProfScope prof("cosine_scan_kernel", st);
    hipLaunchKernelGGL(cosine_scan_kernel<T>, dim3((unsigned)blocks), dim3(COS_BLOCK), 0, st, (const T *)K, sim, inv_norm,
                       sh.seq_lens, sh.H_kv, sh.N, tiles);
}

template <typename T>
static void launch_anchor_run(const kvm_shape &sh, const void *K, const float *inv_norm, const uint8_t *flags,
                              int32_t *run, float eps, hipStream_t st)
{
    const int tiles = (sh.N + RUN_TILE - 1) / RUN_TILE;
    const long long blocks = (long long)sh.B * sh.H_kv * tiles;
    ProfScope prof("anchor_run_kernel", st);
    hipLaunchKernelGGL(anchor_run_kernel<T>, dim3((unsigned)blocks), dim3(RUN_BLOCK), 0, st, (const T *)K, inv_norm, flags,
                       run, sh.seq_lens, sh.H_kv, sh.N, tiles, eps);
}

kvm_status launch_sim_append(const kvm_shape &sh, const void *K, float *sim, hipStream_t st)
{
    const long long slices = (long long)sh.B * sh.H_kv;
    if (slices == 0 || sh.N == 0) return KVM_OK;
    const dim3 grid((unsigned)((slices + 15) / 16)), block(256);
    ProfScope prof("sim_append_kernel", st);
    switch (sh.dtype) {
    case KVM_F32: hipLaunchKernelGGL(sim_append_kernel<float>, grid, block, 0, st, (const float *)K, sim, sh.seq_lens, sh.H_kv, sh.N, (int)slices); break;
    case KVM_F16: hipLaunchKernelGGL(sim_append_kernel<half_t>, grid, block, 0, st, (const half_t *)K, sim, sh.seq_lens, sh.H_kv, sh.N, (int)slices); break;
    default: hipLaunchKernelGGL(sim_append_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)K, sim, sh.seq_lens, sh.H_kv, sh.N, (int)slices); break;
    }
    return check_launch("sim_append_kernel");
}

// The scan alone (for callers inside the library that want the similarities without the sets).
kvm_status launch_cosine_scan(const kvm_shape &sh, const void *K, float *sim, hipStream_t st)
{
    if ((long long)sh.B * sh.H_kv == 0 || sh.N == 0) return KVM_OK;
    switch (sh.dtype) {
    case KVM_F32: launch_cosine<float>(sh, K, sim, nullptr, st); break;
    case KVM_F16: launch_cosine<half_t>(sh, K, sim, nullptr, st); break;
    default: launch_cosine<bf16_t>(sh, K, sim, nullptr, st); break;
    }
    return check_launch("cosine_scan_kernel");
}

kvm_status launch_identify(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const float *mass,
                           int32_t *set_id, int32_t *set_start, int32_t *pivot, int32_t *n_sets, float *sim,
                           float *inv_norm, int32_t *run, uint8_t *flags, int32_t *slice_status, hipStream_t st)
{
    const long long slices = (long long)sh.B * sh.H_kv;
    if (slices == 0) return KVM_OK;
    const bool anchor = pr.set_rule == KVM_SETS_ANCHOR;
    if (sh.N > 0 && !pr.sim_given) {
        float *rn = anchor ? inv_norm : nullptr;
        switch (sh.dtype) {
        case KVM_F32: launch_cosine<float>(sh, K, sim, rn, st); break;
        case KVM_F16: launch_cosine<half_t>(sh, K, sim, rn, st); break;
        default: launch_cosine<bf16_t>(sh, K, sim, rn, st); break;
        }
        kvm_status rc = check_launch("cosine_scan_kernel");
        if (rc != KVM_OK) return rc;
    }
    SegArgs a;
    a.mass = mass;
    a.sim = sim;
    a.flags = flags;
    a.set_id = set_id;
    a.set_start = set_start;
    a.pivot = pivot;
    a.n_sets = n_sets;
    a.slice_status = slice_status;
    a.seq_lens = sh.seq_lens;
    a.H = sh.H_kv;
    a.N = sh.N;
    a.cap_rows = cap_rows;
    a.enforce = pr.enforce_budget;
    a.budget = pr.budget;
    a.recent_ratio = pr.recent_ratio;
    a.heavy_ratio = pr.heavy_ratio;
    a.threshold = pr.threshold;
    a.pivot_rule = pr.pivot_rule;
    a.pivot_seed = pr.pivot_seed;
    a.run = run;
    a.set_rule = pr.set_rule;
    a.phase = SEG_ALL;
    a.walk_in_lds = 0;
    size_t walk_lds_bytes = 0;
    if (anchor && sh.N > 0) {
        // the conserved tokens first, then the run lengths (which stop at conserved tokens),
        // then the walk over the runs and everything after it
        a.phase = SEG_FLAGS_ONLY;
        {
            ProfScope prof("segment_kernel", st);
            hipLaunchKernelGGL(segment_kernel, dim3((unsigned)slices), dim3(SEG_BLOCK), 0, st, a);
        }
        kvm_status rc = check_launch("segment_kernel");
        if (rc != KVM_OK) return rc;
        switch (sh.dtype) {
        case KVM_F32: launch_anchor_run<float>(sh, K, inv_norm, flags, run, pr.threshold, st); break;
        case KVM_F16: launch_anchor_run<half_t>(sh, K, inv_norm, flags, run, pr.threshold, st); break;
        default: launch_anchor_run<bf16_t>(sh, K, inv_norm, flags, run, pr.threshold, st); break;
        }
        rc = check_launch("anchor_run_kernel");
        if (rc != KVM_OK) return rc;
        a.phase = SEG_AFTER_FLAGS;
        if (sh.N <= 16384) {
            a.walk_in_lds = 1;
            walk_lds_bytes = (size_t)sh.N * 3;
        }
    }
    const bool in_registers = !anchor && sh.N > 0 && sh.N <= 1024 * SR_ITEMS;
    ProfScope prof(in_registers ? "segment_reg_kernel" : "segment_kernel", st);
    if (in_registers) {
        // 16 tokens per thread in registers: as many threads as the slice needs
        if (sh.N <= 256 * SR_ITEMS) hipLaunchKernelGGL(segment_reg_kernel<256>, dim3((unsigned)slices), dim3(256), 0, st, a);
        else if (sh.N <= 512 * SR_ITEMS) hipLaunchKernelGGL(segment_reg_kernel<512>, dim3((unsigned)slices), dim3(512), 0, st, a);
        else hipLaunchKernelGGL(segment_reg_kernel<1024>, dim3((unsigned)slices), dim3(1024), 0, st, a);
    } else {
        hipLaunchKernelGGL(segment_kernel, dim3((unsigned)slices), dim3(SEG_BLOCK), walk_lds_bytes, st, a);
    }
    return check_launch("segment_kernel");
}

}  // namespace kvm
