// Gaussian-kernel weighted merging with a compacting write (Section 4.2: Def. 4.2 Eq. (4),
// Eq. (5), (6); Algorithm 2).
//
// Work is dealt out by tokens, not by sets, because set lengths are very uneven (most sets
// are conserved singletons, most tokens sit in sets of 17..128): a small planning kernel
// finds, for every tile of MERGE_TILE tokens, the first set that starts in it; one wave then
// owns the sets that start inside its tile.  A row of 128 elements is spread over 16 lanes
// (8 elements = 16 B each for 16-bit types), so one wave instruction moves four rows.  Per
// set: one sweep over its keys for the distances to the pivot (sigma), a second sweep (served
// by L2, the set was just read) that forms the weights and accumulates keys and values in
// fp32, then one rounded row is written per output.  Loads are issued 16 rows at a time; a
// set of up to 16 tokens is read exactly once and held in registers.  Runs of singleton sets
// are copied bit for bit.  HBM traffic: K once, V once, 2 M rows out.
//
// Kernels:
//   merge_plan_kernel   per slice: first set of every 64-token tile, and the list of sets of more
//                       than LONG_SET_MIN tokens
//   merge_kernel        one wave per tile (merge_one_set per set, runs of singletons copied)
//   merge_long_kernel   the listed long sets, one 1024-thread workgroup per slice
//   refresh_kernel      decode time: compares the new maps with the previous ones, moves the rows of
//                       unchanged sets in place and merges the changed sets again
// and the launcher that keeps the plan in a file-scope device array for callers that cannot
// bring a workspace (kvm_merge_static).
#include <mutex>

#include "kvm_common.h"

namespace kvm {

constexpr int MERGE_BLOCK = 64;          // one wave per workgroup: waves finish independently
constexpr int MERGE_TILE = 64;           // tokens per wave (its sets are those that start in the tile)
constexpr int PLAN_BLOCK = 256;
// Sets of more than LONG_SET_MIN tokens are left to merge_long_kernel, which puts a whole workgroup
// on each of them: one wave would stream such a set for hundreds of dependent round trips while
// the rest of the chip has nothing to do (identical keys make one set of a whole slice).
constexpr int LONG_SET_MIN = 512;
constexpr int LONG_SET_BLOCK = 1024;
// 4-row groups whose loads are issued together: 16 rows of K and of V.  Larger batches read
// more sets in a single sweep but cost registers; the kernel is bound by memory latency, and
// four waves per SIMD with 16-row batches beat two waves with 32-row batches.
template <typename T> struct MergeUnroll { static constexpr int value = 4; };

// int32 entries of a slice's plan: tiles + 1 tile edges, the number of long sets, their indices
static int merge_plan_stride(int N)
{
    const int tiles = (N + MERGE_TILE - 1) / MERGE_TILE;
    return tiles + 2 + N / (LONG_SET_MIN + 1) + 1;
}

size_t merge_workspace_bytes(const kvm_shape &sh)
{
    return (size_t)sh.B * sh.H_kv * merge_plan_stride(sh.N) * sizeof(int32_t);
}

struct MergeArgs {
    const int32_t *set_start, *pivot, *n_sets, *seq_lens;
    float *w_opt;
    const int32_t *plan;    // (slices, plan_stride): first set starting at or after each of the tiles_per_slice + 1
                            // tile edges, then the number of long sets of the slice, then their indices
    int plan_stride;
    int H, N, cap_rows, tiles_per_slice;
    int mode;               // MERGE_ADAPTIVE, MERGE_FIXED (uses inv_two_sigma_sq) or MERGE_AVERAGE
    float inv_two_sigma_sq; // 1 / (2 sigma^2) for the fixed-sigma mode
    int value_scale;
};

// plan[t] = smallest s with set_start[s] >= t * MERGE_TILE (M if there is none), t = 0..tiles;
// plan[tiles + 1] = number of sets of more than LONG_SET_MIN tokens, their indices after it (in no
// particular order: each is merged on its own).
__global__ __launch_bounds__(PLAN_BLOCK) void merge_plan_kernel(const int32_t *__restrict__ set_start,
                                                                const int32_t *__restrict__ n_sets,
                                                                const int32_t *__restrict__ seq_lens, int32_t *__restrict__ plan,
                                                                int H, int N, int cap_rows, int tiles, int plan_stride)
{
    __shared__ int n_long;
    const int slice = blockIdx.x;
    const int n = clamp_len(seq_lens, slice / H, N);
    const int M = min(max(n_sets[slice], 0), cap_rows);
    const int32_t *sst = set_start + (size_t)slice * (cap_rows + 1);
    int32_t *pl = plan + (size_t)slice * plan_stride;
    const int max_long = plan_stride - (tiles + 2);
    if (threadIdx.x == 0) n_long = 0;
    __syncthreads();
    for (int s = threadIdx.x; s <= M; s += PLAN_BLOCK) {
        const int prev = s > 0 ? min(max(sst[s - 1], 0), n) : -1;
        const int t_lo = prev < 0 ? 0 : prev / MERGE_TILE + 1;
        const int here = min(max(sst[s], 0), n);              // (set_start has an entry for s = M too: the end of the last stored set)
        const int t_hi = s < M ? min(here / MERGE_TILE, tiles) : tiles;
        for (int t = t_lo; t <= t_hi; ++t) pl[t] = s;
        if (s > 0 && here - prev > LONG_SET_MIN) {               // set s-1 = [prev, here)
            const int k = atomicAdd(&n_long, 1);
            if (k < max_long) pl[tiles + 2 + k] = s - 1;       // (with consistent maps there is always room)
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) pl[tiles + 1] = min(n_long, max_long);
}

// Squared distance of 8 elements, summed over the 16 lanes of the row.
__device__ __forceinline__ float sq_dist16(const float *kp, const float *x) {
    float d[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) d[e] = kp[e] - x[e];
    const float s0 = fmaf(d[1], d[1], d[0] * d[0]), s1 = fmaf(d[3], d[3], d[2] * d[2]);
    const float s2 = fmaf(d[5], d[5], d[4] * d[4]), s3 = fmaf(d[7], d[7], d[6] * d[6]);
    return row16_sum((s0 + s1) + (s2 + s3));
}

// WITH_W: also write the per-token weights.  MODE: how the weights are formed -- Gaussian
// kernel with sigma derived from the set, Gaussian kernel with a given sigma, or uniform
// (average weighted merging).  Both are compile-time so that the row loops stay free of
// branches and the compiler can interleave the independent rows.
enum { MERGE_ADAPTIVE = 0, MERGE_FIXED = 1, MERGE_AVERAGE = 2 };

// One set [lo, hi) of 1 .. LONG_SET_MIN tokens with pivot p (lo <= p < hi), merged by one wave into
// the rows k_row, v_row.  Shared by merge_kernel and the refresh of single sets, so that a set gives
// the same bits wherever it is merged.
template <typename T, bool WITH_W, int MODE>
__device__ __forceinline__ void merge_one_set(const T *Ks, const T *Vs, T *k_row, T *v_row, float *wo, int lo, int hi, int p,
                                              const MergeArgs &a, int lane)
{
    using E = Elem<T>;
    using Raw = typename E::Raw;
    constexpr int U = MergeUnroll<T>::value;   // row groups (of 4 rows) in flight
    const int slot = lane >> 4;          // which of the four rows of an instruction
    const int c = lane & 15;             // which 8-element chunk of the row
    const int m = hi - lo;
    const Raw kp_raw = E::load(Ks + (size_t)p * HEAD_DIM, c);
    float kp[8];
    float ak[8], av[8], gsum = 0.f, inv_mean = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ak[e] = 0.f; av[e] = 0.f; }
    // Rows past the end of the set are clamped to its last row and given weight zero, so
    // that every lane runs the same straight-line code.
    auto load_rows = [&](const T *base, int j0, Raw *r) {
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = E::load(base + (size_t)min(j0 + 4 * u + slot, hi - 1) * HEAD_DIM, c);
    };
    auto distances = [&](int j0, const Raw *kr) {
        float acc = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float x[8];
            E::to_float(kr[u], x);
            const float dist = __builtin_amdgcn_sqrtf(sq_dist16(kp, x));
            acc += (j0 + 4 * u + slot < hi) ? dist : 0.f;
        }
        return acc;
    };
    // g_j = exp(-D_j^2 / (2 sigma^2)); with sigma = dsum / (sqrt(2) m) that is exp(-(D_j m / dsum)^2)
    auto accumulate = [&](int j0, const Raw *kr, const Raw *vr) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = j0 + 4 * u + slot;
            float x[8], v[8];
            E::to_float(kr[u], x);
            float g;
            if (MODE == MERGE_AVERAGE) {
                g = 1.f;
            } else if (MODE == MERGE_FIXED) {
                g = __expf(-sq_dist16(kp, x) * a.inv_two_sigma_sq);
            } else {
                const float r = __builtin_amdgcn_sqrtf(sq_dist16(kp, x)) * inv_mean;
                g = __expf(-r * r);
            }
            g = row < hi ? g : 0.f;
            gsum += g;
            E::to_float(vr[u], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) { ak[e] = fmaf(g, x[e], ak[e]); av[e] = fmaf(g, v[e], av[e]); }
            if (WITH_W && c == 0 && row < hi) wo[row] = g;
        }
    };

    if (m <= 4 * U) {
        // the whole set is read once: all loads issued together, both sweeps from registers
        Raw k0[U], v0[U];
        load_rows(Ks, lo, k0);
        load_rows(Vs, lo, v0);
        E::to_float(kp_raw, kp);
        if (MODE == MERGE_ADAPTIVE) {
            const float dsum = rows4_sum(distances(lo, k0));
            inv_mean = dsum > 0.f ? (float)m / dsum : 0.f;
        }
        accumulate(lo, k0, v0);
    } else {
        E::to_float(kp_raw, kp);
        if (MODE == MERGE_ADAPTIVE) {
            // sweep 1: sum of the distances to the pivot
            float dsum = 0.f;
            for (int j0 = lo; j0 < hi; j0 += 4 * U) {
                Raw kr[U];
                load_rows(Ks, j0, kr);
                dsum += distances(j0, kr);
            }
            dsum = rows4_sum(dsum);
            inv_mean = dsum > 0.f ? (float)m / dsum : 0.f;
        }
        // sweep 2: weights and weighted sums (K again, now from L2; V for the first time)
        for (int j0 = lo; j0 < hi; j0 += 4 * U) {
            Raw kr[U], vr[U];
            load_rows(Ks, j0, kr);
            load_rows(Vs, j0, vr);
            accumulate(j0, kr, vr);
        }
    }
    gsum = rows4_sum(gsum);
    const float inv_g = 1.f / gsum;
    const float vscale = a.value_scale ? inv_g * (float)m : inv_g;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        ak[e] = rows4_sum(ak[e]) * inv_g;
        av[e] = rows4_sum(av[e]) * vscale;
    }
    if (slot == 0) E::store(k_row, c, E::from_float(ak));
    if (slot == 1) E::store(v_row, c, E::from_float(av));
    if (WITH_W && c == 0) {                                        // each writer normalises its own g_j
        for (int row = lo + slot; row < hi; row += 4) wo[row] *= inv_g;
    }
}

template <typename T, bool WITH_W, int MODE>
__global__ __launch_bounds__(MERGE_BLOCK) void merge_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                            T *__restrict__ K_out, T *__restrict__ V_out, MergeArgs a)
{
    using E = Elem<T>;
    using Raw = typename E::Raw;
    constexpr int US = 4;                      // row groups (of 4 rows) in flight in runs of singleton sets
    const int slice = blockIdx.x / a.tiles_per_slice;
    const int tile = blockIdx.x - slice * a.tiles_per_slice;
    const int lane = threadIdx.x & 63;
    const int slot = lane >> 4;          // which of the four rows of an instruction
    const int c = lane & 15;             // which 8-element chunk of the row
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    if (tile * MERGE_TILE >= n) return;
    const int M = min(max(a.n_sets[slice], 0), a.cap_rows);
    // sets [s_lo, s_hi) start inside this tile (entries are clamped: the plan may hold garbage
    // when the maps are inconsistent)
    const int32_t *pl = a.plan + (size_t)slice * a.plan_stride + tile;
    const int s_lo = min(max(pl[0], 0), M);
    const int s_hi = min(max(pl[1], s_lo), M);
    const int cnt = min(s_hi - s_lo, MERGE_TILE);
    if (cnt == 0) return;

    const int32_t *sst = a.set_start + (size_t)slice * (a.cap_rows + 1);
    const int32_t *piv = a.pivot + (size_t)slice * a.cap_rows;
    const T *Ks = K + (size_t)slice * a.N * HEAD_DIM;
    const T *Vs = V + (size_t)slice * a.N * HEAD_DIM;
    T *Ko = K_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    T *Vo = V_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    float *wo = WITH_W ? a.w_opt + (size_t)slice * a.N : nullptr;

    // lane i holds the first token of set s_lo+i and its pivot; entries are clamped into the
    // slice so that inconsistent maps cannot address outside K and V
    int my_start = n, my_piv = 0;
    if (lane < cnt) {
        my_start = min(max(sst[s_lo + lane], 0), n);
        my_piv = piv[s_lo + lane];
    }
    const int t_end = min(max(sst[s_lo + cnt], 0), n);               // end of the wave's last set
    int my_next = __shfl_down(my_start, 1, WAVE);
    if (lane == cnt - 1) my_next = t_end;
    const unsigned long long single_mask = __ballot(lane < cnt && my_next - my_start == 1);

    int i = 0;
    while (i < cnt) {
        // ---- runs of singleton sets: plain copy, up to 4*U sets per step, all loads in flight ------
        if ((single_mask >> i) & 1ull) {
            int run = 1;
            while (run < 4 * US && i + run < cnt && ((single_mask >> (i + run)) & 1ull)) ++run;
            Raw rk[US], rv[US];
            int src[US];
#pragma unroll
            for (int u = 0; u < US; ++u) {
                const int r = 4 * u + slot;
                src[u] = __shfl(my_start, i + min(r, run - 1), WAVE);
                if (r < run) {
                    rk[u] = E::load(Ks + (size_t)src[u] * HEAD_DIM, c);
                    rv[u] = E::load(Vs + (size_t)src[u] * HEAD_DIM, c);
                }
            }
#pragma unroll
            for (int u = 0; u < US; ++u) {
                const int r = 4 * u + slot;
                if (r < run) {
                    E::store(Ko + (size_t)(s_lo + i + r) * HEAD_DIM, c, rk[u]);
                    E::store(Vo + (size_t)(s_lo + i + r) * HEAD_DIM, c, rv[u]);
                    if (WITH_W && c == 0) wo[src[u]] = 1.f;
                }
            }
            i += run;
            continue;
        }
        // ---- a set with several tokens --------------------------------------------------------------
        const int lo = __builtin_amdgcn_readlane(my_start, i);
        const int hi = __builtin_amdgcn_readlane(my_next, i);
        const int m = hi - lo;
        if (m <= 0 || m > LONG_SET_MIN) { ++i; continue; }                // inconsistent map: nothing to merge; long set: merge_long_kernel
        int p = __builtin_amdgcn_readlane(my_piv, i);
        p = min(max(p, lo), hi - 1);
        merge_one_set<T, WITH_W, MODE>(Ks, Vs, Ko + (size_t)(s_lo + i) * HEAD_DIM, Vo + (size_t)(s_lo + i) * HEAD_DIM, wo, lo, hi, p, a,
                                       lane);
        ++i;
    }
}

// Sets of more than LONG_SET_MIN tokens, one after the other, by all 64 sixteen-lane groups of a
// 1024-thread workgroup per slice: group g takes the set's rows g, g + 64, ... (four of them in
// flight), the distance sum and then the weighted sums are added up across the groups through
// LDS.  Same arithmetic per row as merge_kernel; only the order of the fp32 additions differs.
template <typename T, bool WITH_W, int MODE>
__global__ __launch_bounds__(LONG_SET_BLOCK) void merge_long_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                                T *__restrict__ K_out, T *__restrict__ V_out, MergeArgs a)
{
    using E = Elem<T>;
    using Raw = typename E::Raw;
    constexpr int U = 4;                                     // rows of a group in flight
    constexpr int GROUPS = LONG_SET_BLOCK / 16, WAVES = LONG_SET_BLOCK / WAVE;
    __shared__ float red[WAVES][16][17];                     // per wave and chunk lane: 8 key sums, 8 value sums, weight sum
    __shared__ float red1[WAVES];
    const int slice = blockIdx.x;
    const int32_t *pl = a.plan + (size_t)slice * a.plan_stride + a.tiles_per_slice + 1;
    const int n_long = min(max(pl[0], 0), a.plan_stride - (a.tiles_per_slice + 2));
    if (n_long == 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = tid & 15, group = tid >> 4;
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    const int M = min(max(a.n_sets[slice], 0), a.cap_rows);
    const int32_t *sst = a.set_start + (size_t)slice * (a.cap_rows + 1);
    const int32_t *piv = a.pivot + (size_t)slice * a.cap_rows;
    const T *Ks = K + (size_t)slice * a.N * HEAD_DIM;
    const T *Vs = V + (size_t)slice * a.N * HEAD_DIM;
    T *Ko = K_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    T *Vo = V_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    float *wo = WITH_W ? a.w_opt + (size_t)slice * a.N : nullptr;

    for (int k = 0; k < n_long; ++k) {
        const int s = pl[1 + k];
        if (s < 0 || s >= M) continue;                        // (the same for the whole workgroup)
        const int lo = min(max(sst[s], 0), n), hi = min(max(sst[s + 1], 0), n);
        const int m = hi - lo;
        if (m <= LONG_SET_MIN) continue;
        const int p = min(max(piv[s], lo), hi - 1);
        float kp[8];
        E::to_float(E::load(Ks + (size_t)p * HEAD_DIM, c), kp);
        float inv_mean = 0.f;
        if (MODE == MERGE_ADAPTIVE) {
            float dsum = 0.f;
            for (int j0 = lo + group; j0 < hi; j0 += GROUPS * U) {
                Raw kr[U];
#pragma unroll
                for (int u = 0; u < U; ++u) kr[u] = E::load(Ks + (size_t)min(j0 + GROUPS * u, hi - 1) * HEAD_DIM, c);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float x[8];
                    E::to_float(kr[u], x);
                    const float dist = __builtin_amdgcn_sqrtf(sq_dist16(kp, x));
                    dsum += (j0 + GROUPS * u < hi) ? dist : 0.f;
                }
            }
            dsum = rows4_sum(dsum);                           // the wave's four groups
            __syncthreads();                                  // red1 may still be read from the set before
            if (lane == 0) red1[wave] = dsum;
            __syncthreads();
            float total = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < WAVES; ++w2) total += red1[w2];
            inv_mean = total > 0.f ? (float)m / total : 0.f;
        }
        float ak[8], av[8], gsum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { ak[e] = 0.f; av[e] = 0.f; }
        for (int j0 = lo + group; j0 < hi; j0 += GROUPS * U) {
            Raw kr[U], vr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t row = (size_t)min(j0 + GROUPS * u, hi - 1) * HEAD_DIM;
                kr[u] = E::load(Ks + row, c);
                vr[u] = E::load(Vs + row, c);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = j0 + GROUPS * u;
                float x[8], v[8];
                E::to_float(kr[u], x);
                float g;
                if (MODE == MERGE_AVERAGE) {
                    g = 1.f;
                } else if (MODE == MERGE_FIXED) {
                    g = __expf(-sq_dist16(kp, x) * a.inv_two_sigma_sq);
                } else {
                    const float r = __builtin_amdgcn_sqrtf(sq_dist16(kp, x)) * inv_mean;
                    g = __expf(-r * r);
                }
                g = row < hi ? g : 0.f;
                gsum += g;
                E::to_float(vr[u], v);
#pragma unroll
                for (int e = 0; e < 8; ++e) { ak[e] = fmaf(g, x[e], ak[e]); av[e] = fmaf(g, v[e], av[e]); }
                if (WITH_W && c == 0 && row < hi) wo[row] = g;
            }
        }
        gsum = rows4_sum(gsum);
#pragma unroll
        for (int e = 0; e < 8; ++e) { ak[e] = rows4_sum(ak[e]); av[e] = rows4_sum(av[e]); }
        __syncthreads();                                      // red may still be read from the set before
        if (lane < 16) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { red[wave][c][e] = ak[e]; red[wave][c][8 + e] = av[e]; }
            red[wave][c][16] = gsum;
        }
        __syncthreads();
        float gtot = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < WAVES; ++w2) gtot += red[w2][0][16];
        const float inv_g = 1.f / gtot;
        if (tid < 32) {                                       // lanes 0..15: the key row, 16..31: the value row
            const bool is_v = tid >= 16;
            const float scale = is_v && a.value_scale ? inv_g * (float)m : inv_g;
            float out[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float t = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < WAVES; ++w2) t += red[w2][c][(is_v ? 8 : 0) + e];
                out[e] = t * scale;
            }
            E::store((is_v ? Vo : Ko) + (size_t)s * HEAD_DIM, c, E::from_float(out));
        }
        if (WITH_W && c == 0) {                               // each writer normalises its own g_j
            for (int row = lo + group; row < hi; row += GROUPS) wo[row] *= inv_g;
        }
    }
}

template <typename T>
static void launch_merge_t(const kvm_shape &sh, const void *K, const void *V, void *K_out, void *V_out,
                           const MergeArgs &a, hipStream_t st)
{
    const long long blocks = (long long)sh.B * sh.H_kv * a.tiles_per_slice;
    ProfScope prof("merge_kernel", st);
    const dim3 grid((unsigned)blocks), block(MERGE_BLOCK);
    const T *k = (const T *)K, *v = (const T *)V;
    T *ko = (T *)K_out, *vo = (T *)V_out;
    if (a.w_opt) {
        if (a.mode == MERGE_AVERAGE) hipLaunchKernelGGL((merge_kernel<T, true, MERGE_AVERAGE>), grid, block, 0, st, k, v, ko, vo, a);
        else if (a.mode == MERGE_FIXED) hipLaunchKernelGGL((merge_kernel<T, true, MERGE_FIXED>), grid, block, 0, st, k, v, ko, vo, a);
        else hipLaunchKernelGGL((merge_kernel<T, true, MERGE_ADAPTIVE>), grid, block, 0, st, k, v, ko, vo, a);
    } else {
        if (a.mode == MERGE_AVERAGE) hipLaunchKernelGGL((merge_kernel<T, false, MERGE_AVERAGE>), grid, block, 0, st, k, v, ko, vo, a);
        else if (a.mode == MERGE_FIXED) hipLaunchKernelGGL((merge_kernel<T, false, MERGE_FIXED>), grid, block, 0, st, k, v, ko, vo, a);
        else hipLaunchKernelGGL((merge_kernel<T, false, MERGE_ADAPTIVE>), grid, block, 0, st, k, v, ko, vo, a);
    }
}

template <typename T>
static void launch_merge_long_t(const kvm_shape &sh, const void *K, const void *V, void *K_out, void *V_out,
                                const MergeArgs &a, hipStream_t st)
{
    ProfScope prof("merge_long_kernel", st);
    const dim3 grid((unsigned)((long long)sh.B * sh.H_kv)), block(LONG_SET_BLOCK);
    const T *k = (const T *)K, *v = (const T *)V;
    T *ko = (T *)K_out, *vo = (T *)V_out;
    if (a.w_opt) {
        if (a.mode == MERGE_AVERAGE) hipLaunchKernelGGL((merge_long_kernel<T, true, MERGE_AVERAGE>), grid, block, 0, st, k, v, ko, vo, a);
        else if (a.mode == MERGE_FIXED) hipLaunchKernelGGL((merge_long_kernel<T, true, MERGE_FIXED>), grid, block, 0, st, k, v, ko, vo, a);
        else hipLaunchKernelGGL((merge_long_kernel<T, true, MERGE_ADAPTIVE>), grid, block, 0, st, k, v, ko, vo, a);
    } else {
        if (a.mode == MERGE_AVERAGE) hipLaunchKernelGGL((merge_long_kernel<T, false, MERGE_AVERAGE>), grid, block, 0, st, k, v, ko, vo, a);
        else if (a.mode == MERGE_FIXED) hipLaunchKernelGGL((merge_long_kernel<T, false, MERGE_FIXED>), grid, block, 0, st, k, v, ko, vo, a);
        else hipLaunchKernelGGL((merge_long_kernel<T, false, MERGE_ADAPTIVE>), grid, block, 0, st, k, v, ko, vo, a);
    }
}

kvm_status launch_merge(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                        const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out,
                        void *V_out, float *w_opt, int32_t *plan, hipStream_t st)
{
    if ((long long)sh.B * sh.H_kv == 0 || cap_rows == 0 || sh.N == 0) return KVM_OK;
    MergeArgs a;
    a.set_start = set_start;
    a.pivot = pivot;
    a.n_sets = n_sets;
    a.seq_lens = sh.seq_lens;
    a.w_opt = w_opt;
    a.plan = plan;
    a.H = sh.H_kv;
    a.N = sh.N;
    a.cap_rows = cap_rows;
    a.tiles_per_slice = (sh.N + MERGE_TILE - 1) / MERGE_TILE;
    a.plan_stride = merge_plan_stride(sh.N);
    a.mode = pr.weights == KVM_WEIGHTS_AVERAGE ? MERGE_AVERAGE : (pr.sigma_mode == KVM_SIGMA_FIXED ? MERGE_FIXED : MERGE_ADAPTIVE);
    a.inv_two_sigma_sq = a.mode == MERGE_FIXED ? 1.f / (2.f * pr.sigma * pr.sigma) : 0.f;
    a.value_scale = pr.value_scale_by_set_size;
    {
        ProfScope prof("merge_plan_kernel", st);
        hipLaunchKernelGGL(merge_plan_kernel, dim3((unsigned)(sh.B * sh.H_kv)), dim3(PLAN_BLOCK), 0, st, set_start, n_sets,
                           sh.seq_lens, plan, sh.H_kv, sh.N, cap_rows, a.tiles_per_slice, a.plan_stride);
        kvm_status rc = check_launch("merge_plan_kernel");
        if (rc != KVM_OK) return rc;
    }
    switch (sh.dtype) {
    case KVM_F32: launch_merge_t<float>(sh, K, V, K_out, V_out, a, st); break;
    case KVM_F16: launch_merge_t<half_t>(sh, K, V, K_out, V_out, a, st); break;
    default: launch_merge_t<bf16_t>(sh, K, V, K_out, V_out, a, st); break;
    }
    kvm_status rc = check_launch("merge_kernel");
    if (rc != KVM_OK || sh.N <= LONG_SET_MIN) return rc;          // (no slice can hold a long set)
    switch (sh.dtype) {
    case KVM_F32: launch_merge_long_t<float>(sh, K, V, K_out, V_out, a, st); break;
    case KVM_F16: launch_merge_long_t<half_t>(sh, K, V, K_out, V_out, a, st); break;
    default: launch_merge_long_t<bf16_t>(sh, K, V, K_out, V_out, a, st); break;
    }
    return check_launch("merge_long_kernel");
}

// ------------------------------------------------------------------------------------------
// Refresh of a compacted cache after the index maps changed a little (decode time: one more
// token moves the recent window, the top-k and a few pivots).  A set of the new maps whose
// extent and pivot already existed in the previous maps has the same merged row as before:
// the row only moves to its new index; the others are merged again.  Result: bit for bit what
// merge_kernel / merge_long_kernel give on the new maps.
//
// refresh_kernel, one 512-thread workgroup per slice, three phases with a barrier between them:
//   compare   src[s] = row of the previous cache that new row s is (-1: merge again), the list
//             of short sets to merge again, and the long ones in the layout merge_long_kernel
//             reads (that kernel follows)
//   move      rows in place.  src is increasing over the rows that move, so rows moving up
//             never need a row that rows moving down overwrite and vice versa; rows moving up
//             are taken from the top down, rows moving down from the bottom up, a batch at a time,
//             all reads of a batch before its writes.
//   merge     one wave per listed set (merge_one_set), the workgroup's waves in turn.  A
//             slice that has little to move gets here early, so the longest set of the launch
//             (one wave, up to LONG_SET_MIN rows) overlaps the other slices' moves.
// ------------------------------------------------------------------------------------------

struct RefreshArgs {
    const int32_t *prev_set_id, *prev_set_start, *prev_pivot, *prev_n_sets;
    int32_t *src;          // (slices, cap_rows)
    int32_t *lists;        // (slices, cap_rows + 1): number of short sets to merge again, then their indices
    int32_t *plan;         // what MergeArgs::plan points to; only the long-set part is filled
    int32_t *n_changed;    // (slices) or NULL: sets merged again
};

constexpr int REFRESH_BLOCK = 512;                           // two workgroups per compute unit (128 registers each)
template <typename T> struct MovePerGroup { static constexpr int value = 16 / sizeof(T); };   // rows a 16-lane group moves per batch

template <typename T, int MODE>
__global__ __launch_bounds__(REFRESH_BLOCK, 4) void refresh_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                                T *__restrict__ K_out, T *__restrict__ V_out, MergeArgs a,
                                                                RefreshArgs r)
{
    using E = Elem<T>;
    using Raw = typename E::Raw;
    constexpr int MOVE_PER_GROUP = MovePerGroup<T>::value;
    constexpr int MOVE_BATCH = (REFRESH_BLOCK / 16) * MOVE_PER_GROUP;   // rows the workgroup moves per batch
    __shared__ int n_short, n_long, first_moved, any_up, any_down;
    const int slice = blockIdx.x;
    const int tid = threadIdx.x, c = tid & 15, group = tid >> 4;
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    const int M = min(max(a.n_sets[slice], 0), a.cap_rows);
    const int M_old = min(max(r.prev_n_sets[slice], 0), a.cap_rows);
    const int32_t *sst = a.set_start + (size_t)slice * (a.cap_rows + 1);
    const int32_t *piv = a.pivot + (size_t)slice * a.cap_rows;
    const int32_t *osst = r.prev_set_start + (size_t)slice * (a.cap_rows + 1);
    const int32_t *opiv = r.prev_pivot + (size_t)slice * a.cap_rows;
    const int32_t *osid = r.prev_set_id + (size_t)slice * a.N;
    int32_t *src = r.src + (size_t)slice * a.cap_rows;
    int32_t *list = r.lists + (size_t)slice * (a.cap_rows + 1);
    int32_t *pl = r.plan + (size_t)slice * a.plan_stride + a.tiles_per_slice + 1;
    const int max_long = a.plan_stride - (a.tiles_per_slice + 2);
    T *Ko = K_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    T *Vo = V_out + (size_t)slice * a.cap_rows * HEAD_DIM;

    // ---- compare ------------------------------------------------------------------------------
    if (tid == 0) { n_short = 0; n_long = 0; first_moved = M; any_up = 0; any_down = 0; }
    __syncthreads();
    int my_first = M;
    bool my_up = false, my_down = false;
    for (int s = tid; s < M; s += REFRESH_BLOCK) {
        const int lo = min(max(sst[s], 0), n), hi = min(max(sst[s + 1], 0), n);
        int from = -1;
        if (hi > lo) {
            const int so = osid[lo];                          // the previous set of the new set's first token
            if (so >= 0 && so < M_old && osst[so] == sst[s] && osst[so + 1] == sst[s + 1] && opiv[so] == piv[s]) from = so;
        }
        src[s] = from;
        if (from < 0) {
            if (hi - lo > LONG_SET_MIN) {
                const int k = atomicAdd(&n_long, 1);
                if (k < max_long) pl[1 + k] = s;
            } else {
                list[1 + atomicAdd(&n_short, 1)] = s;
            }
        } else if (from != s) {
            my_first = min(my_first, s);
            my_up |= from < s;
            my_down |= from > s;
        }
    }
    if (my_first < M) atomicMin(&first_moved, my_first);
    if (my_up) any_up = 1;
    if (my_down) any_down = 1;
    __syncthreads();                                          // src and list are read below by other threads of this workgroup
    const int first = first_moved;
    const bool moves_up = any_up != 0, moves_down = any_down != 0;
    const int cnt = n_short;
    if (tid == 0) {
        list[0] = cnt;
        pl[0] = min(n_long, max_long);
        if (r.n_changed) r.n_changed[slice] = cnt + n_long;
    }

    // ---- move ---------------------------------------------------------------------------------
    // (a direction that no row takes is skipped as a whole: after one more token nearly all rows
    // that move go the same way)
    const int b_lo = first / MOVE_BATCH, b_hi = (M - 1) / MOVE_BATCH;
    int s[MOVE_PER_GROUP], f[MOVE_PER_GROUP], f_next[MOVE_PER_GROUP];
    Raw rk[MOVE_PER_GROUP], rv[MOVE_PER_GROUP];
    auto sources = [&](int bt, int *out) {                    // the batch's sources, before the direction filter
#pragma unroll
        for (int u = 0; u < MOVE_PER_GROUP; ++u) {
            const int row = bt * MOVE_BATCH + u * (REFRESH_BLOCK / 16) + group;
            out[u] = row < M ? src[row] : -1;
        }
    };
    auto move_batch = [&](int bt, bool up, int bt_next, bool more) {
        bool any = false;
#pragma unroll
        for (int u = 0; u < MOVE_PER_GROUP; ++u) {
            s[u] = bt * MOVE_BATCH + u * (REFRESH_BLOCK / 16) + group;
            f[u] = f_next[u];
            if (!(up ? (f[u] >= 0 && f[u] < s[u]) : f[u] > s[u])) f[u] = -1;
            any |= f[u] >= 0;
        }
        if (more) sources(bt_next, f_next);                   // in flight across the barriers
        if (!__syncthreads_or(any ? 1 : 0)) return;
#pragma unroll
        for (int u = 0; u < MOVE_PER_GROUP; ++u)
            if (f[u] >= 0) { rk[u] = E::load(Ko + (size_t)f[u] * HEAD_DIM, c); rv[u] = E::load(Vo + (size_t)f[u] * HEAD_DIM, c); }
        __syncthreads();                                      // every source row of the batch is in registers
#pragma unroll
        for (int u = 0; u < MOVE_PER_GROUP; ++u)
            if (f[u] >= 0) { E::store(Ko + (size_t)s[u] * HEAD_DIM, c, rk[u]); E::store(Vo + (size_t)s[u] * HEAD_DIM, c, rv[u]); }
    };
    if (moves_up) {                                           // new index above the old one: batches from the top down
        sources(b_hi, f_next);
        for (int bt = b_hi; bt >= b_lo; --bt) move_batch(bt, true, bt - 1, bt > b_lo);
    }
    if (moves_up && moves_down) __syncthreads();
    if (moves_down) {                                         // batches from the bottom up
        sources(b_lo, f_next);
        for (int bt = b_lo; bt <= b_hi; ++bt) move_batch(bt, false, bt + 1, bt < b_hi);
    }
    if (moves_up || moves_down) __syncthreads();              // a row merged below may be one that was a source above

    // ---- merge the listed sets again -------------------------------------------------------------
    const int lane = tid & 63;
    const T *Ks = K + (size_t)slice * a.N * HEAD_DIM;
    const T *Vs = V + (size_t)slice * a.N * HEAD_DIM;
    for (int k = tid >> 6; k < cnt; k += REFRESH_BLOCK / WAVE) {
        const int s = list[1 + k];
        if (s < 0 || s >= M) continue;                        // (the same for the whole wave)
        const int lo = min(max(sst[s], 0), n), hi = min(max(sst[s + 1], 0), n);
        if (hi - lo <= 0 || hi - lo > LONG_SET_MIN) continue;
        const int p = min(max(piv[s], lo), hi - 1);
        merge_one_set<T, false, MODE>(Ks, Vs, Ko + (size_t)s * HEAD_DIM, Vo + (size_t)s * HEAD_DIM, nullptr, lo, hi, p, a, lane);
    }
}

template <typename T>
static kvm_status launch_refresh_t(const kvm_shape &sh, const void *K, const void *V, void *K_out, void *V_out,
                                   const MergeArgs &ma, const RefreshArgs &ra, hipStream_t st)
{
    const dim3 grid((unsigned)((long long)sh.B * sh.H_kv)), block(REFRESH_BLOCK);
    {
        ProfScope prof("refresh_kernel", st);
        const T *k = (const T *)K, *v = (const T *)V;
        T *ko = (T *)K_out, *vo = (T *)V_out;
        if (ma.mode == MERGE_AVERAGE) hipLaunchKernelGGL((refresh_kernel<T, MERGE_AVERAGE>), grid, block, 0, st, k, v, ko, vo, ma, ra);
        else if (ma.mode == MERGE_FIXED) hipLaunchKernelGGL((refresh_kernel<T, MERGE_FIXED>), grid, block, 0, st, k, v, ko, vo, ma, ra);
        else hipLaunchKernelGGL((refresh_kernel<T, MERGE_ADAPTIVE>), grid, block, 0, st, k, v, ko, vo, ma, ra);
    }
    kvm_status rc = check_launch("refresh_kernel");
    if (rc != KVM_OK || sh.N <= LONG_SET_MIN) return rc;
    launch_merge_long_t<T>(sh, K, V, K_out, V_out, ma, st);
    return check_launch("merge_long_kernel");
}

size_t merge_refresh_workspace_bytes(const kvm_shape &sh, int cap_rows)
{
    return (size_t)sh.B * sh.H_kv * ((size_t)merge_plan_stride(sh.N) + 2 * (size_t)cap_rows + 1) * sizeof(int32_t);
}

kvm_status launch_merge_refresh(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                                const int32_t *prev_set_id, const int32_t *prev_set_start, const int32_t *prev_pivot,
                                const int32_t *prev_n_sets, const int32_t *set_start, const int32_t *pivot,
                                const int32_t *n_sets, void *K_out, void *V_out, int32_t *n_changed, int32_t *ws, hipStream_t st)
{
    const size_t slices = (size_t)sh.B * sh.H_kv;
    if (slices == 0 || cap_rows == 0 || sh.N == 0) return KVM_OK;
    const int plan_stride = merge_plan_stride(sh.N);
    RefreshArgs ra;
    ra.prev_set_id = prev_set_id;
    ra.prev_set_start = prev_set_start;
    ra.prev_pivot = prev_pivot;
    ra.prev_n_sets = prev_n_sets;
    ra.src = ws + slices * plan_stride;
    ra.lists = ra.src + slices * cap_rows;
    ra.plan = ws;
    ra.n_changed = n_changed;
    MergeArgs ma;
    ma.set_start = set_start;
    ma.pivot = pivot;
    ma.n_sets = n_sets;
    ma.seq_lens = sh.seq_lens;
    ma.w_opt = nullptr;
    ma.plan = ws;
    ma.plan_stride = plan_stride;
    ma.H = sh.H_kv;
    ma.N = sh.N;
    ma.cap_rows = cap_rows;
    ma.tiles_per_slice = (sh.N + MERGE_TILE - 1) / MERGE_TILE;
    ma.mode = pr.weights == KVM_WEIGHTS_AVERAGE ? MERGE_AVERAGE : (pr.sigma_mode == KVM_SIGMA_FIXED ? MERGE_FIXED : MERGE_ADAPTIVE);
    ma.inv_two_sigma_sq = ma.mode == MERGE_FIXED ? 1.f / (2.f * pr.sigma * pr.sigma) : 0.f;
    ma.value_scale = pr.value_scale_by_set_size;
    switch (sh.dtype) {
    case KVM_F32: return launch_refresh_t<float>(sh, K, V, K_out, V_out, ma, ra, st);
    case KVM_F16: return launch_refresh_t<half_t>(sh, K, V, K_out, V_out, ma, ra, st);
    default: return launch_refresh_t<bf16_t>(sh, K, V, K_out, V_out, ma, ra, st);
    }
}

// ------------------------------------------------------------------------------------------
// The merge for callers that cannot allocate: the work plan goes into a file-scope device
// array instead of a caller-supplied workspace.  Every GPU the library runs on holds its own
// copy of the array at its own address; the address is looked up once per device, with that
// device current, and host code only ever uses the looked-up pointer.
// ------------------------------------------------------------------------------------------

constexpr size_t STATIC_PLAN_INTS = (size_t)KVM_MERGE_STATIC_MAX_PLAN_ENTRIES;
static __device__ __align__(256) int32_t scratch[STATIC_PLAN_INTS];

constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static int32_t *g_scratch_ptr[STATIC_MAX_DEVICES];           // per device; nullptr = not looked up yet

static kvm_status static_plan_ptr(int32_t **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) {
        set_error("kvm_merge_static: no usable current device (%s)", e != hipSuccess ? hipGetErrorString(e) : "index out of range");
        return KVM_ERR_LAUNCH;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("kvm_merge_static: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
            return KVM_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = static_cast<int32_t *>(p);
    }
    *out = g_scratch_ptr[dev];
    return KVM_OK;
}

kvm_status launch_merge_static(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                               const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out,
                               void *V_out, float *w_opt, hipStream_t st)
{
    const size_t need = merge_workspace_bytes(sh) / sizeof(int32_t);
    if (need > STATIC_PLAN_INTS) {
        set_error("kvm_merge_static: the work plan needs %zu entries (B*H_kv*(ceil(N/64)+floor(N/513)+3)), the built-in buffer holds %zu; "
                  "use kvm_merge with a workspace", need, STATIC_PLAN_INTS);
        return KVM_ERR_WORKSPACE;
    }
    int32_t *plan = nullptr;
    kvm_status rc = static_plan_ptr(&plan);
    if (rc != KVM_OK) return rc;
    // every plan entry a merge wave reads is written by the plan kernel of the same call (or
    // clamped when the maps are inconsistent), so nothing has to be cleared between calls
    return launch_merge(sh, pr, cap_rows, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, plan, st);
}

}  // namespace kvm
