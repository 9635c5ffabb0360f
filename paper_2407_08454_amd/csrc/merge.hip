// Gaussian-kernel weighted merging with a compacting write (Section 4.2: Def. 4.2 Eq. (4),
// Eq. (5), (6); Algorithm 2).
//
// One wave owns MERGE_SETS_PER_WAVE consecutive output rows (sets) of one slice.  A row of
// 128 elements is spread over 16 lanes (8 elements = 16 B each for 16-bit types), so one
// wave instruction moves four rows.  Per set: one sweep over its keys for the distances to
// the pivot (sigma), a second sweep (served by L1/L2, the set was just read) that forms the
// weights and accumulates keys and values in fp32, then one rounded row is written per
// output.  Runs of singleton sets are copied bit for bit, four rows per instruction.
// HBM traffic: K once, V once, 2 M rows out.
#include "kvm_common.h"

namespace kvm {

constexpr int MERGE_BLOCK = 256;
constexpr int MERGE_SETS_PER_WAVE = 16;
constexpr int MERGE_SETS_PER_BLOCK = (MERGE_BLOCK / WAVE) * MERGE_SETS_PER_WAVE;

struct MergeArgs {
    const int32_t *set_start, *pivot, *n_sets, *seq_lens;
    float *w_opt;
    int H, N, cap_rows, blocks_per_slice;
    int sigma_fixed;        // 1: use inv_two_sigma_sq
    float inv_two_sigma_sq; // 1 / (2 sigma^2) for the fixed-sigma mode
    int value_scale;
};

template <typename T>
__global__ __launch_bounds__(MERGE_BLOCK) void merge_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                            T *__restrict__ K_out, T *__restrict__ V_out, MergeArgs a)
{
    const int slice = blockIdx.x / a.blocks_per_slice;
    const int blk = blockIdx.x - slice * a.blocks_per_slice;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int slot = lane >> 4;          // which of the four rows of an instruction
    const int c = lane & 15;             // which 8-element chunk of the row
    const int n = clamp_len(a.seq_lens, slice / a.H, a.N);
    int M = a.n_sets[slice];
    if (M > a.cap_rows) M = a.cap_rows;
    const int s_lo = blk * MERGE_SETS_PER_BLOCK + wave * MERGE_SETS_PER_WAVE;
    if (s_lo >= M) return;
    const int cnt = min(MERGE_SETS_PER_WAVE, M - s_lo);

    const int32_t *sst = a.set_start + (size_t)slice * (a.cap_rows + 1);
    const int32_t *piv = a.pivot + (size_t)slice * a.cap_rows;
    const T *Ks = K + (size_t)slice * a.N * HEAD_DIM;
    const T *Vs = V + (size_t)slice * a.N * HEAD_DIM;
    T *Ko = K_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    T *Vo = V_out + (size_t)slice * a.cap_rows * HEAD_DIM;
    float *wo = a.w_opt ? a.w_opt + (size_t)slice * a.N : nullptr;

    // lane i holds the first token of set s_lo+i (i <= cnt) and its pivot; entries are clamped
    // into the slice so that inconsistent maps cannot address outside K and V
    int my_start = n, my_piv = 0;
    if (lane <= cnt) my_start = min(max(sst[s_lo + lane], 0), n);
    if (lane < cnt) my_piv = piv[s_lo + lane];
    int my_len = __shfl_down(my_start, 1, WAVE) - my_start;       // lane i: |S_i| (garbage for i >= cnt)
    const unsigned long long single_mask = __ballot(lane < cnt && my_len == 1);

    int i = 0;
    while (i < cnt) {
        // ---- runs of singleton sets: plain copy, up to four sets per step --------------------------
        if ((single_mask >> i) & 1ull) {
            int run = 1;
            while (run < 4 && i + run < cnt && ((single_mask >> (i + run)) & 1ull)) ++run;
            const int src = __shfl(my_start, i + min(slot, run - 1), WAVE);
            if (slot < run) {
                typename Elem<T>::Raw rk = Elem<T>::load(Ks + (size_t)src * HEAD_DIM, c);
                typename Elem<T>::Raw rv = Elem<T>::load(Vs + (size_t)src * HEAD_DIM, c);
                Elem<T>::store(Ko + (size_t)(s_lo + i + slot) * HEAD_DIM, c, rk);
                Elem<T>::store(Vo + (size_t)(s_lo + i + slot) * HEAD_DIM, c, rv);
                if (wo && c == 0) wo[src] = 1.f;
            }
            i += run;
            continue;
        }
        // ---- a set with several tokens --------------------------------------------------------------
        const int lo = __builtin_amdgcn_readlane(my_start, i);
        const int hi = __builtin_amdgcn_readlane(my_start, i + 1);
        const int m = hi - lo;
        if (m <= 0) { ++i; continue; }                                // inconsistent map: nothing to merge
        int p = __builtin_amdgcn_readlane(my_piv, i);
        p = min(max(p, lo), hi - 1);
        float kp[8];
        Elem<T>::to_float(Elem<T>::load(Ks + (size_t)p * HEAD_DIM, c), kp);

        // first four rows stay in registers for the second sweep
        float x0[8];
        const bool v0 = lo + slot < hi;
#pragma unroll
        for (int e = 0; e < 8; ++e) x0[e] = 0.f;
        if (v0) Elem<T>::to_float(Elem<T>::load(Ks + (size_t)(lo + slot) * HEAD_DIM, c), x0);

        // sweep 1: distances to the pivot
        float dsum = 0.f;
        for (int j0 = lo; j0 < hi; j0 += 4) {
            const int row = j0 + slot;
            float x[8];
            if (j0 == lo) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = x0[e];
            } else if (row < hi) {
                Elem<T>::to_float(Elem<T>::load(Ks + (size_t)row * HEAD_DIM, c), x);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = kp[e];
            }
            float sq = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float df = kp[e] - x[e]; sq = fmaf(df, df, sq); }
            sq = row16_sum(sq);
            dsum += row < hi ? sqrtf(sq) : 0.f;
        }
        dsum = rows4_sum(dsum);
        // g_j = exp(-D_j^2 / (2 sigma^2)); with sigma = dsum / (sqrt(2) m) that is exp(-(D_j m / dsum)^2)
        const float inv_mean = dsum > 0.f ? (float)m / dsum : 0.f;

        // sweep 2: weights, weighted sums
        float ak[8], av[8], gsum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { ak[e] = 0.f; av[e] = 0.f; }
        for (int j0 = lo; j0 < hi; j0 += 4) {
            const int row = j0 + slot;
            if (row < hi) {
                float x[8], v[8];
                if (j0 == lo) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = x0[e];
                } else {
                    Elem<T>::to_float(Elem<T>::load(Ks + (size_t)row * HEAD_DIM, c), x);
                }
                Elem<T>::to_float(Elem<T>::load(Vs + (size_t)row * HEAD_DIM, c), v);
                float sq = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) { const float df = kp[e] - x[e]; sq = fmaf(df, df, sq); }
                sq = row16_sum(sq);
                float g;
                if (a.sigma_fixed) {
                    g = __expf(-sq * a.inv_two_sigma_sq);
                } else {
                    const float r = sqrtf(sq) * inv_mean;
                    g = __expf(-r * r);
                }
                gsum += g;
#pragma unroll
                for (int e = 0; e < 8; ++e) { ak[e] = fmaf(g, x[e], ak[e]); av[e] = fmaf(g, v[e], av[e]); }
                if (wo && c == 0) wo[row] = g;
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
        if (slot == 0) Elem<T>::store(Ko + (size_t)(s_lo + i) * HEAD_DIM, c, Elem<T>::from_float(ak));
        if (slot == 1) Elem<T>::store(Vo + (size_t)(s_lo + i) * HEAD_DIM, c, Elem<T>::from_float(av));
        if (wo && c == 0) {                                            // each writer normalises its own g_j
            for (int row = lo + slot; row < hi; row += 4) wo[row] *= inv_g;
        }
        ++i;
    }
}

template <typename T>
static void launch_merge_t(const kvm_shape &sh, const void *K, const void *V, void *K_out, void *V_out,
                           const MergeArgs &a, hipStream_t st)
{
    const long long blocks = (long long)sh.B * sh.H_kv * a.blocks_per_slice;
    hipLaunchKernelGGL(merge_kernel<T>, dim3((unsigned)blocks), dim3(MERGE_BLOCK), 0, st, (const T *)K, (const T *)V,
                       (T *)K_out, (T *)V_out, a);
}

kvm_status launch_merge(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                        const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out,
                        void *V_out, float *w_opt, hipStream_t st)
{
    if ((long long)sh.B * sh.H_kv == 0 || cap_rows == 0 || sh.N == 0) return KVM_OK;
    MergeArgs a;
    a.set_start = set_start;
    a.pivot = pivot;
    a.n_sets = n_sets;
    a.seq_lens = sh.seq_lens;
    a.w_opt = w_opt;
    a.H = sh.H_kv;
    a.N = sh.N;
    a.cap_rows = cap_rows;
    a.blocks_per_slice = (cap_rows + MERGE_SETS_PER_BLOCK - 1) / MERGE_SETS_PER_BLOCK;
    a.sigma_fixed = pr.sigma_mode == KVM_SIGMA_FIXED;
    a.inv_two_sigma_sq = a.sigma_fixed ? 1.f / (2.f * pr.sigma * pr.sigma) : 0.f;
    a.value_scale = pr.value_scale_by_set_size;
    switch (sh.dtype) {
    case KVM_F32: launch_merge_t<float>(sh, K, V, K_out, V_out, a, st); break;
    case KVM_F16: launch_merge_t<half_t>(sh, K, V, K_out, V_out, a, st); break;
    default: launch_merge_t<bf16_t>(sh, K, V, K_out, V_out, a, st); break;
    }
    return check_launch("merge_kernel");
}

}  // namespace kvm
