// Decode-time update of the aggregated attention scores: the newest token's query attends to
// all keys of the cache (Section 2.4 Eq. (1) for one query row), and the row is added into
// the column sums (Section 4.2 Eq. (7): a sum over query rows, so one more row is one more
// term per key).
//
// One query row against N keys is a matrix-vector product: every key is read once and used
// for G dot products, so the update is bound by the HBM read of K (N d s bytes per slice) and
// the matrix cores have nothing to offer.  Two launches, because the softmax denominator
// spans the whole row:
//   append_scores_kernel      thread j of a workgroup owns key j of a 256-key tile; a row is
//                             spread over 16 lanes as in the other streaming kernels.  Scores
//                             (base-2 logarithm units) go to the workspace, with the maximum
//                             and the sum of exponentials of every wave's 64 keys beside them
//                             (no exchange between waves, so no barrier).
//   append_accumulate_kernel  merges the waves' statistics of a query head into its
//                             log-sum-exp and adds exp2(score - lse) of all G heads to mass.
#include "kvm_common.h"

namespace kvm {

constexpr int APP_BLOCK = 256;
constexpr int APP_ROWS_PER_GROUP = 16;                      // one row per lane of the group in the end
constexpr int APP_WAVES = APP_BLOCK / WAVE;
constexpr int ACC_PER_THREAD = 8;                           // keys per thread of the second kernel
constexpr int ACC_CHUNK = APP_BLOCK * ACC_PER_THREAD;

int attn_lse_stride(int N);

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, WAVE));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

template <typename T>
__global__ __launch_bounds__(APP_BLOCK) void append_scores_kernel(const T *__restrict__ q_new, const T *__restrict__ K,
                                                                   float *__restrict__ scores, float *__restrict__ stats,
                                                                   const int32_t *__restrict__ seq_lens, int H, int G,
                                                                   int N, int n_pad, int tiles_per_slice, float c)
{
    typedef typename Elem<T>::Raw Raw;
    const int slice = blockIdx.x / tiles_per_slice;          // (b, h)
    const int tile = blockIdx.x - slice * tiles_per_slice;
    const int b = slice / H;
    const int n = clamp_len(seq_lens, b, N);
    const int j_wave = tile * APP_BLOCK + (threadIdx.x & ~63);   // a wave's 64 keys share one pair of statistics
    if (j_wave >= n) return;                                 // the other kernel looks at keys below n only
    const int lane16 = threadIdx.x & 15, group = threadIdx.x >> 4;
    const int j0 = tile * APP_BLOCK + group * APP_ROWS_PER_GROUP;
    const T *Ks = K + (size_t)slice * N * HEAD_DIM;

    // all rows of the group at once; rows past the end repeat the last valid one and are masked below
    Raw raw[APP_ROWS_PER_GROUP];
#pragma unroll
    for (int i = 0; i < APP_ROWS_PER_GROUP; ++i) raw[i] = Elem<T>::load(Ks + (size_t)min(j0 + i, n - 1) * HEAD_DIM, lane16);

    const int j = tile * APP_BLOCK + threadIdx.x;            // the key whose score this thread keeps
    const int stats_per_row = n_pad / WAVE;
    for (int g = 0; g < G; ++g) {
        const size_t qslice = (size_t)slice * G + g;
        const Raw q = Elem<T>::load(q_new + qslice * HEAD_DIM, lane16);
        float mine = 0.f;
#pragma unroll
        for (int i = 0; i < APP_ROWS_PER_GROUP; ++i) {
            const float dot = row16_sum(RowDot<T>::dot(raw[i], q));
            if (lane16 == i) mine = dot;
        }
        const float x = j < n ? mine * c : -INFINITY;
        if (j < n) scores[qslice * n_pad + j] = x;
        const float m = wave_max(x);                         // finite: key j_wave is below n
        const float l = wave_sum(__builtin_amdgcn_exp2f(x - m));
        if ((threadIdx.x & 63) == 0) {
            float *st = stats + (qslice * stats_per_row + j_wave / WAVE) * 2;
            st[0] = m;
            st[1] = l;
        }
    }
}

__global__ __launch_bounds__(APP_BLOCK) void append_accumulate_kernel(const float *__restrict__ scores,
                                                                       const float *__restrict__ stats, float *__restrict__ mass,
                                                                       const int32_t *__restrict__ seq_lens, int H, int G, int N,
                                                                       int n_pad, int chunks_per_slice)
{
    __shared__ float slots[2 * APP_WAVES];
    const int slice = blockIdx.x / chunks_per_slice;
    const int chunk = blockIdx.x - slice * chunks_per_slice;
    const int n = clamp_len(seq_lens, slice / H, N);
    const int j_block = chunk * ACC_CHUNK;
    if (j_block >= n) return;
    const int valid_tiles = (n + WAVE - 1) / WAVE;           // statistics come per 64 keys
    const int stats_per_row = n_pad / WAVE;
    float add[ACC_PER_THREAD];
#pragma unroll
    for (int u = 0; u < ACC_PER_THREAD; ++u) add[u] = 0.f;
    for (int g = 0; g < G; ++g) {
        const size_t qslice = (size_t)slice * G + g;
        const float *st = stats + qslice * stats_per_row * 2;
        // log-sum-exp of the row from the waves' statistics: threads take them in turn, then the
        // workgroup reduces (two steps of the same rule: maximum first, sums scaled to it)
        float tm = -INFINITY;
        for (int t = threadIdx.x; t < valid_tiles; t += APP_BLOCK) tm = fmaxf(tm, st[2 * t]);
        const float wm = wave_max(tm);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) slots[threadIdx.x >> 6] = wm;
        __syncthreads();
        float m = slots[0];
#pragma unroll
        for (int i = 1; i < APP_WAVES; ++i) m = fmaxf(m, slots[i]);
        float tl = 0.f;
        for (int t = threadIdx.x; t < valid_tiles; t += APP_BLOCK) tl += st[2 * t + 1] * __builtin_amdgcn_exp2f(st[2 * t] - m);
        const float wl = wave_sum(tl);
        if ((threadIdx.x & 63) == 0) slots[APP_WAVES + (threadIdx.x >> 6)] = wl;
        __syncthreads();
        float l = 0.f;
#pragma unroll
        for (int i = 0; i < APP_WAVES; ++i) l += slots[APP_WAVES + i];
        const float lse = m + __log2f(l);
#pragma unroll
        for (int u = 0; u < ACC_PER_THREAD; ++u) {
            const int j = j_block + u * APP_BLOCK + threadIdx.x;
            if (j < n) add[u] += __builtin_amdgcn_exp2f(scores[qslice * n_pad + j] - lse);
        }
    }
#pragma unroll
    for (int u = 0; u < ACC_PER_THREAD; ++u) {
        const int j = j_block + u * APP_BLOCK + threadIdx.x;
        if (j < n) {
            float *a = mass + (size_t)slice * N + j;
            *a = j == n - 1 ? add[u] : *a + add[u];          // the newest token's entry starts here
        }
    }
}

template <typename T>
static kvm_status launch_t(const kvm_shape &sh, const void *q_new, const void *K, float *mass, float *ws, hipStream_t st)
{
    const int tiles = (sh.N + APP_BLOCK - 1) / APP_BLOCK;
    const int n_pad = attn_lse_stride(sh.N);
    const size_t n_q = (size_t)sh.B * sh.H_kv * sh.G;
    float *scores = ws, *stats = ws + n_q * n_pad;
    const float c = (float)(1.4426950408889634 / sqrt((double)sh.d));
    const long long blocks = (long long)sh.B * sh.H_kv * tiles;
    {
        ProfScope prof("append_scores_kernel", st);
        hipLaunchKernelGGL(append_scores_kernel<T>, dim3((unsigned)blocks), dim3(APP_BLOCK), 0, st, (const T *)q_new,
                           (const T *)K, scores, stats, sh.seq_lens, sh.H_kv, sh.G, sh.N, n_pad, tiles, c);
    }
    kvm_status rc = check_launch("append_scores_kernel");
    if (rc != KVM_OK) return rc;
    ProfScope prof("append_accumulate_kernel", st);
    const int chunks = (sh.N + ACC_CHUNK - 1) / ACC_CHUNK;
    hipLaunchKernelGGL(append_accumulate_kernel, dim3((unsigned)((long long)sh.B * sh.H_kv * chunks)), dim3(APP_BLOCK), 0, st,
                       (const float *)scores, (const float *)stats, mass, sh.seq_lens, sh.H_kv, sh.G, sh.N, n_pad, chunks);
    return check_launch("append_accumulate_kernel");
}

// ws: scores (B H_kv G, stride attn_lse_stride(N)) followed by two floats per (query slice, 64 keys).
kvm_status launch_attn_append(const kvm_shape &sh, const void *q_new, const void *K, float *mass, float *ws, hipStream_t st)
{
    if ((long long)sh.B * sh.H_kv == 0 || sh.N == 0) return KVM_OK;
    switch (sh.dtype) {
    case KVM_F32: return launch_t<float>(sh, q_new, K, mass, ws, st);
    case KVM_F16: return launch_t<half_t>(sh, q_new, K, mass, ws, st);
    default: return launch_t<bf16_t>(sh, q_new, K, mass, ws, st);
    }
}

}  // namespace kvm
