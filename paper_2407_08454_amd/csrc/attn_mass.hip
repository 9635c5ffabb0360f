// Aggregated attention score per key (Section 2.4 Eq. (1); Section 4.2 Eq. (7);
// Algorithm 2 step 2): mass[j] = sum over query heads g and rows t >= j of
// softmax_row_t(Q_g K^T / sqrt(d))[j], causal.
//
// The n x n map is never stored.  Two MFMA kernels recompute the scores:
//   attn_lse_kernel     row-stationary: a workgroup keeps its query rows in registers,
//                       streams K tiles through LDS and keeps an online (max, sum) per row;
//                       writes L_t = log2 sum_j exp2(c s_tj), c = log2(e)/sqrt(d).
//   attn_colsum_kernel  column-stationary: a workgroup keeps its keys in registers, streams
//                       Q tiles (and their L_t) through LDS and adds exp2(c s_tj - L_t) into
//                       per-lane column sums.  In the 32x32 MFMA result layout a lane's 16
//                       accumulators all belong to one column, so the column sum needs no
//                       cross-lane traffic until the very end and no atomics: deterministic.
// The operand that sits in registers is the MFMA B operand in both kernels; the streamed
// tile is the A operand, read from LDS with an XOR swizzle of its 16-byte chunks.
#include "kvm_common.h"

namespace kvm {

constexpr int ATT_BLOCK = 256;           // 4 waves
constexpr int ATT_WAVES = ATT_BLOCK / WAVE;

template <typename T> struct Mma;

template <> struct Mma<half_t> {
    static constexpr int CHUNKS = 16;    // 16-byte chunks per 128-element row
    static constexpr int FRAGS = 8;      // 16-byte fragments a lane holds per 32-row block
    static constexpr int NBLK = 2;       // 32-row blocks per streamed tile and per wave's stationary operand
    static __device__ __forceinline__ void mma(f32x16 &acc, const u32x4 &a, const u32x4 &b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
    }
};

template <> struct Mma<bf16_t> {
    static constexpr int CHUNKS = 16;
    static constexpr int FRAGS = 8;
    static constexpr int NBLK = 2;
    static __device__ __forceinline__ void mma(f32x16 &acc, const u32x4 &a, const u32x4 &b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
};

template <> struct Mma<float> {
    static constexpr int CHUNKS = 32;
    static constexpr int FRAGS = 16;
    static constexpr int NBLK = 1;
    static __device__ __forceinline__ void mma(f32x16 &acc, const u32x4 &a, const u32x4 &b) {
        // (the elements are copied out first: a bit cast applied directly to a vector
        // element lvalue reads element 0 with this compiler)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t ai = a[i], bi = b[i];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, ai), __builtin_bit_cast(float, bi), acc, 0, 0, 0);
        }
    }
};

// In a 32x32 MFMA result, accumulator i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32.
__device__ __forceinline__ int acc_row(int i, int lane) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

// A streamed tile in LDS: TR rows of CHUNKS 16-byte chunks; chunk ch of row r sits at
// position ch ^ (r mod CHUNKS), so that 16 lanes reading one chunk column of 16
// consecutive rows hit 16 different bank groups.
template <typename T> struct Tile {
    static constexpr int CH = Mma<T>::CHUNKS;
    static constexpr int TR = 32 * Mma<T>::NBLK;
    static constexpr int PER_THREAD = TR * CH / ATT_BLOCK;
    static __device__ __forceinline__ int lds_index(int row, int ch) { return row * CH + (ch ^ (row & (CH - 1))); }

    // rows [row0, row0+TR) of a (N x 128) matrix; rows >= n_valid read as zero
    static __device__ __forceinline__ void load(const T *base, int row0, int n_valid, u32x4 *regs) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int id = threadIdx.x + ATT_BLOCK * i;
            const int row = id / CH, ch = id % CH;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (row0 + row < n_valid)
                v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(base + (size_t)(row0 + row) * HEAD_DIM) + ch * 16);
            regs[i] = v;
        }
    }
    static __device__ __forceinline__ void store(u32x4 *lds, const u32x4 *regs) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int id = threadIdx.x + ATT_BLOCK * i;
            lds[lds_index(id / CH, id % CH)] = regs[i];
        }
    }
    // fragment f of 32-row block blk for this lane (MFMA A operand)
    static __device__ __forceinline__ u32x4 frag(const u32x4 *lds, int blk, int f, int lane) {
        return lds[lds_index(32 * blk + (lane & 31), 2 * f + (lane >> 5))];
    }
};

// The stationary operand: rows [row0, row0+32) straight from global memory into registers.
template <typename T>
__device__ __forceinline__ void load_stationary(const T *base, int row0, int n_valid, int lane, u32x4 *frags) {
    const int row = row0 + (lane & 31);
#pragma unroll
    for (int f = 0; f < Mma<T>::FRAGS; ++f) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (row < n_valid)
            v = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(base + (size_t)row * HEAD_DIM) + (2 * f + (lane >> 5)) * 16);
        frags[f] = v;
    }
}

// blockIdx -> (slice, tile).  Workgroups are dealt round-robin to the 8 XCDs, each with its
// own L2: all tiles of a slice go to one XCD so that the slice's K and Q are fetched once.
// Within a slice the tiles with the most causal work come first.
struct TileMap {
    int slice, tile;
    bool valid;
};
__device__ __forceinline__ TileMap map_block(int n_slices, int tiles_per_slice) {
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    TileMap m;
    m.slice = (idx / tiles_per_slice) * 8 + xcd;
    m.tile = idx % tiles_per_slice;
    m.valid = m.slice < n_slices;
    return m;
}

// ------------------------------------------------------------------------------------------
// pass 1: row log-sum-exp
// ------------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(ATT_BLOCK, 2) void attn_lse_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                 float *__restrict__ lse, const int32_t *__restrict__ seq_lens,
                                                                 int n_qslices, int HG, int G, int N, int tiles_per_slice,
                                                                 float c)
{
    using M = Mma<T>;
    using TL = Tile<T>;
    constexpr int NB = M::NBLK, TR = TL::TR;
    constexpr int ROWS_PER_BLOCK = ATT_WAVES * 32 * NB;       // query rows of a workgroup
    __shared__ u32x4 lds[2][TR * M::CHUNKS];

    const TileMap tm = map_block(n_qslices, tiles_per_slice);
    if (!tm.valid) return;
    const int qslice = tm.slice;                              // (b, h*G + g)
    const int tile = tiles_per_slice - 1 - tm.tile;          // longest rows first
    const int b = qslice / HG;
    const int kvslice = b * (HG / G) + (qslice % HG) / G;
    const int n = clamp_len(seq_lens, b, N);
    const int q_begin = tile * ROWS_PER_BLOCK;
    if (q_begin >= n) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const T *Qs = Q + (size_t)qslice * N * HEAD_DIM;
    const T *Ks = K + (size_t)kvslice * N * HEAD_DIM;
    const int q0 = q_begin + wave * 32 * NB;                  // first query row of this wave

    u32x4 qf[NB][M::FRAGS];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) load_stationary<T>(Qs, q0 + 32 * qb, n, lane, qf[qb]);

    float m_run[NB], l_run[NB];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

    const int q_last = min(q_begin + ROWS_PER_BLOCK, n) - 1; // last valid query row of the workgroup
    const int steps = q_last / TR + 1;                        // key tiles 0 .. steps-1
    u32x4 pre[TL::PER_THREAD];
    TL::load(Ks, 0, n, pre);
    TL::store(lds[0], pre);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        if (s + 1 < steps) TL::load(Ks, (s + 1) * TR, n, pre);
#pragma unroll
        for (int kb = 0; kb < NB; ++kb) {
            const int key0 = s * TR + 32 * kb;
#pragma unroll
            for (int qb = 0; qb < NB; ++qb) {
                const int qrow0 = q0 + 32 * qb;
                if (key0 > qrow0 + 31) continue;             // every key of the block is in the future
                f32x16 acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                for (int f = 0; f < M::FRAGS; ++f) M::mma(acc, TL::frag(lds[buf], kb, f, lane), qf[qb][f]);
                // acc[i]: key = key0 + acc_row(i), query = qrow0 + lane%32
                if (key0 + 31 > qrow0) {
                    const int q = qrow0 + (lane & 31);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (key0 + acc_row(i, lane) > q) acc[i] = -INFINITY;
                }
                float tmax = acc[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, acc[i]);
                const float m_new = fmaxf(m_run[qb], tmax);
                if (m_new > -INFINITY) {
                    const float mc = m_new * c;
                    float sum = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(acc[i], c, -mc));
                    l_run[qb] = l_run[qb] * __builtin_amdgcn_exp2f(m_run[qb] * c - mc) + sum;
                    m_run[qb] = m_new;
                }
            }
        }
        if (s + 1 < steps) TL::store(lds[buf ^ 1], pre);
        __syncthreads();
    }
    // lanes l and l+32 hold the two halves of a row's keys
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) {
        const float m_o = __shfl_xor(m_run[qb], 32, WAVE), l_o = __shfl_xor(l_run[qb], 32, WAVE);
        const float m = fmaxf(m_run[qb], m_o);
        float l = 0.f;
        if (m_run[qb] > -INFINITY) l += l_run[qb] * __builtin_amdgcn_exp2f((m_run[qb] - m) * c);
        if (m_o > -INFINITY) l += l_o * __builtin_amdgcn_exp2f((m_o - m) * c);
        const int q = q0 + 32 * qb + (lane & 31);
        if (lane < 32 && q < n) lse[(size_t)qslice * N + q] = m * c + __log2f(l);
    }
}

// ------------------------------------------------------------------------------------------
// pass 2: column sums
// ------------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(ATT_BLOCK, 2) void attn_colsum_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                    const float *__restrict__ lse, float *__restrict__ mass,
                                                                    const int32_t *__restrict__ seq_lens, int n_kvslices,
                                                                    int H, int G, int N, int tiles_per_slice, float c)
{
    using M = Mma<T>;
    using TL = Tile<T>;
    constexpr int NB = M::NBLK, TR = TL::TR;
    constexpr int KEYS_PER_BLOCK = ATT_WAVES * 32 * NB;
    __shared__ u32x4 lds[2][TR * M::CHUNKS];
    __shared__ __attribute__((aligned(16))) float lds_lse[2][TR];

    const TileMap tm = map_block(n_kvslices, tiles_per_slice);
    if (!tm.valid) return;
    const int kvslice = tm.slice, tile = tm.tile;             // tile 0 has the most rows below it
    const int b = kvslice / H, h = kvslice % H;
    const int n = clamp_len(seq_lens, b, N);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k_begin = tile * KEYS_PER_BLOCK;
    const int k0 = k_begin + wave * 32 * NB;
    float *mass_s = mass + (size_t)kvslice * N;
    if (k_begin >= n) {                                       // padding only: defined zeros
        for (int j = k_begin + threadIdx.x; j < min(k_begin + KEYS_PER_BLOCK, N); j += ATT_BLOCK) mass_s[j] = 0.f;
        return;
    }
    const T *Ks = K + (size_t)kvslice * N * HEAD_DIM;

    u32x4 kf[NB][M::FRAGS];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) load_stationary<T>(Ks, k0 + 32 * kb, n, lane, kf[kb]);

    float colsum[NB];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) colsum[kb] = 0.f;

    const int first = k_begin / TR;                           // first query tile that sees these keys
    const int last = (n - 1) / TR;
    const int steps_per_head = last - first + 1;
    const int steps = steps_per_head * G;
    u32x4 pre[TL::PER_THREAD];
    float pre_lse = 0.f;

    auto prefetch = [&](int s) {
        const int g = s / steps_per_head, qt = first + s % steps_per_head;
        const size_t qslice = (size_t)b * H * G + (size_t)h * G + g;
        TL::load(Q + qslice * N * HEAD_DIM, qt * TR, n, pre);
        if (threadIdx.x < TR) {
            const int t = qt * TR + threadIdx.x;
            pre_lse = t < n ? lse[qslice * N + t] : INFINITY; // exp2(-inf) = 0: padded rows add nothing
        }
    };
    auto commit = [&](int buf) {
        TL::store(lds[buf], pre);
        if (threadIdx.x < TR) lds_lse[buf][threadIdx.x] = pre_lse;
    };

    prefetch(0);
    commit(0);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        const int qt = first + s % steps_per_head;
        if (s + 1 < steps) prefetch(s + 1);
#pragma unroll
        for (int qb = 0; qb < NB; ++qb) {
            const int qrow0 = qt * TR + 32 * qb;
            float L[16];
            bool have_L = false;
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) {
                const int key0 = k0 + 32 * kb;
                if (qrow0 + 31 < key0) continue;             // every query of the block precedes the keys
                if (!have_L) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const f32x4 v = *reinterpret_cast<const f32x4 *>(&lds_lse[buf][32 * qb + 8 * r + 4 * (lane >> 5)]);
#pragma unroll
                        for (int e = 0; e < 4; ++e) L[4 * r + e] = v[e];
                    }
                    have_L = true;
                }
                f32x16 acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                for (int f = 0; f < M::FRAGS; ++f) M::mma(acc, TL::frag(lds[buf], qb, f, lane), kf[kb][f]);
                // acc[i]: query = qrow0 + acc_row(i), key = key0 + lane%32
                float part[4] = {0.f, 0.f, 0.f, 0.f};
                if (qrow0 < key0 + 31) {                      // block touches the diagonal
                    const int key = key0 + (lane & 31);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(acc[i], c, -L[i]));
                        part[i & 3] += (qrow0 + acc_row(i, lane) >= key) ? p : 0.f;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) part[i & 3] += __builtin_amdgcn_exp2f(fmaf(acc[i], c, -L[i]));
                }
                colsum[kb] += (part[0] + part[1]) + (part[2] + part[3]);
            }
        }
        if (s + 1 < steps) commit(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
        const float total = colsum[kb] + __shfl_xor(colsum[kb], 32, WAVE);
        const int key = k0 + 32 * kb + (lane & 31);
        if (lane < 32 && key < N) mass_s[key] = key < n ? total : 0.f;
    }
}

// ------------------------------------------------------------------------------------------
// host launcher
// ------------------------------------------------------------------------------------------

template <typename T>
static kvm_status launch_t(const kvm_shape &sh, const void *Q, const void *K, float *mass, float *lse, hipStream_t st)
{
    constexpr int ROWS = ATT_WAVES * 32 * Mma<T>::NBLK;
    const int tiles = (sh.N + ROWS - 1) / ROWS;
    const float c = (float)(1.4426950408889634 / sqrt((double)sh.d));
    const int n_q = sh.B * sh.H_kv * sh.G, n_kv = sh.B * sh.H_kv;
    {
        const long long blocks = (long long)((n_q + 7) / 8) * 8 * tiles;
        ProfScope prof("attn_lse_kernel", st);
        hipLaunchKernelGGL(attn_lse_kernel<T>, dim3((unsigned)blocks), dim3(ATT_BLOCK), 0, st, (const T *)Q, (const T *)K,
                           lse, sh.seq_lens, n_q, sh.H_kv * sh.G, sh.G, sh.N, tiles, c);
        kvm_status rc = check_launch("attn_lse_kernel");
        if (rc != KVM_OK) return rc;
    }
    {
        const long long blocks = (long long)((n_kv + 7) / 8) * 8 * tiles;
        ProfScope prof("attn_colsum_kernel", st);
        hipLaunchKernelGGL(attn_colsum_kernel<T>, dim3((unsigned)blocks), dim3(ATT_BLOCK), 0, st, (const T *)Q,
                           (const T *)K, (const float *)lse, mass, sh.seq_lens, n_kv, sh.H_kv, sh.G, sh.N, tiles, c);
        return check_launch("attn_colsum_kernel");
    }
}

kvm_status launch_attn_mass(const kvm_shape &sh, const void *Q, const void *K, float *mass, float *lse, hipStream_t st)
{
    if ((long long)sh.B * sh.H_kv == 0 || sh.N == 0) return KVM_OK;
    switch (sh.dtype) {
    case KVM_F32: return launch_t<float>(sh, Q, K, mass, lse, st);
    case KVM_F16: return launch_t<half_t>(sh, Q, K, mass, lse, st);
    default: return launch_t<bf16_t>(sh, Q, K, mass, lse, st);
    }
}

}  // namespace kvm
