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
// tile is the A operand.  Tiles go from global memory straight into one of two LDS stages
// (global_load_lds, no registers in between), one tile ahead of the one being used, with an
// XOR swizzle of their 16-byte chunks so that the fragment reads are conflict-free.
//
// On this chip the pair (one MFMA block, its softmax arithmetic) is bound by VALU issue slots
// and by power, not by the matrix pipe: at d = 128 a 32x32 block costs 8 MFMAs (256 cycles) and
// at least 48 VALU instructions (one fma, one exp2, one add per score), and packed fp32
// arithmetic is not used.  Hence the attention to every VALU instruction in the block loops.
#include "attn_tile.h"

namespace kvm {

// ------------------------------------------------------------------------------------------
// per-block reductions
//
// A wave issues at most one instruction every other issue slot of its SIMD, so the vector
// ALU and the matrix pipe only stay busy with several waves per SIMD.  The kernels are
// written to fit three waves per SIMD (168 registers, 64 of them for the stationary operand):
// one accumulator block at a time, the eight fragments of a block fetched together, and the
// overlap of MFMA, exp2 and LDS traffic is left to the hardware interleaving the waves.
// ------------------------------------------------------------------------------------------

// pass 1: the online (max, sum) of a row absorbs 16 more scores (-inf = masked)
__device__ __forceinline__ void rowstat_update(const f32x16 &acc, float c, float &m_run, float &l_run) {
    const float m_new = fmaxf(m_run, max16(acc));
    const float mc = m_new * c;
    float p0 = 0.f, p1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        p0 += __builtin_amdgcn_exp2f(fmaf(acc[i], c, -mc));
        p1 += __builtin_amdgcn_exp2f(fmaf(acc[i + 1], c, -mc));
    }
    // (the difference is taken before the scaling: M_INIT * c - round(M_INIT * c), fused, would be
    // the rounding error of a huge product instead of zero)
    l_run = l_run * __builtin_amdgcn_exp2f((m_run - m_new) * c) + (p0 + p1);
    m_run = m_new;
}

// pass 1 with the reference held: 16 more terms exp2(c s - mc) of a row's sum, no maximum and
// no rescaling.  Any reference gives the same log-sum-exp as long as no term overflows; the
// caller checks the finished sums for that.
__device__ __forceinline__ void rowsum_held(const f32x16 &acc, float c, float mc, float &l_run) {
    float p0 = __builtin_amdgcn_exp2f(fmaf(acc[0], c, -mc)), p1 = __builtin_amdgcn_exp2f(fmaf(acc[1], c, -mc));
#pragma unroll
    for (int i = 2; i < 16; i += 2) {
        p0 += __builtin_amdgcn_exp2f(fmaf(acc[i], c, -mc));
        p1 += __builtin_amdgcn_exp2f(fmaf(acc[i + 1], c, -mc));
    }
    l_run += p0 + p1;
}

// pass 2: the row statistics L of a 32-row block of the streamed tile, in the order of a
// lane's accumulators (accumulator i of lane l is row 8*(i/4) + 4*(l/32) + i%4)
struct RowStats { f32x4 v[4]; };
__device__ __forceinline__ RowStats load_rowstats(const float *lse_tile, int blk, int lane) {
    RowStats L;
#pragma unroll
    for (int r = 0; r < 4; ++r) L.v[r] = *reinterpret_cast<const f32x4 *>(&lse_tile[32 * blk + 8 * r + 4 * (lane >> 5)]);
    return L;
}
// part[0..1] += exp2(c * acc - L)
__device__ __forceinline__ void colsum_update(const f32x16 &acc, const RowStats &L, float c, float *part) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        part[0] += __builtin_amdgcn_exp2f(fmaf(acc[4 * r], c, -L.v[r][0]));
        part[1] += __builtin_amdgcn_exp2f(fmaf(acc[4 * r + 1], c, -L.v[r][1]));
        part[0] += __builtin_amdgcn_exp2f(fmaf(acc[4 * r + 2], c, -L.v[r][2]));
        part[1] += __builtin_amdgcn_exp2f(fmaf(acc[4 * r + 3], c, -L.v[r][3]));
    }
}

constexpr int FRAG_BATCH = 2;            // A fragments fetched from LDS per batch of MFMAs (generic path)

// one 32x32 block of scores: A fragments from the LDS tile, B fragments from registers
template <typename T>
__device__ __forceinline__ f32x16 score_block(const u32x4 *tile, int blk, const u32x4 *bfrag, int lane) {
    using M = Mma<T>;
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int f0 = 0; f0 < M::FRAGS; f0 += FRAG_BATCH) {
        u32x4 a[FRAG_BATCH];
#pragma unroll
        for (int f = 0; f < FRAG_BATCH; ++f) a[f] = Tile<T>::frag(tile, blk, f0 + f, lane);
#pragma unroll
        for (int f = 0; f < FRAG_BATCH; ++f) M::mma(acc, a[f], bfrag[f0 + f]);
    }
    return acc;
}

template <typename T>
__device__ __forceinline__ f32x16 score_block8(const u32x4 *a, const u32x4 *bfrag) {
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int f = 0; f < 8; ++f) Mma<T>::mma(acc, a[f], bfrag[f]);
    return acc;
}

// ------------------------------------------------------------------------------------------
// pass 1: row log-sum-exp
// ------------------------------------------------------------------------------------------

// HOLD (16-bit types only): the running maximum is taken from key tile 0 and held for the tiles
// below the diagonal, which saves the maximum and the rescaling of every block; the diagonal
// tile updates it again.  Should a later score exceed the held maximum by so much that a term
// overflows, the sums are not finite: the workgroup then records the row tile in `redo`, and a
// second launch without HOLD, which looks only at recorded tiles, computes it with the maximum
// updated at every block.  Without HOLD and with redo == NULL every tile is computed.
template <typename T, bool HOLD>
__global__ __launch_bounds__(ATT_BLOCK, ATT_MIN_BLOCKS) void attn_lse_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                 float *__restrict__ lse, int32_t *__restrict__ redo,
                                                                 const int32_t *__restrict__ seq_lens,
                                                                 int n_qslices, int HG, int G, int N, int n_pad,
                                                                 int tiles_per_slice, int wgs_per_slice, float c,
                                                                 float out_scale, float pad)
{
    using M = Mma<T>;
    using TL = Tile<T>;
    constexpr int NB = M::NBLK, TR = TL::TR;
    constexpr int ROWS_PER_BLOCK = ATT_WAVES * 32 * NB;       // query rows of a workgroup
    // one LDS object per stage: the compiler then knows that the fragment reads of a step do
    // not touch the stage the next tile is being loaded into, and does not wait for that load
    __shared__ u32x4 lds_a[TL::SLOTS], lds_b[TL::SLOTS];

    const TileMap tm = map_block(n_qslices, wgs_per_slice);
    if (!tm.valid) return;
    const int qslice = tm.slice;                              // (b, h*G + g)
    const int b = qslice / HG;
    const int kvslice = b * (HG / G) + (qslice % HG) / G;
    const int n = clamp_len(seq_lens, b, N);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // scalar: per-wave branches stay scalar
    const T *Qs = Q + (size_t)qslice * N * HEAD_DIM;
    const T *Ks = K + (size_t)kvslice * N * HEAD_DIM;
    const typename TL::Offsets off = TL::offsets(wave, lane);
    const FragSlots fs = frag_slots<T>(lane);

    // Workgroup t of a slice takes row tile tiles-1-t, the one with the longest rows left; with
    // fewer workgroups than tiles it then also takes tile t, the shortest left, so that all
    // workgroups of a launch carry the same load.
    // The repeat launch (redo given, no HOLD) has one workgroup per slice, which looks at all
    // of the slice's flags.
    const bool paired = wgs_per_slice < tiles_per_slice;
    const bool repeat = !HOLD && redo;
    const int passes = repeat ? tiles_per_slice : 2;
    for (int pass = 0; pass < passes; ++pass) {
    const int tile = repeat ? pass : (pass == 0 ? tiles_per_slice - 1 - tm.tile : tm.tile);
    if (!repeat && pass == 1 && (!paired || tm.tile >= tiles_per_slice - 1 - tm.tile)) break;
    const int q_begin = tile * ROWS_PER_BLOCK;
    if (q_begin >= n) continue;
    if (repeat && !redo[(size_t)qslice * tiles_per_slice + tile]) continue;
    const int q0 = q_begin + wave * 32 * NB;                  // first query row of this wave

    const int q_last = min(q_begin + ROWS_PER_BLOCK, n) - 1; // last valid query row of the workgroup
    const int steps = q_last / TR + 1;                        // key tiles 0 .. steps-1
    auto issue = [&](int t, u32x4 *stage) {                   // key tile t on its way into LDS
        TL::issue(Ks, t * TR, n, off, stage, wave, lane);
    };

    u32x4 qf[NB][M::FRAGS];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) load_stationary<T>(Qs, q0 + 32 * qb, n, lane, qf[qb]);

    float m_run[NB], l_run[NB];
    issue(0, lds_a);
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) { m_run[qb] = M_INIT; l_run[qb] = 0.f; }

    // (16-bit types: TR = 64 = the rows of a wave) key tiles before `diag` lie entirely below
    // this wave's diagonal, tile `diag` holds it, later tiles are in this wave's future; a wave
    // without valid rows computes nothing
    const int diag = q0 < n ? q0 / TR : -1;

    auto step = [&](int s, const u32x4 *cur, u32x4 *nxt) {
        // this thread's part of tile s has landed; after the barrier everybody's part has, and
        // everybody is done with the stage that tile s+1 now overwrites
        wait_vmcnt<0>();
        barrier_no_fence();
        if (s + 1 < steps) issue(s + 1, nxt);
        if constexpr (NB == 2) {
            // the fences keep the scheduler from hoisting later blocks' LDS reads, which would
            // not fit the register budget
            if (HOLD && s < diag && s > 0) {                  // four full blocks, maximum held
                const float mc0 = m_run[0] * c, mc1 = m_run[1] * c;
                u32x4 a[8];
                load_frags8<T>(cur, 0, fs, a);
                f32x16 acc = score_block8<T>(a, qf[0]);
                rowsum_held(acc, c, mc0, l_run[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[1]);
                load_frags8<T>(cur, 1, fs, a);              // in flight during the reduction below
                rowsum_held(acc, c, mc1, l_run[1]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[0]);
                rowsum_held(acc, c, mc0, l_run[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[1]);
                rowsum_held(acc, c, mc1, l_run[1]);
            } else if (s < diag) {                            // four full blocks
                u32x4 a[8];
                load_frags8<T>(cur, 0, fs, a);
                f32x16 acc = score_block8<T>(a, qf[0]);
                rowstat_update(acc, c, m_run[0], l_run[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[1]);
                load_frags8<T>(cur, 1, fs, a);              // in flight during the reduction below
                rowstat_update(acc, c, m_run[1], l_run[1]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[0]);
                rowstat_update(acc, c, m_run[0], l_run[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[1]);
                rowstat_update(acc, c, m_run[1], l_run[1]);
            } else if (s == diag) {                           // two blocks on the diagonal, one below it
                u32x4 a[8];
                load_frags8<T>(cur, 0, fs, a);              // keys q0 .. q0+31
                f32x16 acc = score_block8<T>(a, qf[0]);
                mask_rows_above_col(acc, lane);               // accumulator rows are keys, columns queries
                rowstat_update(acc, c, m_run[0], l_run[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[1]);
                load_frags8<T>(cur, 1, fs, a);              // keys q0+32 .. q0+63
                rowstat_update(acc, c, m_run[1], l_run[1]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, qf[1]);
                mask_rows_above_col(acc, lane);
                rowstat_update(acc, c, m_run[1], l_run[1]);
            }
        } else {
            if (diag < 0) return;
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) {
                const int key0 = s * TR + 32 * kb;
#pragma unroll
                for (int qb = 0; qb < NB; ++qb) {
                    const int qrow0 = q0 + 32 * qb;
                    if (key0 > qrow0 + 31) continue;         // every key of the block is in the future
                    f32x16 acc = score_block<T>(cur, kb, qf[qb], lane);
                    // acc[i]: key = key0 + acc_row(i), query = qrow0 + lane%32
                    if (key0 + 31 > qrow0) {
                        const int q = qrow0 + (lane & 31);
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            if (key0 + acc_row(i, lane) > q) acc[i] = -INFINITY;
                    }
                    rowstat_update(acc, c, m_run[qb], l_run[qb]);
                }
            }
        }
    };
    for (int s = 0; s < steps; s += 2) {
        step(s, lds_a, lds_b);
        if (s + 1 < steps) step(s + 1, lds_b, lds_a);
    }
    wait_vmcnt<0>();                                          // no load may still target this workgroup's LDS
    // lanes l and l+32 hold the two halves of a row's keys.  The statistic is stored as
    // out_scale * L_t; rows in [n, n_pad) get `pad`, the infinity whose sign makes the second pass
    // weigh them with exp2(-inf) = 0.
    bool finite = true;
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) {
        const float m_o = __shfl_xor(m_run[qb], 32, WAVE), l_o = __shfl_xor(l_run[qb], 32, WAVE);
        const float m = fmaxf(m_run[qb], m_o);
        const float l = l_run[qb] * __builtin_amdgcn_exp2f((m_run[qb] - m) * c) + l_o * __builtin_amdgcn_exp2f((m_o - m) * c);
        const float L = m * c + __log2f(l);
        const int q = q0 + 32 * qb + (lane & 31);
        // (checked on the combined sum: two finite halves can still add up to infinity)
        if (q < n) finite = finite && fabsf(L) <= 3.0e38f;    // false for infinities and NaN
        if (lane < 32 && q < n_pad) lse[(size_t)qslice * n_pad + q] = q < n ? L * out_scale : pad;
    }
    if constexpr (HOLD) {
        const int bad = __syncthreads_or(finite ? 0 : 1);
        if (threadIdx.x == 0) redo[(size_t)qslice * tiles_per_slice + tile] = bad;
    }
    barrier_no_fence();                                       // everybody is done with LDS before the next tile's loads
    }
}

// ------------------------------------------------------------------------------------------
// pass 2: column sums
// ------------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(ATT_BLOCK, ATT_MIN_BLOCKS) void attn_colsum_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                    const float *__restrict__ lse, float *__restrict__ mass,
                                                                    float *__restrict__ sim_opt,
                                                                    const int32_t *__restrict__ seq_lens, int n_kvslices,
                                                                    int H, int G, int N, int n_pad, int tiles_per_slice,
                                                                    int wgs_per_slice, float c)
{
    using M = Mma<T>;
    using TL = Tile<T>;
    constexpr int NB = M::NBLK, TR = TL::TR;
    constexpr int KEYS_PER_BLOCK = ATT_WAVES * 32 * NB;
    // one LDS object per stage (see attn_lse_kernel)
    __shared__ u32x4 lds_a[TL::SLOTS], lds_b[TL::SLOTS];
    __shared__ __attribute__((aligned(16))) float lse_a[64], lse_b[64];

    const TileMap tm = map_block(n_kvslices, wgs_per_slice);
    if (!tm.valid) return;
    const int kvslice = tm.slice;
    const int b = kvslice / H, h = kvslice % H;
    const int n = clamp_len(seq_lens, b, N);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // scalar: per-wave branches stay scalar
    float *mass_s = mass + (size_t)kvslice * N;
    float *sim_s = sim_opt ? sim_opt + (size_t)kvslice * N : nullptr;
    const T *Ks = K + (size_t)kvslice * N * HEAD_DIM;
    const typename TL::Offsets off = TL::offsets(wave, lane);
    const FragSlots fs = frag_slots<T>(lane);
    // workgroup t takes key tile t (tile 0 has the most rows below it) and, when there are fewer
    // workgroups than tiles, then also tile tiles-1-t (see attn_lse_kernel)
    const bool paired = wgs_per_slice < tiles_per_slice;
    for (int pass = 0; pass < 2; ++pass) {
    const int tile = pass == 0 ? tm.tile : tiles_per_slice - 1 - tm.tile;
    if (pass == 1 && (!paired || tm.tile >= tiles_per_slice - 1 - tm.tile)) break;
    const int k_begin = tile * KEYS_PER_BLOCK;
    const int k0 = k_begin + wave * 32 * NB;
    if (k_begin >= n) {                                       // padding only: defined zeros
        for (int j = k_begin + threadIdx.x; j < min(k_begin + KEYS_PER_BLOCK, N); j += ATT_BLOCK) {
            mass_s[j] = 0.f;
            if (sim_s) sim_s[j] = 0.f;
        }
        continue;
    }

    // Query tiles first .. last see these keys.  They are streamed from the last one down, head
    // after head: every workgroup of a slice then starts at the same tile and walks down in step
    // with the others, so that a tile is fetched from memory once for all of them.
    const int first = k_begin / TR;
    const int last = (n - 1) / TR;
    const int steps = (last - first + 1) * G;
    auto issue = [&](int g, int qt, u32x4 *stage, float *stage_lse) {   // Q rows and their statistics -> LDS
        const size_t qslice = ((size_t)b * H + h) * G + g;
        const T *Qh = Q + qslice * N * HEAD_DIM;
        const int row0 = qt * TR;
        TL::issue(Qh, row0, n, off, stage, wave, lane);
        if (lane < TR)
            __builtin_amdgcn_global_load_lds((gptr_t)(lse + qslice * n_pad + row0 + lane), (lptr_t)stage_lse, 4, 0, 0);
    };
    int g_next = 0, qt_next = last;                           // the tile that is loaded next
    auto issue_next = [&](u32x4 *stage, float *stage_lse) {
        issue(g_next, qt_next, stage, stage_lse);
        if (qt_next == first) { qt_next = last; ++g_next; } else --qt_next;
    };
    issue_next(lds_a, lse_a);
    u32x4 kf[NB][M::FRAGS];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) load_stationary<T>(Ks, k0 + 32 * kb, n, lane, kf[kb]);
    if constexpr (sizeof(T) == 2) {
        if (sim_s) {                                          // the keys are here anyway: their adjacent similarities
            u32x4 before[NB];
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) before[kb] = load_predecessor<T>(Ks, k0 + 32 * kb, n, lane);
#pragma unroll
            for (int kb = 0; kb < NB; ++kb) stationary_cosine<T>(k0 + 32 * kb, n, N, lane, kf[kb], before[kb], sim_s);
        }
    }

    float part[NB][2];
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) part[kb][0] = part[kb][1] = 0.f;

    // (16-bit types: TR = 64 = the keys of a wave) query tiles after `diag` lie entirely below
    // this wave's diagonal, tile `diag` holds it, earlier tiles precede all of the wave's keys;
    // a wave without valid keys computes nothing
    const int diag = k0 < n ? k0 / TR : last + 1;
    int qt = last + 1;                                        // tile of the current step
    auto step = [&](int s, const u32x4 *cur, const float *cur_lse, u32x4 *nxt, float *nxt_lse) {
        qt = qt == first ? last : qt - 1;
        wait_vmcnt<0>();
        barrier_no_fence();
        if (s + 1 < steps) issue_next(nxt, nxt_lse);
        if constexpr (NB == 2) {
            // the fences keep the scheduler from hoisting later blocks' LDS reads, which would
            // not fit the register budget
            if (qt > diag) {                                  // four full blocks
                u32x4 a[8];
                load_frags8<T>(cur, 0, fs, a);
                RowStats L = load_rowstats(cur_lse, 0, lane);
                f32x16 acc = score_block8<T>(a, kf[0]);
                colsum_update(acc, L, c, part[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, kf[1]);
                load_frags8<T>(cur, 1, fs, a);              // in flight during the reduction below
                colsum_update(acc, L, c, part[1]);
                __builtin_amdgcn_sched_barrier(0);
                L = load_rowstats(cur_lse, 1, lane);
                acc = score_block8<T>(a, kf[0]);
                colsum_update(acc, L, c, part[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, kf[1]);
                colsum_update(acc, L, c, part[1]);
            } else if (qt == diag) {                          // two blocks on the diagonal, one below it
                u32x4 a[8];
                load_frags8<T>(cur, 0, fs, a);              // queries k0 .. k0+31
                RowStats L = load_rowstats(cur_lse, 0, lane);
                f32x16 acc = score_block8<T>(a, kf[0]);
                load_frags8<T>(cur, 1, fs, a);              // queries k0+32 .. k0+63
                mask_rows_below_col(acc, lane);               // accumulator rows are queries, columns keys
                colsum_update(acc, L, c, part[0]);
                __builtin_amdgcn_sched_barrier(0);
                L = load_rowstats(cur_lse, 1, lane);
                acc = score_block8<T>(a, kf[0]);
                colsum_update(acc, L, c, part[0]);
                __builtin_amdgcn_sched_barrier(0);
                acc = score_block8<T>(a, kf[1]);
                mask_rows_below_col(acc, lane);
                colsum_update(acc, L, c, part[1]);
            }
        } else {
            if (k0 >= n) return;
#pragma unroll
            for (int qb = 0; qb < NB; ++qb) {
                const int qrow0 = qt * TR + 32 * qb;
                const RowStats L = load_rowstats(cur_lse, qb, lane);
#pragma unroll
                for (int kb = 0; kb < NB; ++kb) {
                    const int key0 = k0 + 32 * kb;
                    if (qrow0 + 31 < key0) continue;         // every query of the block precedes the keys
                    f32x16 acc = score_block<T>(cur, qb, kf[kb], lane);
                    // acc[i]: query = qrow0 + acc_row(i), key = key0 + lane%32
                    if (qrow0 < key0 + 31) {                  // block touches the diagonal
                        const int key = key0 + (lane & 31);
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            if (qrow0 + acc_row(i, lane) < key) acc[i] = -INFINITY;
                    }
                    colsum_update(acc, L, c, part[kb]);
                }
            }
        }
    };
    for (int s = 0; s < steps; s += 2) {
        step(s, lds_a, lse_a, lds_b, lse_b);
        if (s + 1 < steps) step(s + 1, lds_b, lse_b, lds_a, lse_a);
    }
    wait_vmcnt<0>();                                          // no load may still target this workgroup's LDS
#pragma unroll
    for (int kb = 0; kb < NB; ++kb) {
        const float colsum = part[kb][0] + part[kb][1];
        const float total = colsum + __shfl_xor(colsum, 32, WAVE);
        const int key = k0 + 32 * kb + (lane & 31);
        if (lane < 32 && key < N) mass_s[key] = key < n ? total : 0.f;
    }
    barrier_no_fence();                                       // everybody is done with LDS before the next tile's loads
    }
}

// ------------------------------------------------------------------------------------------
// host launcher
// ------------------------------------------------------------------------------------------

int attn_lse_stride(int N);

// Row statistics handed in by the caller: natural-log sums, one per query row, without padding.
// They are copied into the padded layout that the column-sum kernel streams (scale = log2(e): L_t
// in base 2, or -sqrt(d): -L_t / c for attn_colsum_pipe_kernel); rows past the slice's length get
// the infinity that makes their terms vanish.
__global__ void __launch_bounds__(256) lse_import_kernel(const float *__restrict__ row_lse, float *__restrict__ lse,
                                                         const int32_t *__restrict__ seq_lens, int HG, int N, int n_pad,
                                                         int blocks_per_slice, float scale, float pad)
{
    const int qslice = blockIdx.x / blocks_per_slice;
    const int q = (blockIdx.x % blocks_per_slice) * 256 + threadIdx.x;
    if (q >= n_pad) return;
    int n = seq_lens ? seq_lens[qslice / HG] : N;
    n = n < 0 ? 0 : (n > N ? N : n);
    lse[(size_t)qslice * n_pad + q] = q < n ? row_lse[(size_t)qslice * N + q] * scale : pad;
}

void launch_colsum_pipe(const kvm_shape &sh, const void *Q, const void *K, const float *neg_lse, float *mass, float *sim_opt,
                        int n_pad, float c, hipStream_t st);

// From this length on the column sums of 16-bit inputs are taken by attn_colsum_pipe_kernel
// (attn_pipe.hip): measured 5 % faster at N = 16384, 1-3 % slower at N = 4096, where the eight
// diagonal steps of its 512-key workgroups weigh more.
constexpr int COLSUM_PIPE_MIN_N = 8192;

template <typename T>
static kvm_status launch_t(const kvm_shape &sh, const void *Q, const void *K, const float *row_lse, float *mass, float *lse,
                           float *sim_opt, hipStream_t st)
{
    constexpr int ROWS = ATT_WAVES * 32 * Mma<T>::NBLK;
    const int tiles = (sh.N + ROWS - 1) / ROWS;
    const float c = (float)(1.4426950408889634 / sqrt((double)sh.d));
    const int n_q = sh.B * sh.H_kv * sh.G, n_kv = sh.B * sh.H_kv;
    const int n_pad = attn_lse_stride(sh.N);
    const bool pipe = Mma<T>::NBLK == 2 && sh.N >= COLSUM_PIPE_MIN_N;
    // how the row statistic is stored for the second pass: L_t, or -L_t / c for attn_colsum_pipe_kernel
    const float out_scale = pipe ? -1.f / c : 1.f, pad = pipe ? -INFINITY : INFINITY;
    if (row_lse) {
        ProfScope prof("lse_import_kernel", st);
        const int per = (n_pad + 255) / 256;
        hipLaunchKernelGGL(lse_import_kernel, dim3((unsigned)((long long)per * n_q)), dim3(256), 0, st, row_lse, lse,
                           sh.seq_lens, sh.H_kv * sh.G, sh.N, n_pad, per, 1.44269504088896341f * out_scale, pad);
        kvm_status rc = check_launch("lse_import_kernel");
        if (rc != KVM_OK) return rc;
    } else {
        // long sequences: half as many workgroups, each with one long and one short row tile
        // (measured faster from 8 tiles per slice on; below that the second tile's start-up,
        // which nothing overlaps, costs more than the even load gains)
        const int wgs = tiles >= 8 ? (tiles + 1) / 2 : tiles;
        const long long blocks = (long long)((n_q + 7) / 8) * 8 * wgs;
        int32_t *redo = reinterpret_cast<int32_t *>(lse + (size_t)n_q * n_pad);   // one flag per (query slice, row tile)
        if constexpr (Mma<T>::NBLK == 2) {
            {
                ProfScope prof("attn_lse_kernel", st);
                hipLaunchKernelGGL((attn_lse_kernel<T, true>), dim3((unsigned)blocks), dim3(ATT_BLOCK), 0, st, (const T *)Q,
                                   (const T *)K, lse, redo, sh.seq_lens, n_q, sh.H_kv * sh.G, sh.G, sh.N, n_pad, tiles, wgs, c,
                                   out_scale, pad);
            }
            kvm_status rc = check_launch("attn_lse_kernel");
            if (rc != KVM_OK) return rc;
            ProfScope prof("attn_lse_redo_kernel", st);
            hipLaunchKernelGGL((attn_lse_kernel<T, false>), dim3((unsigned)((n_q + 7) / 8 * 8)), dim3(ATT_BLOCK), 0, st,
                               (const T *)Q, (const T *)K, lse, redo, sh.seq_lens, n_q, sh.H_kv * sh.G, sh.G, sh.N, n_pad,
                               tiles, 1, c, out_scale, pad);
        } else {
            ProfScope prof("attn_lse_kernel", st);
            hipLaunchKernelGGL((attn_lse_kernel<T, false>), dim3((unsigned)blocks), dim3(ATT_BLOCK), 0, st, (const T *)Q,
                               (const T *)K, lse, (int32_t *)nullptr, sh.seq_lens, n_q, sh.H_kv * sh.G, sh.G, sh.N, n_pad,
                               tiles, wgs, c, out_scale, pad);
        }
        kvm_status rc = check_launch("attn_lse_kernel");
        if (rc != KVM_OK) return rc;
    }
    {
        const int wgs = tiles >= 8 ? (tiles + 1) / 2 : tiles;   // as for the row statistics
        const long long blocks = (long long)((n_kv + 7) / 8) * 8 * wgs;
        ProfScope prof(pipe ? "attn_colsum_pipe_kernel" : "attn_colsum_kernel", st);
        if (pipe) launch_colsum_pipe(sh, Q, K, lse, mass, sim_opt, n_pad, c, st);
        else hipLaunchKernelGGL(attn_colsum_kernel<T>, dim3((unsigned)blocks), dim3(ATT_BLOCK), 0, st, (const T *)Q,
                           (const T *)K, (const float *)lse, mass, sizeof(T) == 2 ? sim_opt : nullptr, sh.seq_lens, n_kv, sh.H_kv,
                           sh.G, sh.N, n_pad, tiles, wgs, c);
        return check_launch("attn_colsum_kernel");
    }
}

// Row statistics are stored with the sequence length rounded up to a whole streamed tile.
int attn_lse_stride(int N) { return (N + 63) / 64 * 64; }
// Row tiles per slice, for the flags that follow the row statistics in the workspace.
int attn_row_tiles(int N) { return (N + 255) / 256; }

// row_lse == nullptr: the row statistics are computed here (first score pass); otherwise the
// caller's are imported and only the column-sum pass runs.
// sim_opt != nullptr: the column-sum kernels also write the adjacent-key similarities (16-bit types;
// fp32 keys sit in another register layout and get the streaming scan instead).
kvm_status launch_attn_mass(const kvm_shape &sh, const void *Q, const void *K, const float *row_lse, float *mass, float *lse,
                            float *sim_opt, hipStream_t st)
{
    if ((long long)sh.B * sh.H_kv == 0 || sh.N == 0) return KVM_OK;
    switch (sh.dtype) {
    case KVM_F32: {
        kvm_status rc = launch_t<float>(sh, Q, K, row_lse, mass, lse, nullptr, st);
        return rc == KVM_OK && sim_opt ? launch_cosine_scan(sh, K, sim_opt, st) : rc;
    }
    case KVM_F16: return launch_t<half_t>(sh, Q, K, row_lse, mass, lse, sim_opt, st);
    default: return launch_t<bf16_t>(sh, Q, K, row_lse, mass, lse, sim_opt, st);
    }
}

}  // namespace kvm
