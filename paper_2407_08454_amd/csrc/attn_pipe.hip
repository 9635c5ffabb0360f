// Column sums of the attention map for 16-bit inputs and long sequences (Section 4.2 Eq. (7);
// Algorithm 2 step 2): the second score pass of attn_mass.hip,
//     mass_j = sum_g sum_{t>=j} exp2(c (s_tj - L_t / c)),   c = log2(e)/sqrt(d),
// in a shape that moves fewer bytes per MFMA.  It takes the row statistics as -L_t / c.
//
// Shape of a step.  A wave keeps FOUR 32-key blocks in registers (128 VGPRs), so a 16-byte
// fragment read from the streamed query tile in LDS feeds four MFMAs, and a workgroup of four
// waves covers 512 keys; two workgroups per CU (256 registers per wave).  One (streamed block,
// stationary block) pair is a "unit": 8 MFMAs 32x32x16 into 16 accumulators, then one multiply, one
// exp2 and one add per accumulator.  The MFMAs of a unit are issued among the softmax arithmetic of
// the unit before it (two accumulator sets per wave), so that a single wave keeps both the matrix
// pipe and the vector ALU busy: a chain of 8 dependent MFMAs issued back to back lets a wave issue
// nothing else for 256 cycles, and two waves per SIMD cannot cover for each other.  The order
// inside a region is fixed with sched_group_barrier: MFMA, 2 x mul, 2 x exp2, 2 x add, eight times.
//
// Every accumulator starts at -L_t / c, so that the MFMA chain leaves s_tj - L_t / c and the term
// is exp2(c * acc): below the diagonal the 16 statistics of a streamed block sit in registers and
// enter as the addend of the first MFMA of each of its four units; rows past the sequence end
// carry -inf there and vanish.
//
// The 16 blocks of a workgroup's 512 keys are dealt to the waves as {w, 7-w, 8+w, 15-w}: in the
// eight steps around the diagonal every wave then has the same number of units (34), instead of
// one wave doing 58 and another 10.  For a streamed block the units on or below the diagonal are a
// prefix of the wave's ascending block list, the unit on the diagonal being its end; the diagonal
// steps run one streamed block at a time through code specialised on the length of that prefix.
//
// What this buys: on this chip both score passes are limited by power, not by issue slots (the
// same throughput shows as 54 % matrix-pipe utilisation at 1.76 GHz here and as 60 % at 1.5 GHz in
// attn_colsum_kernel), so only what lowers the energy per score counts: half the LDS fragment
// reads, a quarter of the row-statistic reads and half the tile traffic per MFMA.  That is worth
// 5 % at N = 16384; at N = 4096 the eight diagonal steps of a 512-key workgroup (against four of a
// 256-key one) cost more than that, hence the length from which the launcher picks this kernel.
#include "attn_tile.h"

namespace kvm {

constexpr int PIPE_R = 4;                                  // stationary 32-row blocks per wave
constexpr int PIPE_ROWS = ATT_WAVES * 32 * PIPE_R;         // rows of a workgroup (512)
constexpr int PIPE_WGS_PER_CU = 2;                         // two waves per SIMD: 256 registers each
#ifndef PIPE_PAIR_MIN_TILES
#define PIPE_PAIR_MIN_TILES 4
#endif

// i-th (ascending) of the four blocks of wave w among the 16 blocks of the workgroup's rows
__device__ __forceinline__ int owned_block(int wave, int i) {
    return i == 0 ? wave : (i == 1 ? 7 - wave : (i == 2 ? 8 + wave : 15 - wave));
}

// element idx (0..3, the same for the whole wave) of a four-element array held in scalar registers
__device__ __forceinline__ int pick4(const int *v, int idx) {
    return idx <= 0 ? v[0] : (idx == 1 ? v[1] : (idx == 2 ? v[2] : v[3]));
}

// The order of one region: each of the 8 MFMAs is followed by the arithmetic of two scores of the
// unit before it (and, where the next streamed block is fetched meanwhile, by one LDS read).
template <int LDS_READS>
__device__ __forceinline__ void interleave_slot() {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // 1 MFMA
    if (LDS_READS > 0) __builtin_amdgcn_sched_group_barrier(0x100, LDS_READS, 0);   // LDS reads
    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);                 // 2 VALU: multiply(-add)
    __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);                 // 2 transcendental: exp2
    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);                 // 2 VALU: add
}
// LDS_READS of them (0, 8 or 12) are spread over the region's eight slots
template <int LDS_READS>
__device__ __forceinline__ void interleave_region() {
    constexpr int EARLY = LDS_READS > 8 ? 2 : (LDS_READS > 0 ? 1 : 0), LATE = LDS_READS > 0 ? 1 : 0;
    interleave_slot<EARLY>();
    interleave_slot<EARLY>();
    interleave_slot<EARLY>();
    interleave_slot<EARLY>();
    interleave_slot<LATE>();
    interleave_slot<LATE>();
    interleave_slot<LATE>();
    interleave_slot<LATE>();
}

// The eight A fragments of 32-row block blk of a streamed tile.  The slot of fragment f is
// slot0 ^ 2f (the swizzle of Tile::lds_index written out); slot0 is passed through an empty asm so
// that the eight slots are rebuilt here (8 XORs) rather than kept in eight registers for the whole
// kernel, which the register budget of this kernel does not have.
template <typename T>
__device__ __forceinline__ void load_frags_x(const u32x4 *tile, int blk, int slot0, u32x4 *a) {
    asm volatile("" : "+v"(slot0));
#pragma unroll
    for (int f = 0; f < 8; ++f) a[f] = tile[(slot0 ^ (2 * f)) + 32 * Tile<T>::CH * blk];
}
__device__ __forceinline__ int frag_slot0(int lane) { return (lane & 31) * 16 + ((lane >> 5) ^ (lane & 15)); }

// Tile<T>::issue for 16-bit types with the four per-lane byte offsets rebuilt from the lane number
// at every call (same reason).  Load i of a lane fills slot (row, pos) = (16 wave + 4 i + lane/16,
// lane%16) with source chunk pos ^ (row mod 16); rows past the end of the matrix are replaced by
// the last valid row.
template <typename T>
__device__ __forceinline__ void issue_tile(const T *base, int row0, int n_valid, u32x4 *stage, int wave, int lane) {
    asm volatile("" : "+v"(lane));
    const int t = lane >> 4, p = lane & 15;
    const int last_row = n_valid - row0 - 1;                  // >= 0
    const uint64_t u = reinterpret_cast<uint64_t>(base + (size_t)row0 * HEAD_DIM);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    const char *first_row = reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = wave * 16 + 4 * i + t;
        const uint32_t off = (uint32_t)(min(row, last_row) * (HEAD_DIM * (int)sizeof(T)) + ((p ^ (4 * i + t)) * 16));
        __builtin_amdgcn_global_load_lds((gptr_t)(first_row + off), (lptr_t)(stage + (wave * 4 + i) * 64), 16, 0, 0);
    }
}

// keeps the running sums where the program has them: without it the optimiser moves the softmax
// arithmetic of several units into one place and the interleaving is lost
__device__ __forceinline__ void pin1(float &p) { asm volatile("" : "+v"(p)); }

template <typename T>
__device__ __forceinline__ void mfma_chain(f32x16 &acc, const u32x4 *a, const u32x4 *b) {
#pragma unroll
    for (int f = 0; f < 8; ++f) Mma<T>::mma(acc, a[f], b[f]);
}

__device__ __forceinline__ f32x16 neg_inf_acc() {
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = -INFINITY;
    return acc;
}

// pass 2: accumulators of a unit start at -L_t / c of their rows (accumulator i of lane l is row
// 8*(i/4) + 4*(l/32) + i%4 of the streamed 32-row block)
__device__ __forceinline__ f32x16 init_from_rowstats(const float *neg_lse_tile, int blk, int lane) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(&neg_lse_tile[32 * blk + 8 * r + 4 * (lane >> 5)]);
        acc[4 * r] = v[0];
        acc[4 * r + 1] = v[1];
        acc[4 * r + 2] = v[2];
        acc[4 * r + 3] = v[3];
    }
    return acc;
}

// pass 2: part += exp2(c * acc) (one running sum: the adds sit between MFMAs, their latency is covered)
__device__ __forceinline__ void colsum_terms(const f32x16 &acc, float c, float &part) {
#pragma unroll
    for (int i = 0; i < 16; ++i) part += __builtin_amdgcn_exp2f(acc[i] * c);
}

// The unit whose softmax terms are still to be added: its 16 accumulators and which of the wave's
// four running sums they belong to (idx is the same for the whole wave).  In the steps below the
// diagonal idx is known at compile time; in the diagonal steps the units that exist depend on the
// wave and the step, so the terms are summed into a temporary and added where idx says.
struct Pending {
    f32x16 acc;
    int idx;
};
__device__ __forceinline__ void add_at(float *sums, int idx, float v) {
    if (idx == 0) sums[0] += v;
    else if (idx == 1) sums[1] += v;
    else if (idx == 2) sums[2] += v;
    else sums[3] += v;
}

// ------------------------------------------------------------------------------------------
// pass 2: column sums
// ------------------------------------------------------------------------------------------

// One streamed block in the diagonal steps: NF units entirely below the diagonal against the
// wave's first NF stationary blocks, then, if `masked`, the unit on the diagonal against block NF.
// Every unit's MFMAs are issued among the terms of the pending unit, which may stem from the block
// or the step before; the last unit of this block is pending on return.
template <typename T, int NF>
__device__ __forceinline__ void colsum_diag_block(bool masked, const u32x4 *cur, const float *cur_lse, int blk, int slot0,
                                                  const u32x4 (*kf)[8], float *part, float c, int lane, Pending &pend)
{
    u32x4 a[8];
    load_frags_x<T>(cur, blk, slot0, a);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        f32x16 acc = init_from_rowstats(cur_lse, blk, lane);  // (read again for every unit: no registers to hold them here)
        mfma_chain<T>(acc, a, kf[i]);
        float sum = 0.f;
        colsum_terms(pend.acc, c, sum);
        pin1(sum);
        interleave_region<0>();
        __builtin_amdgcn_sched_barrier(0);
        add_at(part, pend.idx, sum);
        pend.acc = acc;
        pend.idx = i;
    }
    if (NF < PIPE_R && masked) {
        f32x16 acc = init_from_rowstats(cur_lse, blk, lane);
        mfma_chain<T>(acc, a, kf[NF < PIPE_R ? NF : 0]);
        float sum = 0.f;
        colsum_terms(pend.acc, c, sum);
        pin1(sum);
        interleave_region<0>();
        __builtin_amdgcn_sched_barrier(0);
        add_at(part, pend.idx, sum);
        mask_rows_below_col(acc, lane);                       // accumulator rows are queries, columns keys
        pend.acc = acc;
        pend.idx = NF;
    }
    {   // the block's last unit is added here rather than carried into the next block: carrying it
        // costs more registers than this kernel has (the compiler then spills stationary fragments)
        float sum = 0.f;
        colsum_terms(pend.acc, c, sum);
        add_at(part, pend.idx, sum);
        pend.acc = neg_inf_acc();
        pend.idx = PIPE_R - 1;
        __builtin_amdgcn_sched_barrier(0);
    }
}

// nf units below the diagonal, then the masked one if there is one; both are the same for the
// whole wave: scalar branches
template <typename T>
__device__ __forceinline__ void colsum_diag_dispatch(int nf, bool masked, const u32x4 *cur, const float *cur_lse, int blk,
                                                     int slot0, const u32x4 (*kf)[8], float *part, float c,
                                                     int lane, Pending &pend)
{
    switch (nf) {
    case 0: if (masked) colsum_diag_block<T, 0>(true, cur, cur_lse, blk, slot0, kf, part, c, lane, pend); break;
    case 1: colsum_diag_block<T, 1>(masked, cur, cur_lse, blk, slot0, kf, part, c, lane, pend); break;
    case 2: colsum_diag_block<T, 2>(masked, cur, cur_lse, blk, slot0, kf, part, c, lane, pend); break;
    case 3: colsum_diag_block<T, 3>(masked, cur, cur_lse, blk, slot0, kf, part, c, lane, pend); break;
    default: colsum_diag_block<T, 4>(false, cur, cur_lse, blk, slot0, kf, part, c, lane, pend); break;
    }
}

template <typename T>
__global__ __launch_bounds__(ATT_BLOCK, PIPE_WGS_PER_CU) void attn_colsum_pipe_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const float *__restrict__ neg_lse, float *__restrict__ mass,
    float *__restrict__ sim_opt, const int32_t *__restrict__ seq_lens, int n_kvslices, int H, int G, int N, int n_pad,
    int tiles_per_slice, int wgs_per_slice, float c)
{
    using TL = Tile<T>;
    constexpr int TR = TL::TR;                                // 64 rows per streamed tile
    static_assert(TR == 64 && Mma<T>::FRAGS == 8, "16-bit types only");
    // one LDS object per stage: the compiler then knows that the fragment reads of a step do
    // not touch the stage the next tile is being loaded into, and does not wait for that load
    __shared__ u32x4 lds_a[TL::SLOTS], lds_b[TL::SLOTS];
    __shared__ __attribute__((aligned(16))) float lse_a[TR], lse_b[TR];

    const TileMap tm = map_block(n_kvslices, wgs_per_slice);
    if (!tm.valid) return;
    const int kvslice = tm.slice;
    const int b = kvslice / H, h = kvslice % H;
    const int n = clamp_len(seq_lens, b, N);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float *mass_s = mass + (size_t)kvslice * N;
    float *sim_s = sim_opt ? sim_opt + (size_t)kvslice * N : nullptr;
    const T *Ks = K + (size_t)kvslice * N * HEAD_DIM;
    const int slot0 = frag_slot0(lane);
    int blk_of[PIPE_R];                                       // the wave's blocks, ascending (scalar)
#pragma unroll
    for (int i = 0; i < PIPE_R; ++i) blk_of[i] = owned_block(wave, i);

    // workgroup t takes key tile t (the one with the most rows below it) and, when there are fewer
    // workgroups than tiles, then also tile tiles-1-t, so that all workgroups carry the same load
    const bool paired = wgs_per_slice < tiles_per_slice;
    for (int pass = 0; pass < 2; ++pass) {
    const int tile = pass == 0 ? tm.tile : tiles_per_slice - 1 - tm.tile;
    if (pass == 1 && (!paired || tm.tile >= tiles_per_slice - 1 - tm.tile)) break;
    const int k_begin = tile * PIPE_ROWS;
    if (k_begin >= n) {                                       // padding only: defined zeros
        for (int j = k_begin + threadIdx.x; j < min(k_begin + PIPE_ROWS, N); j += ATT_BLOCK) {
            mass_s[j] = 0.f;
            if (sim_s) sim_s[j] = 0.f;
        }
        continue;
    }
    // Query tiles first .. last see these keys; tiles first .. first+7 hold the diagonal.  They are
    // streamed from the last one down, head after head: every workgroup of a slice starts at the
    // same tile and walks down in step with the others, so a tile is fetched from memory once.
    const int first = k_begin / TR;
    const int last = (n - 1) / TR;
    const int steps = (last - first + 1) * G;
    auto issue = [&](int g, int qt, u32x4 *stage, float *stage_lse) {
        const size_t qslice = ((size_t)b * H + h) * G + g;
        const T *Qh = Q + qslice * N * HEAD_DIM;
        const int row0 = qt * TR;
        issue_tile<T>(Qh, row0, n, stage, wave, lane);
        if (wave == 0)
            __builtin_amdgcn_global_load_lds((gptr_t)(neg_lse + qslice * n_pad + row0 + lane), (lptr_t)stage_lse, 4, 0, 0);
    };
    int g_next = 0, qt_next = last;
    auto issue_next = [&](u32x4 *stage, float *stage_lse) {
        issue(g_next, qt_next, stage, stage_lse);
        if (qt_next == first) { qt_next = last; ++g_next; } else --qt_next;
    };
    issue_next(lds_a, lse_a);
    u32x4 kf[PIPE_R][8];
#pragma unroll
    for (int i = 0; i < PIPE_R; ++i) load_stationary<T>(Ks, k_begin + 32 * blk_of[i], n, lane, kf[i]);
    if (sim_s) {                                              // the keys are here anyway: their adjacent similarities
        u32x4 before[PIPE_R];
#pragma unroll
        for (int i = 0; i < PIPE_R; ++i) before[i] = load_predecessor<T>(Ks, k_begin + 32 * blk_of[i], n, lane);
#pragma unroll
        for (int i = 0; i < PIPE_R; ++i) stationary_cosine<T>(k_begin + 32 * blk_of[i], n, N, lane, kf[i], before[i], sim_s);
    }
    float part[PIPE_R];
#pragma unroll
    for (int i = 0; i < PIPE_R; ++i) part[i] = 0.f;

    Pending pend;                                             // below the diagonal a step ends with a unit of block 3
    pend.acc = neg_inf_acc();                                 // (-inf: terms of zero)
    pend.idx = PIPE_R - 1;
    int qt = last + 1;
    auto step = [&](int s, const u32x4 *cur, const float *cur_lse, u32x4 *nxt, float *nxt_lse) {
        qt = qt == first ? last : qt - 1;
        wait_vmcnt<0>();                                      // this thread's part of the tile has landed
        barrier_no_fence();                                   // everybody's has; everybody is done with the other stage
        if (s + 1 < steps) issue_next(nxt, nxt_lse);
        const int rel = qt - first;                           // 0..7: the tile holds part of the diagonal
        if (rel >= 8) {
            // eight units, each unit's MFMAs among the softmax terms of the unit before it; the
            // row statistics of a streamed block sit in 16 registers and enter as the addend of
            // the first MFMA of each of its four units
            u32x4 a[8];
            load_frags_x<T>(cur, 0, slot0, a);
            f32x16 rowstats = init_from_rowstats(cur_lse, 0, lane);
            int slot1 = slot0;
            asm volatile("" : "+v"(slot1));
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
                for (int i = 0; i < PIPE_R; ++i) {
                    const bool fetch_next = blk == 0 && i == PIPE_R - 1;
                    f32x16 acc = rowstats;
#pragma unroll
                    for (int f = 0; f < 8; ++f) {
                        Mma<T>::mma(acc, a[f], kf[i][f]);
                        if (fetch_next) a[f] = cur[(slot1 ^ (2 * f)) + 32 * TL::CH];   // next block, same registers
                    }
                    if (fetch_next) rowstats = init_from_rowstats(cur_lse, 1, lane);
                    colsum_terms(pend.acc, c, part[(i + PIPE_R - 1) % PIPE_R]);
                    pin1(part[(i + PIPE_R - 1) % PIPE_R]);
                    if (fetch_next) interleave_region<12>();
                    else interleave_region<0>();
                    __builtin_amdgcn_sched_barrier(0);
                    pend.acc = acc;
                }
            }
        } else {
#pragma unroll 1
            for (int blk = 0; blk < 2; ++blk) {
                const int qb = 2 * rel + blk;                 // the streamed block among the workgroup's 16
                int nf = 0;                                   // stationary blocks entirely above it (keys before the queries)
#pragma unroll
                for (int i = 0; i < PIPE_R; ++i) nf += blk_of[i] < qb ? 1 : 0;
                const bool masked = nf < PIPE_R && pick4(blk_of, nf) == qb;
                colsum_diag_dispatch<T>(nf, masked, cur, cur_lse, blk, slot0, kf, part, c, lane, pend);
            }
            if (rel == 0) {                                   // last step of a head: add what is pending
                float sum = 0.f;
                colsum_terms(pend.acc, c, sum);
                add_at(part, pend.idx, sum);
                pend.acc = neg_inf_acc();
                pend.idx = PIPE_R - 1;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    for (int s = 0; s < steps; s += 2) {
        step(s, lds_a, lse_a, lds_b, lse_b);
        if (s + 1 < steps) step(s + 1, lds_b, lse_b, lds_a, lse_a);
    }
    wait_vmcnt<0>();                                          // no load may still target this workgroup's LDS
#pragma unroll
    for (int i = 0; i < PIPE_R; ++i) {
        const float colsum = part[i];
        const float total = colsum + __shfl_xor(colsum, 32, WAVE);
        const int key = k_begin + 32 * blk_of[i] + (lane & 31);
        if (lane < 32 && key < N) mass_s[key] = key < n ? total : 0.f;
    }
    barrier_no_fence();                                       // everybody is done with LDS before the next tile's loads
    }
}

// ------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------

template <typename T>
static void launch_colsum_pipe_t(const kvm_shape &sh, const void *Q, const void *K, const float *neg_lse, float *mass,
                                 float *sim_opt, int n_pad, float c, hipStream_t st)
{
    const int tiles = (sh.N + PIPE_ROWS - 1) / PIPE_ROWS;
    const int wgs = tiles >= PIPE_PAIR_MIN_TILES ? (tiles + 1) / 2 : tiles;
    const int n_kv = sh.B * sh.H_kv;
    const long long blocks = (long long)((n_kv + 7) / 8) * 8 * wgs;
    hipLaunchKernelGGL(attn_colsum_pipe_kernel<T>, dim3((unsigned)blocks), dim3(ATT_BLOCK), 0, st, (const T *)Q, (const T *)K,
                       neg_lse, mass, sim_opt, sh.seq_lens, n_kv, sh.H_kv, sh.G, sh.N, n_pad, tiles, wgs, c);
}

void launch_colsum_pipe(const kvm_shape &sh, const void *Q, const void *K, const float *neg_lse, float *mass, float *sim_opt,
                        int n_pad, float c, hipStream_t st)
{
    if (sh.dtype == KVM_F16) launch_colsum_pipe_t<half_t>(sh, Q, K, neg_lse, mass, sim_opt, n_pad, c, st);
    else launch_colsum_pipe_t<bf16_t>(sh, Q, K, neg_lse, mass, sim_opt, n_pad, c, st);
}

}  // namespace kvm
