// Building blocks shared by the attention-mass kernels (Section 2.4 Eq. (1); Section 4.2 Eq. (7)):
// the MFMA wrappers, the streamed tile in LDS with its swizzle and asynchronous loads, the
// stationary operand in registers, and the blockIdx -> (slice, tile) map.
#pragma once

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
typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

constexpr int ATT_MIN_BLOCKS = 3;        // workgroups per CU the register budget is held to (3 waves per SIMD)

// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14; other counters at max)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for
// every outstanding global_load_lds, i.e. for the tiles that are meant to stay in flight.
// The LDS data a step needs is waited for explicitly with wait_vmcnt before the barrier.
__device__ __forceinline__ void barrier_no_fence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <typename T> struct Tile {
    static constexpr int CH = Mma<T>::CHUNKS;
    static constexpr int TR = 32 * Mma<T>::NBLK;
    static constexpr int SLOTS = TR * CH;                     // 16-byte slots per stage
    static constexpr int PER_THREAD = SLOTS / ATT_BLOCK;      // global_load_lds instructions per wave and tile
    static __device__ __forceinline__ int lds_index(int row, int ch) { return row * CH + (ch ^ (row & (CH - 1))); }

    // Rows [row0, row0+TR) of an (N x 128) matrix -> one LDS stage, asynchronously.  One
    // instruction fills 64 consecutive slots (lane l -> slot base + l), so the swizzle is
    // applied on the source side: the lane that fills slot (row, pos) fetches chunk
    // pos ^ (row mod CH).  The byte offsets of a lane's loads relative to the first row of
    // the tile do not depend on the tile: they are computed once, and a full tile is then
    // fetched with a scalar base address and no per-lane arithmetic.
    struct Offsets { uint32_t v[PER_THREAD]; };
    static __device__ __forceinline__ Offsets offsets(int wave, int lane) {
        Offsets o;
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int slot0 = (wave * PER_THREAD + i) * 64;
            const int row = slot0 / CH + lane / CH;
            const int pos = lane % CH;
            o.v[i] = (uint32_t)(row * (HEAD_DIM * (int)sizeof(T)) + ((pos ^ (row & (CH - 1))) * 16));
        }
        return o;
    }
    // the same offsets for a ragged tile with only rows_valid (1 <= rows_valid < TR) rows:
    // rows past the end are replaced by the last valid row (finite data whose scores are
    // masked or weighted by zero later), so that nothing outside the matrix is read
    static __device__ __forceinline__ Offsets offsets_clamped(int wave, int lane, int rows_valid) {
        Offsets o;
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int slot0 = (wave * PER_THREAD + i) * 64;
            const int row = slot0 / CH + lane / CH;
            const int pos = lane % CH;
            o.v[i] = (uint32_t)(min(row, rows_valid - 1) * (HEAD_DIM * (int)sizeof(T)) + ((pos ^ (row & (CH - 1))) * 16));
        }
        return o;
    }
    // Rows [row0, row0+TR) of the matrix whose row 0 is at `base`, clamped to n_valid rows.  The
    // tile's first row goes through readfirstlane so that it stays in scalar registers and the
    // loads take the (scalar base + 32-bit lane offset) form.
    static __device__ __forceinline__ void issue(const T *base, int row0, int n_valid, const Offsets &full, u32x4 *stage,
                                                 int wave, int lane) {
        Offsets o = full;
        if (row0 + TR > n_valid) o = offsets_clamped(wave, lane, n_valid - row0);
        const uint64_t u = reinterpret_cast<uint64_t>(base + (size_t)row0 * HEAD_DIM);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
        const char *first_row = reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(first_row + o.v[i]), (lptr_t)(stage + (wave * PER_THREAD + i) * 64), 16, 0, 0);
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

// Cosine similarity of adjacent keys (Section 3.1 Eq. (2)) from a stationary block of keys that a
// column-sum kernel holds in registers anyway: sim[j] = cos(k_{j-1}, k_j) for the 32 rows from row0
// on (0 for j = 0, for a zero-norm key and on padding), the values cosine_scan_kernel writes, up to
// the order of the fp32 additions.  Lanes l and l+32 hold the even and the odd 16-byte chunks of
// row l; the row before is one lane below, except for the block's first row, whose predecessor
// comes from memory (load_predecessor).  16-bit types only.
// The predecessor of a block's first row: one 16-byte chunk per lane of the first 16 (issued with
// the loads of the stationary operand, used by stationary_cosine).
template <typename T>
__device__ __forceinline__ u32x4 load_predecessor(const T *Ks, int row0, int n, int lane)
{
    u32x4 chunk = {0u, 0u, 0u, 0u};
    if (lane < 16 && row0 >= 1 && row0 < n)
        chunk = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(Ks + (size_t)(row0 - 1) * HEAD_DIM) + lane * 16);
    return chunk;
}

template <typename T>
__device__ __forceinline__ void stationary_cosine(int row0, int n, int N, int lane, const u32x4 *frags, const u32x4 &chunk,
                                                  float *sim_s)
{
    typedef typename Elem<T>::Raw Raw;
    const int row = row0 + (lane & 31);
    const bool first = (lane & 31) == 0;                     // lanes 0 and 32 collect the even and the odd chunks
    float dot = 0.f, nn = 0.f, pn = 0.f;
#pragma unroll
    for (int f = 0; f < Mma<T>::FRAGS; ++f) {
        u32x4 prev, far;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            prev[i] = (uint32_t)__shfl_up((int)frags[f][i], 1, WAVE);
            far[i] = (uint32_t)__shfl((int)chunk[i], 2 * f + (lane >> 5), WAVE);
        }
        if (first) prev = far;
        pn += RowDot<T>::dot(Raw{far}, Raw{far});             // (used by the first lanes only)
        dot += RowDot<T>::dot(Raw{frags[f]}, Raw{prev});
        nn += RowDot<T>::dot(Raw{frags[f]}, Raw{frags[f]});
    }
    dot += __shfl_xor(dot, 32, WAVE);
    nn += __shfl_xor(nn, 32, WAVE);
    pn += __shfl_xor(pn, 32, WAVE);
    float nn_prev = __shfl_up(nn, 1, WAVE);
    if (first) nn_prev = pn;
    const float s = (row >= 1 && row < n) ? (dot * inv_norm(nn)) * inv_norm(nn_prev) : 0.f;
    if (lane < 32 && row < N) sim_s[row] = s;
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


__device__ __forceinline__ float max16(const f32x16 &v) {
    const float a = fmaxf(fmaxf(v[0], v[1]), v[2]), b = fmaxf(fmaxf(v[3], v[4]), v[5]);
    const float c = fmaxf(fmaxf(v[6], v[7]), v[8]), d = fmaxf(fmaxf(v[9], v[10]), v[11]);
    const float e = fmaxf(fmaxf(v[12], v[13]), v[14]);
    return fmaxf(fmaxf(fmaxf(a, b), fmaxf(c, d)), fmaxf(e, v[15]));
}

constexpr float M_INIT = -3.0e38f;       // "no score seen yet": finite, so that no inf - inf arises

// Unmasked tiles (16-bit types): the 8 A fragments of a 32-row block are fetched once, all
// reads in flight together, and serve both stationary blocks of the wave.
// The slot of fragment f of a lane within a 32-row block does not depend on the block or the
// stage; the eight slots are computed once and the block and stage become constant offsets.
struct FragSlots { int v[8]; };
template <typename T>
__device__ __forceinline__ FragSlots frag_slots(int lane) {
    FragSlots s;
#pragma unroll
    for (int f = 0; f < 8; ++f) s.v[f] = Tile<T>::lds_index(lane & 31, 2 * f + (lane >> 5));
    return s;
}
template <typename T>
__device__ __forceinline__ void load_frags8(const u32x4 *tile, int blk, const FragSlots &s, u32x4 *a) {
#pragma unroll
    for (int f = 0; f < 8; ++f) a[f] = tile[s.v[f] + 32 * Tile<T>::CH * blk];
}

// accumulator i of lane l: is its row index inside the 32x32 block above / below the lane's column?
__device__ __forceinline__ void mask_rows_above_col(f32x16 &acc, int lane) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (acc_row(i, lane) > (lane & 31)) acc[i] = -INFINITY;
}
__device__ __forceinline__ void mask_rows_below_col(f32x16 &acc, int lane) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (acc_row(i, lane) < (lane & 31)) acc[i] = -INFINITY;
}


}  // namespace kvm
