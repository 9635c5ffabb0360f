// Internal helpers shared by the HIP kernels of libkvm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvm.h"

namespace kvm {

constexpr int HEAD_DIM = 128;          // the only head dimension v1 supports
constexpr int WAVE = 64;

typedef _Float16 half_t;
typedef __bf16 bf16_t;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ---- a lane's 8 consecutive elements of a 128-wide row (chunk c of 16) --------------

template <typename T> struct Elem;

template <> struct Elem<half_t> {
    static constexpr int kDtype = KVM_F16;
    struct Raw { u32x4 v; };
    static __device__ __forceinline__ Raw load(const half_t *row, int c) {
        return Raw{*reinterpret_cast<const u32x4 *>(row + c * 8)};
    }
    static __device__ __forceinline__ void store(half_t *row, int c, const Raw &r) {
        *reinterpret_cast<u32x4 *>(row + c * 8) = r.v;
    }
    static __device__ __forceinline__ void to_float(const Raw &r, float *x) {
        f16x8 h = __builtin_bit_cast(f16x8, r.v);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = (float)h[i];
    }
    static __device__ __forceinline__ Raw from_float(const float *x) {
        f16x8 h;
#pragma unroll
        for (int i = 0; i < 8; ++i) h[i] = (half_t)x[i];   // round to nearest even
        return Raw{__builtin_bit_cast(u32x4, h)};
    }
};

template <> struct Elem<bf16_t> {
    static constexpr int kDtype = KVM_BF16;
    struct Raw { u32x4 v; };
    static __device__ __forceinline__ Raw load(const bf16_t *row, int c) {
        return Raw{*reinterpret_cast<const u32x4 *>(row + c * 8)};
    }
    static __device__ __forceinline__ void store(bf16_t *row, int c, const Raw &r) {
        *reinterpret_cast<u32x4 *>(row + c * 8) = r.v;
    }
    static __device__ __forceinline__ void to_float(const Raw &r, float *x) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __builtin_bit_cast(float, r.v[i] << 16);
            x[2 * i + 1] = __builtin_bit_cast(float, r.v[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ uint32_t rne(float f) {
        uint32_t u = __builtin_bit_cast(uint32_t, f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
        return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ Raw from_float(const float *x) {
        Raw r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[i] = rne(x[2 * i]) | (rne(x[2 * i + 1]) << 16);
        return r;
    }
};

template <> struct Elem<float> {
    static constexpr int kDtype = KVM_F32;
    struct Raw { f32x4 a, b; };
    static __device__ __forceinline__ Raw load(const float *row, int c) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(row + c * 8);
        return Raw{p[0], p[1]};
    }
    static __device__ __forceinline__ void store(float *row, int c, const Raw &r) {
        f32x4 *p = reinterpret_cast<f32x4 *>(row + c * 8);
        p[0] = r.a;
        p[1] = r.b;
    }
    static __device__ __forceinline__ void to_float(const Raw &r, float *x) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[i] = r.a[i]; x[4 + i] = r.b[i]; }
    }
    static __device__ __forceinline__ Raw from_float(const float *x) {
        Raw r;
#pragma unroll
        for (int i = 0; i < 4; ++i) { r.a[i] = x[i]; r.b[i] = x[4 + i]; }
        return r;
    }
};

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// partial dot product of a lane's 8 elements of two rows, fp32 accumulation (products of two
// 16-bit values are exact in fp32)
template <typename T> struct RowDot;
template <> struct RowDot<half_t> {
    static __device__ __forceinline__ float dot(const Elem<half_t>::Raw &a, const Elem<half_t>::Raw &b) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t ai = a.v[i], bi = b.v[i];
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, ai), __builtin_bit_cast(f16x2, bi), s, false);
        }
        return s;
    }
};
template <> struct RowDot<bf16_t> {
    static __device__ __forceinline__ float dot(const Elem<bf16_t>::Raw &a, const Elem<bf16_t>::Raw &b) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t ai = a.v[i], bi = b.v[i];
            s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, ai), __builtin_bit_cast(bf16x2, bi), s, false);
        }
        return s;
    }
};
template <> struct RowDot<float> {
    static __device__ __forceinline__ float dot(const Elem<float>::Raw &a, const Elem<float>::Raw &b) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) { s0 = fmaf(a.a[i], b.a[i], s0); s1 = fmaf(a.b[i], b.b[i], s1); }
        return s0 + s1;
    }
};

// 1/sqrt(x) for a squared norm; 0 when the squared norm is zero or below the normal fp32 range
// (such a key counts as a zero-norm key: its similarities are 0)
__device__ __forceinline__ float inv_norm(float nn) { return nn >= 1.17549435e-38f ? __builtin_amdgcn_rsqf(nn) : 0.f; }

// ---- cross-lane helpers -------------------------------------------------------------

// DPP move within a row of 16 lanes; every lane is enabled so no old value is needed.
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);   // row_half_mirror: quad q <-> quad 1-q within each half row
    v += dpp_f<0x140>(v);   // row_mirror: lane i <-> lane 15-i
    return v;
}

// Sum over the four 16-lane rows of a wave (same lane position in each row).
__device__ __forceinline__ float rows4_sum(float v) {
    v += __shfl_xor(v, 16, WAVE);
    v += __shfl_xor(v, 32, WAVE);
    return v;
}

// Order-preserving map of a finite float onto uint32 (-0 and +0 map to the same key).
__device__ __forceinline__ uint32_t sortable_key(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int clamp_len(const int32_t *seq_lens, int b, int N) {
    int n = seq_lens ? seq_lens[b] : N;
    return n < 0 ? 0 : (n > N ? N : n);
}

// ---- host side -----------------------------------------------------------------------

void set_error(const char *fmt, ...);
kvm_status check_launch(const char *what);

// Brackets one kernel launch with two events when profiling is enabled (see kvm_profile_*).
struct ProfScope {
    int slot;
    hipStream_t st;
    ProfScope(const char *name, hipStream_t st);
    ~ProfScope();
};

kvm_status launch_attn_mass(const kvm_shape &sh, const void *Q, const void *K, const float *row_lse, float *mass,
                            float *lse, float *sim_opt, hipStream_t st);
kvm_status launch_cosine_scan(const kvm_shape &sh, const void *K, float *sim, hipStream_t st);
kvm_status launch_attn_append(const kvm_shape &sh, const void *q_new, const void *K, float *mass, float *ws, hipStream_t st);
kvm_status launch_sim_append(const kvm_shape &sh, const void *K, float *sim, hipStream_t st);
kvm_status launch_identify(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K,
                           const float *mass, int32_t *set_id, int32_t *set_start, int32_t *pivot,
                           int32_t *n_sets, float *sim, float *inv_norm, int32_t *run, uint8_t *flags,
                           int32_t *slice_status, hipStream_t st);
kvm_status launch_merge(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                        const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out,
                        void *V_out, float *w_opt, int32_t *plan, hipStream_t st);
kvm_status launch_merge_static(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                               const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out,
                               void *V_out, float *w_opt, hipStream_t st);
kvm_status launch_evict(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                        const float *mass, int32_t *kept, int32_t *n_kept, void *K_out, void *V_out, uint8_t *flags,
                        bool merge_values, hipStream_t st);
size_t merge_workspace_bytes(const kvm_shape &sh);
size_t merge_refresh_workspace_bytes(const kvm_shape &sh, int cap_rows);
kvm_status launch_merge_refresh(const kvm_shape &sh, const kvm_params &pr, int cap_rows, const void *K, const void *V,
                                const int32_t *prev_set_id, const int32_t *prev_set_start, const int32_t *prev_pivot,
                                const int32_t *prev_n_sets, const int32_t *set_start, const int32_t *pivot,
                                const int32_t *n_sets, void *K_out, void *V_out, int32_t *n_changed, int32_t *ws, hipStream_t st);
int attn_lse_stride(int N);
int attn_row_tiles(int N);

}  // namespace kvm
