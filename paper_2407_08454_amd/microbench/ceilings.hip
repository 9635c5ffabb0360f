// Practical ceilings of one MI355X for the two kinds of kernel in this library, measured with
// plain kernels that do nothing else.  The roofline fractions in the benchmark line are quoted
// against the published peaks (2.5 PFLOP/s dense fp16 MFMA, 8 TB/s HBM); this program shows
// what simple code reaches on the same box, which is what the kernels can be held against.
//
//   1. a stream of 32x32x16 fp16 MFMAs fed from registers (zero and random operands: the
//      difference is the chip's power limit at work);
//   2. the attention step built up piece by piece: fragments from LDS (each read feeding two
//      MFMAs), plus the softmax arithmetic of one score (fma, exp2, add), plus the per-step
//      barrier and the asynchronous tile load, plus tiles that really come from memory -- three
//      workgroups of four waves per CU, as the library's kernels run; and two other shapes of
//      the same step that move fewer tile bytes per MFMA;
//   3. issue cost of v_fma_f32, v_exp_f32 and the softmax triple;
//   4. HBM: a read-only and a copy kernel over 1 GiB.
//
// Build and run:  hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops
//                 ceilings.hip -o ceilings && ./ceilings
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

#define CHECK(x)                                                                         \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            std::exit(1);                                                                \
        }                                                                                \
    } while (0)

constexpr int CUS = 256, SIMDS = 4 * CUS;
constexpr double MFMA_FLOPS = 2.0 * 32 * 32 * 16;

// ---- 1. register-fed MFMA stream ---------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_stream(float *out, const u32x4 *src, int iters)
{
    const int lane = threadIdx.x & 63;
    u32x4 a[4], b[4];
    for (int f = 0; f < 4; ++f) {
        a[f] = src[(lane * 8 + f) & 1023];
        b[f] = src[(lane * 8 + 4 + f) & 1023];
    }
    f32x16 acc0, acc1;
    for (int i = 0; i < 16; ++i) acc0[i] = acc1[i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[f]), __builtin_bit_cast(f16x8, b[f]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, b[f]), __builtin_bit_cast(f16x8, a[f]), acc1, 0, 0, 0);
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc0[0] + acc1[5];
}

// ---- 2. the attention step, piece by piece -----------------------------------------------------
// PIECES bit 0: softmax arithmetic on every accumulator; bit 1: barrier + asynchronous tile load
// per step.  A "step" is a 64-row tile against the wave's R stationary 32-row blocks: 2 R blocks
// of 8 MFMAs, 16 fragment reads of 16 bytes per lane.  WAVES waves share the tile; WGS workgroups
// per CU.  With `stream` the tiles come from a large buffer instead of a cache-hot one, `share`
// workgroups of an XCD walking through the same tiles (as the workgroups of one slice do).
template <int PIECES, int WAVES, int WGS, int R>
__global__ __launch_bounds__(64 * WAVES, WGS) void attention_step(float *out, const u32x4 *src, int steps, float c,
                                                                   const u32x4 *stream, size_t stream_tiles, int share)
{
    __shared__ u32x4 tile[2][1024];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 2048; i += 64 * WAVES) (&tile[0][0])[i] = src[i & 1023];
    __syncthreads();
    u32x4 stat[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int f = 0; f < 8; ++f) stat[r][f] = src[(lane * 16 + r * 8 + f + wave) & 1023];
    float l0 = 0.f, l1 = 0.f;
    const float m = 0.25f;
    const size_t group = ((size_t)(blockIdx.x >> 3) / share) * 8 + (blockIdx.x & 7);
    for (int s = 0; s < steps; ++s) {
        const u32x4 *cur = tile[s & 1];
        if (PIECES & 2) {
            __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8));     // vmcnt(0): this wave's part has landed
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // the 16 chunks of 64 slots of the next tile, dealt out to the waves
            const u32x4 *g = stream ? stream + ((group * steps + s) % stream_tiles) * 1024 : src;
            for (int ch = wave; ch < 16; ch += WAVES)
                __builtin_amdgcn_global_load_lds((gptr_t)(g + ch * 64 + lane), (lptr_t)(&tile[(s + 1) & 1][ch * 64]), 16, 0, 0);
        }
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            u32x4 a[8];
#pragma unroll
            for (int f = 0; f < 8; ++f) a[f] = cur[(32 * blk + (lane & 31)) * 16 + ((2 * f + (lane >> 5)) ^ (lane & 15))];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                f32x16 acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                for (int f = 0; f < 8; ++f)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[f]), __builtin_bit_cast(f16x8, stat[r][f]), acc, 0, 0, 0);
                if (PIECES & 1) {
                    float p0 = 0.f, p1 = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; i += 2) {
                        p0 += __builtin_amdgcn_exp2f(fmaf(acc[i], c, -m));
                        p1 += __builtin_amdgcn_exp2f(fmaf(acc[i + 1], c, -m));
                    }
                    l0 += p0;
                    l1 += p1;
                } else {
                    l0 += acc[0];
                    l1 += acc[9];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8));
    out[blockIdx.x * blockDim.x + threadIdx.x] = l0 + l1;
}

// ---- 3. VALU issue cost ------------------------------------------------------------------------
constexpr int CHAINS = 16;
template <int MODE>   // 0: fma, 1: exp2, 2: fma + exp2 + add
__global__ __launch_bounds__(256) void valu_issue(float *out, int iters, float seed)
{
    float v[CHAINS], a[CHAINS];
    for (int i = 0; i < CHAINS; ++i) {
        v[i] = seed + threadIdx.x * 1e-6f + i * 1e-3f;
        a[i] = 0.f;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < CHAINS; ++i) {
            if (MODE == 0) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(v[i]) : "v"(0.999f), "v"(-0.001f));
            if (MODE == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(v[i]));
            if (MODE == 2) {
                float t;
                asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(t) : "v"(v[i]), "v"(0.999f), "v"(-0.001f));
                asm volatile("v_exp_f32 %0, %0" : "+v"(t));
                asm volatile("v_add_f32 %0, %0, %1" : "+v"(a[i]) : "v"(t));
            }
        }
    }
    float s = 0.f;
    for (int i = 0; i < CHAINS; ++i) s += v[i] + a[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- 4. HBM ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void hbm_read(const u32x4 *__restrict__ src, unsigned *out, size_t n_vec)
{
    unsigned acc = 0;
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t base = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; base < n_vec; base += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = base + (size_t)u * 256 < n_vec ? src[base + (size_t)u * 256] : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x12345678u) out[0] = acc;                  // keeps the loads alive, practically never written
}
__global__ __launch_bounds__(256) void hbm_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t base = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; base < n_vec; base += stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = base + (size_t)u * 256 < n_vec ? src[base + (size_t)u * 256] : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + (size_t)u * 256 < n_vec) dst[base + (size_t)u * 256] = v[u];
    }
}

// ---- host --------------------------------------------------------------------------------------
template <typename F> static float time_ms(F launch, int reps)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();
    CHECK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int r = 0; r < reps; ++r) {
        CHECK(hipEventRecord(e0));
        launch();
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        best = ms < best ? ms : best;
    }
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return best;
}

int main()
{
    // pseudo-random fp16 operands in [0.5, 1) with alternating signs, and an all-zero set
    std::vector<unsigned short> h(8192);
    for (int i = 0; i < 8192; ++i) h[i] = (unsigned short)(0x3800 + ((i * 2654435761u) >> 22) % 0x800 + ((i & 1) << 15));
    u32x4 *rnd, *zero;
    CHECK(hipMalloc(&rnd, 1024 * sizeof(u32x4)));
    CHECK(hipMalloc(&zero, 1024 * sizeof(u32x4)));
    CHECK(hipMemcpy(rnd, h.data(), 8192 * 2, hipMemcpyHostToDevice));
    CHECK(hipMemset(zero, 0, 1024 * sizeof(u32x4)));
    float *out;
    CHECK(hipMalloc(&out, (size_t)CUS * 8 * 256 * sizeof(float)));

    std::printf("1. register-fed MFMA 32x32x16 fp16, 4 waves per SIMD, 8 MFMAs per iteration\n");
    for (int which = 0; which < 2; ++which) {
        const int iters = 20000;
        const u32x4 *src = which ? rnd : zero;
        const float ms = time_ms([&] { hipLaunchKernelGGL(mfma_stream, dim3(CUS * 4), dim3(256), 0, 0, out, src, iters); }, 3);
        const double flops = (double)SIMDS * 4 * iters * 8 * MFMA_FLOPS;
        std::printf("   %-16s %8.3f ms   %6.0f TFLOP/s\n", which ? "random operands" : "zero operands", ms, flops / (ms * 1e-3) / 1e12);
    }

    std::printf("2. attention step model (random operands unless said otherwise)\n");
    {
        const int steps = 4000;
        const size_t stream_tiles = 65536;                   // 1 GiB of 16 KB tiles holding the random pattern
        u32x4 *big;
        CHECK(hipMalloc(&big, stream_tiles * 16384));
        for (size_t t = 0; t < stream_tiles; ++t) CHECK(hipMemcpyAsync(big + t * 1024, rnd, 16384, hipMemcpyDeviceToDevice, 0));
        CHECK(hipDeviceSynchronize());
        auto report = [&](const char *name, float ms, double mfma_per_simd) {
            std::printf("   %-66s %8.3f ms   %6.0f TFLOP/s\n", name, ms, (double)SIMDS * mfma_per_simd * MFMA_FLOPS / (ms * 1e-3) / 1e12);
        };
        const u32x4 *none = nullptr;
        const double base = 3.0 * steps * 32;                // three waves per SIMD, 32 MFMAs per wave and step
        report("4-wave workgroups, 3 per CU: fragments from LDS",
               time_ms([&] { hipLaunchKernelGGL((attention_step<0, 4, 3, 2>), dim3(CUS * 3), dim3(256), 0, 0, out, rnd, steps, 0.01f, none, 1, 8); }, 3), base);
        report("  + fma, exp2, add per score",
               time_ms([&] { hipLaunchKernelGGL((attention_step<1, 4, 3, 2>), dim3(CUS * 3), dim3(256), 0, 0, out, rnd, steps, 0.01f, none, 1, 8); }, 3), base);
        report("  + barrier and asynchronous tile load (cache-hot tile)",
               time_ms([&] { hipLaunchKernelGGL((attention_step<3, 4, 3, 2>), dim3(CUS * 3), dim3(256), 0, 0, out, rnd, steps, 0.01f, none, 1, 8); }, 3), base);
        report("  the same on zero operands",
               time_ms([&] { hipLaunchKernelGGL((attention_step<3, 4, 3, 2>), dim3(CUS * 3), dim3(256), 0, 0, out, zero, steps, 0.01f, none, 1, 8); }, 3), base);
        report("  + tiles streamed from a 1 GiB buffer, 8 workgroups per stream",
               time_ms([&] { hipLaunchKernelGGL((attention_step<3, 4, 3, 2>), dim3(CUS * 3), dim3(256), 0, 0, out, rnd, steps, 0.01f, (const u32x4 *)big, stream_tiles, 8); }, 3), base);
        report("12-wave workgroups, 1 per CU: streamed tiles, 3 workgroups per stream",
               time_ms([&] { hipLaunchKernelGGL((attention_step<3, 12, 1, 2>), dim3(CUS), dim3(768), 0, 0, out, rnd, steps, 0.01f, (const u32x4 *)big, stream_tiles, 3); }, 3), base);
        report("4 stationary blocks, 4-wave workgroups, 2 per CU: streamed tiles, 4 per stream",
               time_ms([&] { hipLaunchKernelGGL((attention_step<3, 4, 2, 4>), dim3(CUS * 2), dim3(256), 0, 0, out, rnd, steps / 2, 0.01f, (const u32x4 *)big, stream_tiles, 4); }, 3),
               2.0 * (steps / 2) * 64);
        CHECK(hipFree(big));
    }

    std::printf("3. VALU issue, 8 waves per SIMD, 16 independent chains per lane\n");
    {
        const int iters = 2048;
        const double per_simd = 8.0 * iters * CHAINS;
        float fma = time_ms([&] { hipLaunchKernelGGL((valu_issue<0>), dim3(CUS * 8), dim3(256), 0, 0, out, iters, 0.5f); }, 5);
        float ex = time_ms([&] { hipLaunchKernelGGL((valu_issue<1>), dim3(CUS * 8), dim3(256), 0, 0, out, iters, 0.5f); }, 5);
        float tri = time_ms([&] { hipLaunchKernelGGL((valu_issue<2>), dim3(CUS * 8), dim3(256), 0, 0, out, iters, 0.5f); }, 5);
        std::printf("   v_fma_f32            %6.2f ns per wave instruction and SIMD\n", fma * 1e6 / per_simd);
        std::printf("   v_exp_f32            %6.2f ns  (%.1f x fma)\n", ex * 1e6 / per_simd, ex / fma);
        std::printf("   fma + exp2 + add     %6.2f ns per score  (%.1f x fma)\n", tri * 1e6 / per_simd, tri / fma);
    }

    std::printf("4. HBM, 1 GiB, 8192 workgroups\n");
    {
        const size_t bytes = (size_t)1 << 30, n_vec = bytes / 16;
        u32x4 *a, *b;
        unsigned *flag;
        CHECK(hipMalloc(&a, bytes));
        CHECK(hipMalloc(&b, bytes));
        CHECK(hipMalloc(&flag, 4));
        CHECK(hipMemset(a, 1, bytes));
        CHECK(hipMemset(b, 2, bytes));
        float rd = time_ms([&] { hipLaunchKernelGGL(hbm_read, dim3(8192), dim3(256), 0, 0, a, flag, n_vec); }, 5);
        float cp = time_ms([&] { hipLaunchKernelGGL(hbm_copy, dim3(8192), dim3(256), 0, 0, a, b, n_vec); }, 5);
        std::printf("   read   %7.3f ms   %5.2f TB/s\n", rd, bytes / (rd * 1e-3) / 1e12);
        std::printf("   copy   %7.3f ms   %5.2f TB/s (read + written)\n", cp, 2.0 * bytes / (cp * 1e-3) / 1e12);
        CHECK(hipFree(a));
        CHECK(hipFree(b));
        CHECK(hipFree(flag));
    }
    CHECK(hipFree(rnd));
    CHECK(hipFree(zero));
    CHECK(hipFree(out));
    return 0;
}
