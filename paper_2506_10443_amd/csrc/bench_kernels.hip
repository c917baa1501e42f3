// libmnnq_bench.so - measurement helpers for bench.py, a library of its own: nothing here is part of
// the linear path or of the product's C-ABI.  What this GPU sustains for the two resources
// the decode GEMV and the prefill GEMM are priced against (Section 2.1: decode is bound by memory
// bandwidth, prefill by compute), measured with the simplest kernels that use them.
//   * mnnqb_empty: a kernel that does nothing (the launch floor of a graph of kernels).
//   * mnnqb_peak_read: every byte of a buffer is read once with 128-bit loads, consecutive lanes on
//     consecutive addresses (the access rule of Section 5.1 for GPUs) - the streaming-read rate.
//   * mnnqb_peak_mfma: back-to-back matrix instructions on register operands, optionally followed
//     by the vector work the prefill epilogue needs per MFMA (4 converts + 4 fused multiply-adds,
//     or those plus 8 integer operations) in the order the GEMM issues them (MFMA of tile t + 1,
//     then the dependent epilogue of tile t) - the matrix rate and what each VALU instruction costs.
//     Kinds 3 and 4 are the loop shape of the fp6 GEMM: two chained v_mfma_scale_f32_32x32x64_f8f6f4
//     (fp6 operands) per 32 x 32 tile and group, without and with the 16 multiply-adds behind them.
//     seed 1 gives operands of small constants, any other seed operands whose bits differ from lane to
//     lane like real data: the chip runs these loops against its power limit, and the clock it grants
//     depends on how many bits toggle.  sink[1] receives the shader clock in MHz that wave 0 of
//     workgroup 0 saw over the kernel's life.
// The caller times the launches; nothing else is returned but a status (0 = ok, negative = bad argument).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace {

int num_cus()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    return n;
}

}  // namespace

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void peak_read_kernel(const u32x4* __restrict__ p, int64_t n16, uint32_t* sink)
{
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(p + i);
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;   // keeps the loads alive; practically never taken
}

// Operand words of the matrix loops: small constants (seed 1: hardly a bit toggles in the matrix pipe), or
// for any other seed bits that differ from lane to lane and word to word like those of real operands.
__device__ __forceinline__ int operand_word(int seed, int i)
{
    if (seed == 1) return i == 0 ? seed : i;
    uint32_t h = (uint32_t)(threadIdx.x * 8 + i) * 2654435761u ^ (uint32_t)seed * 0x9e3779b9u;
    h ^= h >> 15; h *= 0x85ebca6bu; h ^= h >> 13;
    return (int)h;
}

// Shader clock in MHz over the kernel's life, seen by wave 0 of workgroup 0: cycles of the clock the SIMDs
// run on against the constant 100 MHz reference counter.
struct ClockProbe {
    uint64_t c0, r0;
    __device__ void start() { c0 = __builtin_amdgcn_s_memtime(); r0 = __builtin_amdgcn_s_memrealtime(); }
    __device__ void stop(float* sink) const
    {
        const uint64_t c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
        if (blockIdx.x == 0 && threadIdx.x == 0 && r1 > r0) sink[1] = (float)(c1 - c0) / (float)(r1 - r0) * 100.0f;
    }
};

// KIND 0: v_mfma_i32_16x16x64_i8, 1: v_mfma_f32_16x16x32_f16, 2: v_mfma_f32_16x16x128_f8f6f4 (fp8).
// EPI (KIND 0 only) 0: none, 1: 4 cvt + 4 fma per MFMA, 2: the same plus 8 integer operations.
template <int KIND, int EPI>
__global__ __launch_bounds__(1024) void peak_mfma_kernel(int iters, int seed, float* sink)
{
    constexpr int NT = 16;
    ClockProbe clock;
    clock.start();
    v4i ai = {operand_word(seed, 0), operand_word(seed, 1), operand_word(seed, 2), operand_word(seed, 3)}, bi[4];
    for (int j = 0; j < 4; ++j)
        bi[j] = v4i{operand_word(seed, 4 + j), operand_word(seed, 8 + j), operand_word(seed, 12 + j), operand_word(seed, 16 + j)};
    h8 ah, bh;
    for (int i = 0; i < 8; ++i) {   // halves: small integers, so that the sums stay finite
        ah[i] = (_Float16)(float)(operand_word(seed, 20 + i) % 64);
        bh[i] = (_Float16)(float)(operand_word(seed, 28 + i) % 64);
    }
    v8i a8, b8;
    for (int i = 0; i < 8; ++i) {   // fp8 (e4m3): the all-ones exponent-and-mantissa pattern (NaN) masked out
        a8[i] = operand_word(seed, 36 + i) & 0x77777777;
        b8[i] = operand_word(seed, 44 + i) & 0x77777777;
    }
    float yacc[NT][4];
    v4f facc[NT];
    for (int t = 0; t < NT; ++t) {
        facc[t] = v4f{0.f, 0.f, 0.f, 0.f};
        for (int r = 0; r < 4; ++r) yacc[t][r] = 0.f;
    }
    const v4i zero = {0, 0, 0, 0};
    const float sc = 1.0f + seed * 1e-6f;
    for (int it = 0; it < iters; ++it) {
        if (KIND == 0) {
            v4i d = __builtin_amdgcn_mfma_i32_16x16x64_i8(ai, bi[0], zero, 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                v4i d_nxt = d;
                if (t + 1 < NT) {
                    d_nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(ai, bi[(t + 1) & 3], zero, 0, 0, 0);
                    asm volatile("" : "+v"(d), "+v"(d_nxt));
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (EPI >= 1) yacc[t][r] = fmaf(sc, (float)d[r], yacc[t][r]);
                    if (EPI == 2) bi[(t + 2) & 3][r] = (bi[(t + 2) & 3][r] & 0x0f0f0f0f) + seed;
                }
                if (EPI == 0) asm volatile("" : "+v"(d));
                asm volatile("" : "+v"(yacc[t][0]), "+v"(yacc[t][1]), "+v"(yacc[t][2]), "+v"(yacc[t][3]),
                             "+v"(bi[(t + 2) & 3]));
                d = d_nxt;
            }
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (KIND == 1) facc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh, facc[t], 0, 0, 0);
                if (KIND == 2)
                    facc[t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, facc[t], 0, 0, 0, 0, 0, 0);
            }
        }
    }
    float s = (float)bi[0][0];
    for (int t = 0; t < NT; ++t) s += yacc[t][0] + yacc[t][1] + yacc[t][2] + yacc[t][3] + facc[t][0];
    if (s == 12345.678f) *sink = s;        // keeps the arithmetic alive; practically never taken
    clock.stop(sink);
}

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ v16f mfma6(v8i a, v8i b, v16f c, int scale_a, int scale_b)
{
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 2, 2, 0, scale_a, 0, scale_b);
}

// Two chained fp6 matrix instructions per 32 x 32 tile and group (high and low parts of the int8
// activations), tile t + 1 issued ahead of tile t's multiply-adds; eight tiles per wave.
template <bool EPI>
__global__ __launch_bounds__(512) void peak_fp6_kernel(int iters, int seed, float* sink)
{
    constexpr int NT = 8;
    ClockProbe clock;
    clock.start();
    v8i a0, a1, b[2];
    for (int i = 0; i < 8; ++i) {   // (every 6-bit pattern is a number in e2m3; registers 6 and 7 are not read)
        a0[i] = operand_word(seed, i);
        a1[i] = operand_word(seed, 8 + i);
        b[0][i] = operand_word(seed, 16 + i);
        b[1][i] = operand_word(seed, 24 + i);
    }
    float yacc[NT][16];
    for (int t = 0; t < NT; ++t)
        for (int r = 0; r < 16; ++r) yacc[t][r] = 0.f;
    const v16f z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float sc = 1.0f + seed * 1e-6f;
    v16f d[2];
    d[0] = mfma6(a1, b[0], mfma6(a0, b[0], z, 137, 127), 133, 127);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            asm volatile("" : "+v"(b[(t + 1) & 1]));
            d[(t + 1) & 1] = mfma6(a1, b[(t + 1) & 1], mfma6(a0, b[(t + 1) & 1], z, 137, 127), 133, 127);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (EPI) yacc[t][r] = fmaf(sc, d[t & 1][r], yacc[t][r]);
                else asm volatile("" : "+v"(d[t & 1][r]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = d[0][0];
    for (int t = 0; t < NT; ++t)
        for (int r = 0; r < 16; ++r) s += yacc[t][r];
    if (s == 12345.678f) *sink = s;
    clock.stop(sink);
}

__global__ void empty_kernel() {}

}  // namespace

extern "C" {

int mnnqb_empty(void* stream)
{
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int mnnqb_peak_read(const void* buf, size_t bytes, void* sink, void* stream)
{
    if (!buf || !sink) return -1;
    if (bytes < 16) return -2;
    if (reinterpret_cast<uintptr_t>(buf) & 15u) return -5;
    const int64_t n16 = (int64_t)(bytes / 16);
    const int blocks = num_cus() * 16;
    hipLaunchKernelGGL(peak_read_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(buf), n16, static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int mnnqb_peak_mfma(int kind, int epilogue, int waves_per_simd, int iters, int seed, void* sink, void* stream)
{
    if (!sink) return -1;
    if (iters <= 0 || waves_per_simd < 1 || waves_per_simd > 4) return -2;
    if (kind < 0 || kind > 4 || epilogue < 0 || epilogue > 2 || (kind != 0 && epilogue != 0)) return -3;
    if (kind >= 3 && waves_per_simd > 2) return -3;   // the fp6 loop needs 200 registers
    const dim3 grid((unsigned)num_cus()), block(256u * (unsigned)waves_per_simd);   // one workgroup per CU
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* out = static_cast<float*>(sink);
    if (kind == 0 && epilogue == 0) hipLaunchKernelGGL((peak_mfma_kernel<0, 0>), grid, block, 0, st, iters, seed, out);
    if (kind == 0 && epilogue == 1) hipLaunchKernelGGL((peak_mfma_kernel<0, 1>), grid, block, 0, st, iters, seed, out);
    if (kind == 0 && epilogue == 2) hipLaunchKernelGGL((peak_mfma_kernel<0, 2>), grid, block, 0, st, iters, seed, out);
    if (kind == 1) hipLaunchKernelGGL((peak_mfma_kernel<1, 0>), grid, block, 0, st, iters, seed, out);
    if (kind == 2) hipLaunchKernelGGL((peak_mfma_kernel<2, 0>), grid, block, 0, st, iters, seed, out);
    if (kind == 3) hipLaunchKernelGGL((peak_fp6_kernel<false>), grid, block, 0, st, iters, seed, out);
    if (kind == 4) hipLaunchKernelGGL((peak_fp6_kernel<true>), grid, block, 0, st, iters, seed, out);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

// matrix instructions per iteration and wave (kinds 3, 4: 16 instructions of 32x32x64 = 131072 operations
// each of which only half are the GEMM's - the activations take two fp6 parts)
int mnnqb_peak_mfma_count(void) { return 16; }

}  // extern "C"
