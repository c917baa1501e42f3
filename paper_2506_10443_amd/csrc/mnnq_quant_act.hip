// Run-time activation quantizer (Section 4.2: activations are quantized to int8
// during calculation): per token, symmetric, scale = max|x| / 127.
//
// Compiled with -ffp-contract=off.  The codes are those of the fixed sequence of
// IEEE binary32 operations divide, round-to-nearest-even, clamp; they are computed
// with a multiply by fl(1 / scale) and the division only next to a tie, which gives
// the same integers (quant4_fast) at a fraction of the vector instructions.
#include "mnnq_common.h"

namespace mnnq {

namespace {

constexpr int kQThreads = 256;

__global__ __launch_bounds__(kQThreads) void quant_act_kernel(const float* __restrict__ x, int64_t K,
                                                              int8_t* __restrict__ xq,
                                                              float* __restrict__ sx,
                                                              int32_t* __restrict__ xsum)
{
    __shared__ float s_part[kQThreads / 64];
    const int64_t m = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t K4 = K / 4;  // a multiple of 16: teams of 16 lanes cover whole groups
    const float4* xr = reinterpret_cast<const float4*>(x + m * K);
    // With few rows (decode) a row is split over gridDim.y workgroups: each finds the
    // row maximum itself and quantizes its own slice of the row.
    const int64_t per = (K4 + gridDim.y - 1) / gridDim.y;
    const int64_t per16 = (per + 15) / 16 * 16;          // slices hold whole groups
    const int64_t i0 = per16 * blockIdx.y;
    const int64_t i1 = (i0 + per16 < K4) ? i0 + per16 : K4;

    float amax = 0.0f;
    for (int64_t i = tid; i < K4; i += kQThreads) {
        const float4 v = xr[i];
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    amax = wave_max_nonneg(amax);
    if ((tid & 63) == 0) s_part[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));

    const bool zero_row = (amax == 0.0f);
    const float scale = zero_row ? 0.0f : amax / 127.0f;
    if (tid == 0 && blockIdx.y == 0) sx[m] = scale;

    uint32_t* out = reinterpret_cast<uint32_t*>(xq + m * K);
    const int64_t G = K / kGroup;
    const float inv = zero_row ? 0.0f : 1.0f / scale;
    const float lim = quant_fast_limit(scale, inv);
    for (int64_t i = i0 + tid; i < i1; i += kQThreads) {
        int codes = 0;
        if (!zero_row) codes = quant4_fast(xr[i], scale, inv, lim);
        out[i] = (uint32_t)codes;
        if (xsum) {
            const int s = row_sum16(__builtin_amdgcn_sdot4(codes, 0x01010101, 0, false));
            if ((tid & 15) == 0) xsum[m * G + i / 16] = s;
        }
    }
}

// Many rows (prefill): the row is held in registers between the maximum and the
// quantization, so it crosses the memory system once and all of a thread's loads
// are in flight together.  NV float4 per thread; K <= NV * 4 * kQThreads.
template <int NV>
__global__ __launch_bounds__(kQThreads) void quant_act_rows_kernel(const float* __restrict__ x, int64_t K,
                                                                   int8_t* __restrict__ xq,
                                                                   float* __restrict__ sx,
                                                                   int32_t* __restrict__ xsum)
{
    __shared__ float s_part[kQThreads / 64];
    const int64_t m = blockIdx.x;
    const int tid = threadIdx.x;
    const int K4 = (int)(K / 4);
    const float4* xr = reinterpret_cast<const float4*>(x + m * K);

    float4 v[NV];
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = tid + j * kQThreads;
        v[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (i < K4) v[j] = xr[i];
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[j].x), fabsf(v[j].y)), fmaxf(fabsf(v[j].z), fabsf(v[j].w))));
    }
    amax = wave_max_nonneg(amax);
    if ((tid & 63) == 0) s_part[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));

    const bool zero_row = (amax == 0.0f);
    const float scale = zero_row ? 0.0f : amax / 127.0f;
    if (tid == 0) sx[m] = scale;

    uint32_t* out = reinterpret_cast<uint32_t*>(xq + m * K);
    const int64_t G = K / kGroup;
    const float inv = zero_row ? 0.0f : 1.0f / scale;
    const float lim = quant_fast_limit(scale, inv);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = tid + j * kQThreads;
        int codes = 0;
        if (!zero_row) codes = quant4_fast(v[j], scale, inv, lim);
        if (i < K4) out[i] = (uint32_t)codes;
        if (xsum) {
            // K4 is a multiple of 16, so a team of 16 lanes is inside the row or outside it as a whole
            const int s = row_sum16(__builtin_amdgcn_sdot4(codes, 0x01010101, 0, false));
            if ((tid & 15) == 0 && i < K4) xsum[m * G + i / 16] = s;
        }
    }
}

}  // namespace

int launch_quant_act(const float* x, int64_t M, int64_t K, int8_t* xq, float* sx, int32_t* xsum,
                     hipStream_t st)
{
    // Decode-sized calls are latency bound: spread a row over several workgroups.
    unsigned slices = 1;
    if (M <= 16) {
        slices = (unsigned)((K / 4 + kQThreads - 1) / kQThreads);
        if (slices > 32) slices = 32;
    }
    if (M > 16 && K <= 20 * 4 * kQThreads) {
        const int nv = (int)((K / 4 + kQThreads - 1) / kQThreads);
#define MNNQ_ROWS(NV)                                                                                          \
    if (nv <= NV) {                                                                                            \
        hipLaunchKernelGGL(quant_act_rows_kernel<NV>, dim3((unsigned)M), dim3(kQThreads), 0, st, x, K, xq, sx, \
                           xsum);                                                                              \
        MNNQ_HIP_TRY(hipGetLastError());                                                                       \
        return MNNQ_OK;                                                                                        \
    }
        MNNQ_ROWS(2) MNNQ_ROWS(4) MNNQ_ROWS(8) MNNQ_ROWS(12) MNNQ_ROWS(20)
#undef MNNQ_ROWS
    }
    hipLaunchKernelGGL(quant_act_kernel, dim3((unsigned)M, slices), dim3(kQThreads), 0, st, x, K, xq, sx, xsum);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace mnnq
