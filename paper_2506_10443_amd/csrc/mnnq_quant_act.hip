// Run-time activation quantizer (Section 4.2: activations are quantized to int8
// during calculation): per token, symmetric, scale = max|x| / 127.
//
// Compiled with -ffp-contract=off; the code is a fixed sequence of IEEE
// binary32 operations (divide, round-to-nearest-even, clamp).
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
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
    if ((tid & 63) == 0) s_part[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));

    const bool zero_row = (amax == 0.0f);
    const float scale = zero_row ? 0.0f : amax / 127.0f;
    if (tid == 0 && blockIdx.y == 0) sx[m] = scale;

    uint32_t* out = reinterpret_cast<uint32_t*>(xq + m * K);
    const int64_t G = K / kGroup;
    for (int64_t i = i0 + tid; i < i1; i += kQThreads) {
        int c0 = 0, c1 = 0, c2 = 0, c3 = 0;
        if (!zero_row) {
            const float4 v = xr[i];
            c0 = (int)fminf(fmaxf(rintf(v.x / scale), -127.0f), 127.0f);
            c1 = (int)fminf(fmaxf(rintf(v.y / scale), -127.0f), 127.0f);
            c2 = (int)fminf(fmaxf(rintf(v.z / scale), -127.0f), 127.0f);
            c3 = (int)fminf(fmaxf(rintf(v.w / scale), -127.0f), 127.0f);
        }
        out[i] = (uint32_t)(c0 & 0xff) | ((uint32_t)(c1 & 0xff) << 8) | ((uint32_t)(c2 & 0xff) << 16) |
                 ((uint32_t)(c3 & 0xff) << 24);
        if (xsum) {
            int s = c0 + c1 + c2 + c3;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 16);
            if ((tid & 15) == 0) xsum[m * G + i / 16] = s;
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
    hipLaunchKernelGGL(quant_act_kernel, dim3((unsigned)M, slices), dim3(kQThreads), 0, st, x, K, xq, sx, xsum);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace mnnq
