// Load-time step: quantize fp32 weights to asymmetric int4 (Section 4.2, Eq. 1,
// groups of 64 along K; with an integer zero point or, as the equation is
// printed, with the group minimum as a float offset) and store them in the chunk layout
// described in mnnq_common.h; plus the inverse view used by tests and export,
// and the import of already quantized weights into the same layout.
//
// This file is compiled with -ffp-contract=off: the quantizer is a fixed
// sequence of IEEE binary32 operations (subtract, divide, round-to-nearest-even,
// add, clamp) and must not be fused.
#include "mnnq_common.h"

namespace mnnq {

namespace {

constexpr int kTeam = 16;           // lanes per (row, group): 16 x float4 = 64 weights
constexpr int kPackThreads = 256;   // 16 teams per workgroup

// Stores one quantization group into the chunk layout.  Called by the 16 lanes of a
// team; lane li holds the codes c0..c3 (each 0..15) of k = 4 li .. 4 li + 3 of group g
// of the packed reduction axis.
__device__ __forceinline__ void store_group(uint8_t* __restrict__ packed, const Layout& L, int64_t n, int64_t g,
                                            int li, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            float scale, float mn, float zero)
{
    // Lane li holds codes j = 4 (li % 4) .. +3 of k-block kb = li / 4.  Codes
    // j % 8 < 4 go to low nibbles, the others to high nibbles of the same bytes.
    uint32_t v = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
    if (li & 1) v <<= 4;
    v |= __shfl_xor(v, 1, kTeam);

    const int64_t t = n / kTileN;
    const int r = (int)(n % kTileN);
    const int64_t c = g / 2;
    const int half = (int)(g & 1);
    const int kb = li / 4;
    const int d = (li % 4) / 2;
    const int64_t chunk = t * L.C + c;
    uint32_t* slot = reinterpret_cast<uint32_t*>(packed + chunk * kChunkBytes + (16 * kb + r) * 16);
    float* sc = reinterpret_cast<float*>(packed + L.scales_off()) + (chunk * 16 + r) * 2;
    uint8_t* zp = packed + L.zeros_off() + (chunk * 16 + r) * 2;
    float* mp = reinterpret_cast<float*>(packed + L.zeros_off()) + (chunk * 16 + r) * 2;
    if ((li & 1) == 0) slot[half * 2 + d] = v;
    if (li == 0) {
        sc[half] = scale;
        if (L.minf) mp[half] = mn;
        else zp[half] = (uint8_t)zero;
    }
    // Odd number of groups: the second half of the last chunk is padding that
    // contributes nothing (codes 0, scale 0, zero / minimum 0).
    if ((L.G & 1) && g == L.G - 1) {
        if ((li & 1) == 0) slot[2 + d] = 0u;
        if (li == 0) {
            sc[1] = 0.0f;
            if (L.minf) mp[1] = 0.0f;
            else zp[1] = 0;
        }
    }
}

// int4 forms.  A workgroup takes kPackChunks consecutive chunks of the layout (16 rows x 128 weights each):
// team r (16 lanes, one float4 each) quantizes the two groups of row 16 t + r, the chunk images are put
// together in LDS in the layout's lane order, and the workgroup stores them - codes, scales, zero points or
// minima - as whole consecutive kilobytes (Section 5.1: consecutive lanes on consecutive addresses; the
// one-group-per-team form before this one wrote 8 bytes here and 8 bytes a kilobyte further on, and the
// memory system wrote 2.4 times the bytes).  All loads are issued before the first is used.
constexpr int kPackChunks = 4;

__global__ __launch_bounds__(kPackThreads) void pack_kernel(const float* __restrict__ W, Layout L,
                                                            uint8_t* __restrict__ packed)
{
    __shared__ __align__(16) uint32_t img[kPackChunks * 256];   // codes: 64 lanes x 16 bytes per chunk
    __shared__ float sc_s[kPackChunks * 32], mn_s[kPackChunks * 32];
    __shared__ uint8_t z_s[kPackChunks * 32];
    const int tid = threadIdx.x;
    const int r = tid / kTeam, li = tid % kTeam;
    const int64_t chunk0 = (int64_t)blockIdx.x * kPackChunks;
    const int64_t n_chunks = L.T * L.C;
    const bool minf = L.minf;

    float4 w[kPackChunks][2];
#pragma unroll
    for (int i = 0; i < kPackChunks; ++i) {
        const int64_t chunk = chunk0 + i;          // uniform over the workgroup
        const int64_t t = chunk / L.C, c = chunk % L.C;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int64_t g = 2 * c + half;
            w[i][half] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (chunk < n_chunks && g < L.G)
                w[i][half] = reinterpret_cast<const float4*>(W + ((t * kTileN + r) * L.G + g) * kGroup)[li];
        }
    }
#pragma unroll
    for (int i = 0; i < kPackChunks; ++i) {
        const int64_t chunk = chunk0 + i;
        const int64_t c = chunk % L.C;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const float4 v4 = w[i][half];
            float scale = 0.0f, zero = 0.0f, mn = 0.0f;
            uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
            // (an odd number of groups: the second half of the last chunk is padding that contributes nothing -
            // codes 0, scale 0, zero / minimum 0)
            if (chunk < n_chunks && 2 * c + half < L.G) {
                mn = fminf(fminf(v4.x, v4.y), fminf(v4.z, v4.w));
                float mx = fmaxf(fmaxf(v4.x, v4.y), fmaxf(v4.z, v4.w));
#pragma unroll
                for (int o = 1; o < kTeam; o <<= 1) {
                    mn = fminf(mn, __shfl_xor(mn, o, kTeam));
                    mx = fmaxf(mx, __shfl_xor(mx, o, kTeam));
                }
                if (!minf) {
                    // Integer zero point: a group that does not straddle zero gets its range widened to contain it.
                    mn = fminf(mn, 0.0f);
                    mx = fmaxf(mx, 0.0f);
                }
                scale = 1.0f;
                if (mx != mn) {
                    scale = (mx - mn) / 15.0f;
                    if (minf) {
                        // Eq. 1 as printed: the minimum is subtracted before the division.
                        c0 = (uint32_t)fminf(fmaxf(rintf((v4.x - mn) / scale), 0.0f), 15.0f);
                        c1 = (uint32_t)fminf(fmaxf(rintf((v4.y - mn) / scale), 0.0f), 15.0f);
                        c2 = (uint32_t)fminf(fmaxf(rintf((v4.z - mn) / scale), 0.0f), 15.0f);
                        c3 = (uint32_t)fminf(fmaxf(rintf((v4.w - mn) / scale), 0.0f), 15.0f);
                    } else {
                        zero = rintf((-mn) / scale);
                        c0 = (uint32_t)fminf(fmaxf(rintf(v4.x / scale) + zero, 0.0f), 15.0f);
                        c1 = (uint32_t)fminf(fmaxf(rintf(v4.y / scale) + zero, 0.0f), 15.0f);
                        c2 = (uint32_t)fminf(fmaxf(rintf(v4.z / scale) + zero, 0.0f), 15.0f);
                        c3 = (uint32_t)fminf(fmaxf(rintf(v4.w / scale) + zero, 0.0f), 15.0f);
                    }
                }
            }
            // Lane li holds codes j = 4 (li % 4) .. +3 of k-block kb = li / 4.  Codes j % 8 < 4 go to low
            // nibbles, the others to high nibbles of the same bytes.
            uint32_t v = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
            if (li & 1) v <<= 4;
            v |= __shfl_xor(v, 1, kTeam);
            const int kb = li / 4, d = (li % 4) / 2;
            if ((li & 1) == 0) img[i * 256 + (16 * kb + r) * 4 + half * 2 + d] = v;
            if (li == 0) {
                sc_s[i * 32 + r * 2 + half] = scale;
                mn_s[i * 32 + r * 2 + half] = mn;
                z_s[i * 32 + r * 2 + half] = (uint8_t)zero;
            }
        }
    }
    __syncthreads();
    // kPackChunks consecutive chunks are consecutive in all three arrays of the layout
    const int live = (int)((n_chunks - chunk0 < kPackChunks) ? (n_chunks - chunk0) : kPackChunks);
    if (tid < live * 64) reinterpret_cast<uint4*>(packed + chunk0 * kChunkBytes)[tid] = reinterpret_cast<const uint4*>(img)[tid];
    if (tid < live * 32) {
        (reinterpret_cast<float*>(packed + L.scales_off()) + chunk0 * 32)[tid] = sc_s[tid];
        if (minf) (reinterpret_cast<float*>(packed + L.zeros_off()) + chunk0 * 32)[tid] = mn_s[tid];
        else (packed + L.zeros_off() + chunk0 * 32)[tid] = z_s[tid];
    }
}

// Byte form of int8 weights (Layout::native8): the 16 bytes of row n, group g, k-block kb.
__device__ __forceinline__ size_t native8_codes_off(const Layout& L, int64_t n, int64_t g, int kb)
{
    const int64_t chunk = (n / kTileN) * L.C + g / 2;
    return (size_t)chunk * (2 * kChunkBytes) + (size_t)(g & 1) * kChunkBytes + (16 * kb + (int)(n % kTileN)) * 16;
}

// Index of the per-group parameters (scale, zero / minimum) of group g, row n.
__device__ __forceinline__ int64_t param_index(const Layout& L, int64_t n, int64_t g)
{
    return (((n / kTileN) * L.C + g / 2) * 16 + n % kTileN) * 2 + (g & 1);
}

// int8 weights: Eq. 1 with clip range 0..255 and a float minimum, stored as two 4-bit
// planes along the doubled reduction axis (see Layout): group g holds the high nibbles
// with step 16 s and the minimum, group G8 + g the low nibbles with step s and minimum 0;
// or, in the byte form, as the bytes q8 - 128 with step s and the minimum.
__global__ __launch_bounds__(kPackThreads) void pack8_kernel(const float* __restrict__ W, Layout L,
                                                             uint8_t* __restrict__ packed)
{
    const int64_t team = (int64_t)blockIdx.x * (kPackThreads / kTeam) + threadIdx.x / kTeam;
    const int li = threadIdx.x % kTeam;
    const int64_t G8 = L.Kx / kGroup;
    if (team >= L.N * G8) return;
    const int64_t n = team / G8;
    const int64_t g = team % G8;

    const float4 w = reinterpret_cast<const float4*>(W + team * kGroup)[li];
    float mn = fminf(fminf(w.x, w.y), fminf(w.z, w.w));
    float mx = fmaxf(fmaxf(w.x, w.y), fmaxf(w.z, w.w));
#pragma unroll
    for (int o = 1; o < kTeam; o <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, o, kTeam));
        mx = fmaxf(mx, __shfl_xor(mx, o, kTeam));
    }
    float step = 1.0f;
    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
    if (mx != mn) {
        step = (mx - mn) / 255.0f;
        c0 = (uint32_t)fminf(fmaxf(rintf((w.x - mn) / step), 0.0f), 255.0f);
        c1 = (uint32_t)fminf(fmaxf(rintf((w.y - mn) / step), 0.0f), 255.0f);
        c2 = (uint32_t)fminf(fmaxf(rintf((w.z - mn) / step), 0.0f), 255.0f);
        c3 = (uint32_t)fminf(fmaxf(rintf((w.w - mn) / step), 0.0f), 255.0f);
    }
    if (L.native8) {
        // lane li holds k = 4 li .. 4 li + 3: dword li % 4 of k-block li / 4
        const uint32_t v = (c0 | (c1 << 8) | (c2 << 16) | (c3 << 24)) ^ 0x80808080u;
        *reinterpret_cast<uint32_t*>(packed + native8_codes_off(L, n, g, li / 4) + (li % 4) * 4) = v;
        if (li == 0) {
            reinterpret_cast<float*>(packed + L.scales_off())[param_index(L, n, g)] = step;
            reinterpret_cast<float*>(packed + L.zeros_off())[param_index(L, n, g)] = mn;
        }
        return;
    }
    store_group(packed, L, n, g, li, c0 >> 4, c1 >> 4, c2 >> 4, c3 >> 4, 16.0f * step, mn, 0.0f);
    store_group(packed, L, n, G8 + g, li, c0 & 15u, c1 & 15u, c2 & 15u, c3 & 15u, step, 0.0f, 0.0f);
}

// 16 codes (one per byte) of k-block kb of group g of the packed axis, row n.
__device__ __forceinline__ uint4 read_codes(const uint8_t* __restrict__ packed, const Layout& L, int64_t n, int64_t g,
                                            int kb)
{
    const int64_t chunk = (n / kTileN) * L.C + g / 2;
    const int r = (int)(n % kTileN);
    const uint2 w = *reinterpret_cast<const uint2*>(packed + chunk * kChunkBytes + (16 * kb + r) * 16 + (g & 1) * 8);
    uint4 o;
    o.x = w.x & 0x0f0f0f0fu;
    o.y = (w.x >> 4) & 0x0f0f0f0fu;
    o.z = w.y & 0x0f0f0f0fu;
    o.w = (w.y >> 4) & 0x0f0f0f0fu;
    return o;
}


__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                     uint8_t* __restrict__ q, float* __restrict__ scale,
                                                     void* __restrict__ zero)
{
    // One thread per (row, group of the weight matrix, k-block): 16 codes.
    const int64_t G = L.Kx / kGroup;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= L.N * G * 4) return;
    const int kb = (int)(idx % 4);
    const int64_t g = (idx / 4) % G;
    const int64_t n = idx / (4 * G);
    if (L.native8) {   // byte form: q8 - 128 as stored, step and minimum of the group itself
        if (q) {
            uint4 o = *reinterpret_cast<const uint4*>(packed + native8_codes_off(L, n, g, kb));
            o.x ^= 0x80808080u; o.y ^= 0x80808080u; o.z ^= 0x80808080u; o.w ^= 0x80808080u;
            *reinterpret_cast<uint4*>(q + n * L.Kx + g * kGroup + 16 * kb) = o;
        }
        if (kb == 0) {
            if (scale) scale[n * G + g] = reinterpret_cast<const float*>(packed + L.scales_off())[param_index(L, n, g)];
            if (zero) static_cast<float*>(zero)[n * G + g] =
                          reinterpret_cast<const float*>(packed + L.zeros_off())[param_index(L, n, g)];
        }
        return;
    }
    const bool w8 = (L.mode == MNNQ_W8_MIN_FLOAT);   // high nibbles in group g, low nibbles in group G + g
    if (q) {
        uint4 o = read_codes(packed, L, n, g, kb);
        if (w8) {
            const uint4 lo = read_codes(packed, L, n, G + g, kb);
            o.x = (o.x << 4) | lo.x; o.y = (o.y << 4) | lo.y; o.z = (o.z << 4) | lo.z; o.w = (o.w << 4) | lo.w;
        }
        *reinterpret_cast<uint4*>(q + n * L.Kx + g * kGroup + 16 * kb) = o;
    }
    if (kb == 0) {
        const float* sc = reinterpret_cast<const float*>(packed + L.scales_off());
        // int8: the low plane carries the step itself, the high plane the minimum
        if (scale) scale[n * G + g] = sc[param_index(L, n, w8 ? G + g : g)];
        if (zero) {
            if (L.minf)
                static_cast<float*>(zero)[n * G + g] =
                    reinterpret_cast<const float*>(packed + L.zeros_off())[param_index(L, n, g)];
            else
                static_cast<uint8_t*>(zero)[n * G + g] = (packed + L.zeros_off())[param_index(L, n, g)];
        }
    }
}

// Writes 16 codes (one per byte, 0..15) of k-block kb of group g of the packed axis and,
// from the thread with kb == 0, the group's parameters.
__device__ __forceinline__ void write_codes(uint8_t* __restrict__ packed, const Layout& L, int64_t n, int64_t g,
                                            int kb, uint4 o, float scale, float mn, uint8_t z)
{
    const int64_t chunk = (n / kTileN) * L.C + g / 2;
    const int r = (int)(n % kTileN);
    const int half = (int)(g & 1);
    uint2 w;
    w.x = (o.x & 0x0f0f0f0fu) | ((o.y & 0x0f0f0f0fu) << 4);
    w.y = (o.z & 0x0f0f0f0fu) | ((o.w & 0x0f0f0f0fu) << 4);
    uint2* slot = reinterpret_cast<uint2*>(packed + chunk * kChunkBytes + (16 * kb + r) * 16);
    slot[half] = w;
    float* sc = reinterpret_cast<float*>(packed + L.scales_off()) + (chunk * 16 + r) * 2;
    uint8_t* zp = packed + L.zeros_off() + (chunk * 16 + r) * 2;
    float* mp = reinterpret_cast<float*>(packed + L.zeros_off()) + (chunk * 16 + r) * 2;
    if (kb == 0) {
        sc[half] = scale;
        if (L.minf) mp[half] = mn;
        else zp[half] = z > 15 ? (uint8_t)15 : z;
    }
    if ((L.G & 1) && g == L.G - 1) {   // padding group of an odd G
        slot[1] = make_uint2(0u, 0u);
        if (kb == 0) {
            sc[1] = 0.0f;
            if (L.minf) mp[1] = 0.0f;
            else zp[1] = 0;
        }
    }
}

// Import of weights that are already quantized (Section 4.2: quantized weights,
// e.g. from GPTQ, can be imported): canonical arrays -> chunk layout, the exact
// inverse of unpack_kernel.  One thread per (row, group, k-block).  int4 codes are
// taken modulo 16, zero points above 15 are stored as 15.
__global__ __launch_bounds__(256) void repack_kernel(const uint8_t* __restrict__ q, const float* __restrict__ scale,
                                                     const void* __restrict__ zero, Layout L,
                                                     uint8_t* __restrict__ packed)
{
    const int64_t G = L.Kx / kGroup;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= L.N * G * 4) return;
    const int kb = (int)(idx % 4);
    const int64_t g = (idx / 4) % G;
    const int64_t n = idx / (4 * G);
    const uint4 o = *reinterpret_cast<const uint4*>(q + n * L.Kx + g * kGroup + 16 * kb);
    const float s = scale[n * G + g];
    if (L.native8) {
        uint4 v = o;
        v.x ^= 0x80808080u; v.y ^= 0x80808080u; v.z ^= 0x80808080u; v.w ^= 0x80808080u;
        *reinterpret_cast<uint4*>(packed + native8_codes_off(L, n, g, kb)) = v;
        if (kb == 0) {
            reinterpret_cast<float*>(packed + L.scales_off())[param_index(L, n, g)] = s;
            reinterpret_cast<float*>(packed + L.zeros_off())[param_index(L, n, g)] = static_cast<const float*>(zero)[n * G + g];
        }
    } else if (L.mode == MNNQ_W8_MIN_FLOAT) {
        const float mn = static_cast<const float*>(zero)[n * G + g];
        uint4 hi;
        hi.x = o.x >> 4; hi.y = o.y >> 4; hi.z = o.z >> 4; hi.w = o.w >> 4;
        write_codes(packed, L, n, g, kb, hi, 16.0f * s, mn, 0);
        write_codes(packed, L, n, G + g, kb, o, s, 0.0f, 0);
    } else if (L.minf) {
        write_codes(packed, L, n, g, kb, o, s, static_cast<const float*>(zero)[n * G + g], 0);
    } else {
        write_codes(packed, L, n, g, kb, o, s, 0.0f, static_cast<const uint8_t*>(zero)[n * G + g]);
    }
}

}  // namespace

int launch_repack(const uint8_t* q, const float* scale, const void* zero, const Layout& L, uint8_t* packed,
                  hipStream_t st)
{
    const int64_t total = L.N * (L.Kx / kGroup) * 4;
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(repack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, q, scale, zero, L, packed);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

int launch_pack(const float* W, const Layout& L, uint8_t* packed, hipStream_t st)
{
    const int64_t teams = L.N * (L.Kx / kGroup);
    const int64_t blocks = (teams + (kPackThreads / kTeam) - 1) / (kPackThreads / kTeam);
    if (L.mode == MNNQ_W8_MIN_FLOAT)
        hipLaunchKernelGGL(pack8_kernel, dim3((unsigned)blocks), dim3(kPackThreads), 0, st, W, L, packed);
    else
        hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((L.T * L.C + kPackChunks - 1) / kPackChunks)), dim3(kPackThreads), 0, st,
                           W, L, packed);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

int launch_unpack(const uint8_t* packed, const Layout& L, uint8_t* q, float* scale, void* zero,
                  hipStream_t st)
{
    const int64_t total = L.N * (L.Kx / kGroup) * 4;
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, packed, L, q, scale, zero);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace mnnq
