// Decode step (one token): W4A8 GEMV, memory-bound (Section 2.1).  The weights
// are streamed exactly once with one 128-bit load per lane per chunk, lanes
// contiguous in memory (the rule of Section 5.1 for GPUs: vectorised 128-bit
// loads, consecutive work items on consecutive addresses), dequantized in
// registers and contracted with v_dot4_i32_i8.
//
//   y[n] = sx * sum_g scale[n,g] * sum_{k in g} xq[k] * (q[n,k] - zero[n,g]) (+ bias[n])
//
// Work split: a wave owns one row tile (16 rows) and a contiguous range of
// chunks; KSPLIT waves of a workgroup share a row tile and their partial sums
// are added in a fixed order through LDS, so results are run-to-run identical.
#include "mnnq_common.h"

#include <stdlib.h>

namespace mnnq {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ChunkRegs {
    u32x4 w;      // 32 codes: .x,.y group 2c ; .z,.w group 2c+1
    float2 s;     // scales of the lane's row for both groups
    uint32_t z;   // zeros, low byte group 2c, next byte group 2c+1
};

__device__ __forceinline__ ChunkRegs load_chunk(const u32x4* wp, const float2* sp, const uint16_t* zp,
                                                int64_t i)
{
    ChunkRegs r;
    r.w = __builtin_nontemporal_load(wp + i * 64);
    r.s = sp[i * 16];
    r.z = zp[i * 16];
    return r;
}

__device__ __forceinline__ int dot16(uint32_t wa, uint32_t wb, const int4& x)
{
    int d = __builtin_amdgcn_sdot4((int)(wa & 0x0f0f0f0fu), x.x, 0, false);
    d = __builtin_amdgcn_sdot4((int)((wa >> 4) & 0x0f0f0f0fu), x.y, d, false);
    d = __builtin_amdgcn_sdot4((int)(wb & 0x0f0f0f0fu), x.z, d, false);
    d = __builtin_amdgcn_sdot4((int)((wb >> 4) & 0x0f0f0f0fu), x.w, d, false);
    return d;
}

// LDS image of the activation row: K int8 padded with zeros to C*128 bytes,
// followed by the sums of every 16-byte block, stored as [c][kb][half].
__device__ __forceinline__ void stage_x(const int8_t* __restrict__ xq, int64_t K, int64_t C,
                                        int4* lds_x, int* lds_xs, int tid, int nthreads)
{
    const int64_t units = C * 8;       // 16-byte units, padded
    const int64_t valid = K / 16;
    for (int64_t u = tid; u < units; u += nthreads) {
        int4 v = make_int4(0, 0, 0, 0);
        if (u < valid) v = reinterpret_cast<const int4*>(xq)[u];
        lds_x[u] = v;
        int s = __builtin_amdgcn_sdot4(v.x, 0x01010101, 0, false);
        s = __builtin_amdgcn_sdot4(v.y, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.z, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.w, 0x01010101, s, false);
        const int64_t c = u / 8;
        const int half = (int)(u % 8) / 4;
        const int kb = (int)(u % 4);
        lds_xs[c * 8 + kb * 2 + half] = s;
    }
}

template <int WAVES, int KSPLIT, int UNROLL, bool ACC>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                            const int8_t* __restrict__ xq,
                                                            const float* __restrict__ sx,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ y,
                                                            int32_t* __restrict__ acc)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int64_t C = L.C;
    int4* lds_x = reinterpret_cast<int4*>(smem);
    int* lds_xs = reinterpret_cast<int*>(smem + C * 128);
    float* lds_part = reinterpret_cast<float*>(smem + C * 160);  // [WAVES][16]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane & 15;
    const int kb = lane >> 4;
    constexpr int TILES_PER_WG = WAVES / KSPLIT;
    const int64_t tile = (int64_t)blockIdx.x * TILES_PER_WG + wave / KSPLIT;
    const int ks = wave % KSPLIT;
    const int64_t m = ACC ? blockIdx.y : 0;
    const bool active = tile < L.T;

    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const u32x4* wp = reinterpret_cast<const u32x4*>(packed) + (tile * C + c0) * 64 + lane;
    const float2* sp = reinterpret_cast<const float2*>(packed + L.scales_off()) + (tile * C + c0) * 16 + row;
    const uint16_t* zp = reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) + (tile * C + c0) * 16 + row;
    const int64_t n_chunks = active ? (c1 - c0) : 0;

    // Start the weight stream before the activation row is staged: the first
    // batch does not depend on x.
    ChunkRegs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        if (u < n_chunks) cur[u] = load_chunk(wp, sp, zp, u);
        else cur[u] = ChunkRegs{};
    }

    stage_x(xq + m * L.K, L.K, C, lds_x, lds_xs, tid, WAVES * 64);
    __syncthreads();

    float accf = 0.0f;
    for (int64_t i = 0; i < n_chunks; i += UNROLL) {
        ChunkRegs nxt[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (i + UNROLL + u < n_chunks) nxt[u] = load_chunk(wp, sp, zp, i + UNROLL + u);
            else nxt[u] = ChunkRegs{};
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (i + u < n_chunks) {
                const int64_t c = c0 + i + u;
                const int4 xa = lds_x[c * 8 + kb];
                const int4 xb = lds_x[c * 8 + 4 + kb];
                const int2 xs = *reinterpret_cast<const int2*>(lds_xs + c * 8 + kb * 2);
                const ChunkRegs& r = cur[u];
                int i0 = dot16(r.w.x, r.w.y, xa) - (int)(r.z & 0xffu) * xs.x;
                int i1 = dot16(r.w.z, r.w.w, xb) - (int)(r.z >> 8) * xs.y;
                if (ACC) {
                    i0 += __shfl_xor(i0, 16, 64); i0 += __shfl_xor(i0, 32, 64);
                    i1 += __shfl_xor(i1, 16, 64); i1 += __shfl_xor(i1, 32, 64);
                    if (kb == 0) {
                        int32_t* o = acc + (m * L.N + tile * kTileN + row) * L.G;
                        o[2 * c] = i0;
                        if (2 * c + 1 < L.G) o[2 * c + 1] = i1;
                    }
                } else {
                    accf = fmaf(r.s.x, (float)i0, accf);
                    accf = fmaf(r.s.y, (float)i1, accf);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) cur[u] = nxt[u];
    }
    if (ACC) return;

    // Sum over the four k-blocks of the row, then over the KSPLIT waves.
    accf += __shfl_xor(accf, 16, 64);
    accf += __shfl_xor(accf, 32, 64);
    if (KSPLIT > 1) {
        if (kb == 0) lds_part[wave * 16 + row] = accf;
        __syncthreads();
        if (ks != 0) return;
        accf = lds_part[wave * 16 + row];
#pragma unroll
        for (int j = 1; j < KSPLIT; ++j) accf += lds_part[(wave + j) * 16 + row];
    }
    if (active && kb == 0) {
        const int64_t n = tile * kTileN + row;
        float r = accf * sx[0];
        if (bias) r += bias[n];
        y[n] = r;
    }
}

template <int WAVES, int KSPLIT, int UNROLL, bool ACC>
int launch_cfg(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
               const float* bias, float* y, int32_t* acc, hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    const size_t smem = (size_t)L.C * 160 + WAVES * 16 * sizeof(float);
    hipLaunchKernelGGL((decode_kernel<WAVES, KSPLIT, UNROLL, ACC>), dim3((unsigned)blocks, (unsigned)M),
                       dim3(WAVES * 64), smem, st, packed, L, xq, sx, bias, y, acc);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

// Waves that share one row tile.  Enough waves to keep every CU streaming
// (about 8 per CU on 256 CUs), but at least two chunks per wave.
int pick_ksplit(const Layout& L)
{
    if (const char* e = getenv("MNNQ_DECODE_KSPLIT")) {
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16) return v;
    }
    int ks = 1;
    while (ks < 16 && L.T * ks < 2048 && L.C / (ks * 2) >= 2) ks *= 2;
    return ks;
}

}  // namespace

int launch_decode(const uint8_t* packed, const Layout& L, const int8_t* xq, const float* sx,
                  const float* bias, float* y, hipStream_t st)
{
    switch (pick_ksplit(L)) {
        case 1:  return launch_cfg<4, 1, 4, false>(packed, L, 1, xq, sx, bias, y, nullptr, st);
        case 2:  return launch_cfg<4, 2, 4, false>(packed, L, 1, xq, sx, bias, y, nullptr, st);
        case 4:  return launch_cfg<4, 4, 4, false>(packed, L, 1, xq, sx, bias, y, nullptr, st);
        case 8:  return launch_cfg<8, 8, 4, false>(packed, L, 1, xq, sx, bias, y, nullptr, st);
        default: return launch_cfg<16, 16, 4, false>(packed, L, 1, xq, sx, bias, y, nullptr, st);
    }
}

int launch_decode_acc(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, int32_t* acc,
                      hipStream_t st)
{
    // Same inner loop as the decode kernel, one grid row per token.
    return launch_cfg<4, 2, 4, true>(packed, L, M, xq, nullptr, nullptr, nullptr, acc, st);
}

}  // namespace mnnq
