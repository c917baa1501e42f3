// Prefill (M tokens): W4A8 GEMM on the gfx950 int8 matrix cores, compute-bound
// (Section 2.1).  One v_mfma_i32_16x16x64_i8 contracts exactly one quantization
// group (K = 64) of a 16 x 16 output tile, so with a zero C operand its result
// is the int32 group accumulator I[m, n, g]; the fused epilogue converts it and
// adds scale[n, g] * I to the fp32 running sum:
//
//   y[m,n] = sx[m] * sum_g scale[n,g] * I[m,n,g] (+ bias[n])
//
// Data movement per workgroup and chunk (128 values of K):
//   A (activations, int8): global -> registers -> LDS (double buffered, rows
//     padded to 144 B so that the 128-bit fragment reads are conflict free).
//   B (weights, int4): one 128-bit global load per lane and row tile straight
//     into registers - the chunk layout already is the MFMA B-operand order -
//     then nibbles -> int8 and the zero point is subtracted per byte.
//
// Lane mapping of the 16x16x64 int8 MFMA (A: 16 x 64, B: 64 x 16, D: 16 x 16):
//   A operand: lane l holds row l % 16, 16 consecutive k of block l / 16;
//   B operand: lane l holds column l % 16, the same 16 k of block l / 16;
//   D:         lane l holds column l % 16, rows 4 (l / 16) + r, r = 0..3.
#include "mnnq_common.h"

namespace mnnq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kAStride = 144;  // bytes per LDS row of A: 128 + 16 padding

// q - z per byte for four codes (0..15) in the bytes of v; z4 = z * 0x01010101.
// Setting bit 7 of every byte first keeps the borrow inside its byte.
__device__ __forceinline__ int sub_zero(uint32_t v, uint32_t z4)
{
    return (int)(((v | 0x80808080u) - z4) ^ 0x80808080u);
}

__device__ __forceinline__ v4i unpack_b(uint32_t w0, uint32_t w1, uint32_t z4)
{
    v4i b;
    b.x = sub_zero(w0 & 0x0f0f0f0fu, z4);
    b.y = sub_zero((w0 >> 4) & 0x0f0f0f0fu, z4);
    b.z = sub_zero(w1 & 0x0f0f0f0fu, z4);
    b.w = sub_zero((w1 >> 4) & 0x0f0f0f0fu, z4);
    return b;
}

template <int BM, int BN, int WGM, int WGN, bool ACC>
__global__ __launch_bounds__(WGM * WGN * 64) void prefill_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                                 int64_t M, const int8_t* __restrict__ xq,
                                                                 const float* __restrict__ sx,
                                                                 const float* __restrict__ bias,
                                                                 float* __restrict__ y,
                                                                 int32_t* __restrict__ acc_out,
                                                                 int MT, int NT)
{
    constexpr int THREADS = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int A_UNITS = BM * 8;                 // 16-byte units of one A stage
    constexpr int A_PER_THREAD = A_UNITS / THREADS;
    static_assert(A_UNITS % THREADS == 0, "A tile must split evenly");

    __shared__ __align__(16) uint8_t lds_a[2][BM * kAStride];

    // Workgroups are dealt to the 8 XCDs round-robin by their linear id.  Give
    // each XCD whole columns of output tiles (one weight row block, all token
    // blocks) so that a weight block is fetched into one L2 only.
    const int xcd = blockIdx.x % 8;
    const int seq = blockIdx.x / 8;
    const int tile_m = seq % MT;
    const int tile_n = (seq / MT) * 8 + xcd;
    if (tile_n >= NT) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int col = lane & 15;
    const int kb = lane >> 4;
    const int64_t m0 = (int64_t)tile_m * BM;
    const int64_t C = L.C;

    // B side: TN row tiles of 16 weight rows each.
    const int64_t rt0 = ((int64_t)tile_n * BN + wn * WN) / 16;
    bool b_ok[TN];
    const u32x4* wp[TN];
    const float2* sp[TN];
    const uint16_t* zp[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int64_t rt = rt0 + j;
        b_ok[j] = rt < L.T;
        const int64_t rtc = b_ok[j] ? rt : 0;
        wp[j] = reinterpret_cast<const u32x4*>(packed) + rtc * C * 64 + lane;
        sp[j] = reinterpret_cast<const float2*>(packed + L.scales_off()) + rtc * C * 16 + col;
        zp[j] = reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) + rtc * C * 16 + col;
    }

    u32x4 bw[TN], bw_n[TN];
    float2 bs[TN], bs_n[TN];
    uint32_t bz[TN], bz_n[TN];
    uint4 areg[A_PER_THREAD];

    auto load_a = [&](int64_t c) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            const int u = tid + i * THREADS;
            const int r = u / 8, cu = u % 8;
            const int64_t m = m0 + r;
            const int64_t k = c * 128 + cu * 16;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m < M && k < L.K) v = *reinterpret_cast<const uint4*>(xq + m * L.K + k);
            areg[i] = v;
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            const int u = tid + i * THREADS;
            const int r = u / 8, cu = u % 8;
            *reinterpret_cast<uint4*>(&lds_a[buf][r * kAStride + cu * 16]) = areg[i];
        }
    };
    auto load_b = [&](int64_t c, u32x4* w, float2* s, uint32_t* z) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            w[j] = wp[j][c * 64];
            s[j] = sp[j][c * 16];
            z[j] = zp[j][c * 16];
        }
    };

    float yacc[TM][TN][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) yacc[i][j][r] = 0.0f;

    load_a(0);
    load_b(0, bw, bs, bz);
    store_a(0);

    for (int64_t c = 0; c < C; ++c) {
        const int buf = (int)(c & 1);
        __syncthreads();
        const bool more = c + 1 < C;
        if (more) {
            load_a(c + 1);
            load_b(c + 1, bw_n, bs_n, bz_n);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4i b[TN];
            float sc[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint32_t zz = h ? (bz[j] >> 8) : (bz[j] & 0xffu);
                const uint32_t z4 = zz * 0x01010101u;
                b[j] = h ? unpack_b(bw[j].z, bw[j].w, z4) : unpack_b(bw[j].x, bw[j].y, z4);
                sc[j] = h ? bs[j].y : bs[j].x;
            }
            const int64_t g = 2 * c + h;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int r = wm * WM + i * 16 + col;
                const v4i a = *reinterpret_cast<const v4i*>(&lds_a[buf][r * kAStride + h * 64 + kb * 16]);
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const v4i zero = {0, 0, 0, 0};
                    const v4i d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[j], zero, 0, 0, 0);
                    if (ACC) {
                        if (b_ok[j] && g < L.G) {
                            const int64_t n = (rt0 + j) * 16 + col;
#pragma unroll
                            for (int rr = 0; rr < 4; ++rr) {
                                const int64_t m = m0 + wm * WM + i * 16 + kb * 4 + rr;
                                if (m < M) acc_out[(m * L.N + n) * L.G + g] = d[rr];
                            }
                        }
                    } else {
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
                            yacc[i][j][rr] = fmaf(sc[j], (float)d[rr], yacc[i][j][rr]);
                    }
                }
            }
        }
        if (more) {
            store_a(buf ^ 1);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                bw[j] = bw_n[j];
                bs[j] = bs_n[j];
                bz[j] = bz_n[j];
            }
        }
    }
    if (ACC) return;

#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int64_t m = m0 + wm * WM + i * 16 + kb * 4 + rr;
            if (m >= M) continue;
            const float sxm = sx[m];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (!b_ok[j]) continue;
                const int64_t n = (rt0 + j) * 16 + col;
                float v = yacc[i][j][rr] * sxm;
                if (bias) v += bias[n];
                y[m * L.N + n] = v;
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, bool ACC>
int launch_tiles(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                 const float* bias, float* y, int32_t* acc, hipStream_t st)
{
    const int MT = (int)((M + BM - 1) / BM);
    const int NT = (int)((L.N + BN - 1) / BN);
    const int64_t blocks = (int64_t)MT * ((NT + 7) / 8) * 8;
    hipLaunchKernelGGL((prefill_kernel<BM, BN, WGM, WGN, ACC>), dim3((unsigned)blocks), dim3(WGM * WGN * 64),
                       0, st, packed, L, M, xq, sx, bias, y, acc, MT, NT);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace

int launch_prefill(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                   const float* bias, float* y, int32_t* acc_debug, hipStream_t st)
{
    if (acc_debug)
        return launch_tiles<128, 128, 2, 2, true>(packed, L, M, xq, sx, bias, y, acc_debug, st);
    return launch_tiles<128, 128, 2, 2, false>(packed, L, M, xq, sx, bias, y, nullptr, st);
}

}  // namespace mnnq
