// A few tokens at once (M <= 16): batched or speculative decoding.  The step is
// still memory-bound (Section 2.1), so the weights are streamed exactly once, as in
// the one-token GEMV, and every chunk meets all M activation rows in the matrix
// cores: one v_mfma_i32_16x16x64_i8 per quantization group contracts the 16 weight
// rows of a row tile with up to 16 tokens, which costs the vector ALU no more than
// the one-token dot products do.
//
//   y[m,n] = sx[m] * sum_g scale[n,g] * sum_{k in g} xq[m,k] * (q[n,k] - zero[n,g]) (+ bias[n])
//
// (float-minimum form: sx[m] * sum_g (scale * sum xq q + min * sum xq), the row sums
// from one more MFMA with an all-ones operand.)
//
// Work split as in the GEMV: a wave owns one row tile and a contiguous chunk range,
// KSPLIT waves share a row tile and add their partial sums in a fixed order through
// LDS.  The activations are small (M * K bytes) and stay in L2.  Where 16 rows of them
// fit in LDS (K <= 4096) a workgroup of 16 waves copies them there once, in the order
// the A operand is read (STAGED), and shares them between its row tiles; for longer
// rows each lane loads its A operand - 16 consecutive k of token lane % 16 - straight
// from L2.
//
// MFMA lane mapping (A: 16 x 64 tokens x k, B: 64 x 16 k x weight rows, D: 16 x 16):
//   A: lane l holds token l % 16, k block l / 16;  B: lane l holds weight row l % 16,
//   the same k block - exactly the lane's 8 bytes of the chunk, unpacked;
//   D: lane l holds weight row l % 16, tokens 4 (l / 16) + r, r = 0..3.
#include "mnnq_common.h"

#include <stdlib.h>

namespace mnnq {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

struct SkinnyRegs {
    u32x4 w;       // 32 codes: .x,.y group 2c ; .z,.w group 2c+1
    float2 s;      // scales of the lane's weight row for both groups
    uint32_t z;    // zero points of both groups                       (integer zero point form)
    float2 mn;     // group minima of both groups                      (float minimum form)
    v4i xa, xb;    // the lane's 16 activations of group 2c and of group 2c+1
};

// q - z per byte for four codes in the bytes of v (c4 = 0x80 - z in every byte).
__device__ __forceinline__ int sub_zero(uint32_t v, uint32_t c4)
{
    return (int)((v + c4) ^ 0x80808080u);
}

template <bool MINF>
__device__ __forceinline__ v4i unpack_group(uint32_t w0, uint32_t w1, uint32_t z)
{
    v4i b;
    if (MINF) {
        b.x = (int)(w0 & 0x0f0f0f0fu);
        b.y = (int)((w0 >> 4) & 0x0f0f0f0fu);
        b.z = (int)(w1 & 0x0f0f0f0fu);
        b.w = (int)((w1 >> 4) & 0x0f0f0f0fu);
    } else {
        const uint32_t c4 = 0x80808080u - z * 0x01010101u;
        b.x = sub_zero(w0 & 0x0f0f0f0fu, c4);
        b.y = sub_zero((w0 >> 4) & 0x0f0f0f0fu, c4);
        b.z = sub_zero(w1 & 0x0f0f0f0fu, c4);
        b.w = sub_zero((w1 >> 4) & 0x0f0f0f0fu, c4);
    }
    return b;
}

template <int WAVES, int KSPLIT, int UNROLL, bool PREFETCH, bool MINF, bool STAGED>
__global__ __launch_bounds__(WAVES * 64) void skinny_kernel(const uint8_t* __restrict__ packed, Layout L, int M,
                                                            const int8_t* __restrict__ xq,
                                                            const float* __restrict__ sx,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ y)
{
    extern __shared__ __align__(16) uint8_t smem[];
    float* lds_part = reinterpret_cast<float*>(smem);                         // [wave][r][lane]
    const v4i* lds_a = reinterpret_cast<const v4i*>(smem + WAVES * 4 * 64 * 4);   // STAGED: [C * 8 units][16 tokens]
    const int64_t C = L.C;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane & 15;     // weight row of the B operand and of the results; token of the A operand
    const int kb = lane >> 4;
    constexpr int TILES_PER_WG = WAVES / KSPLIT;
    const int64_t tile = (int64_t)blockIdx.x * TILES_PER_WG + wave / KSPLIT;
    const int ks = wave % KSPLIT;
    const bool active = tile < L.T;
    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const u32x4* wp = reinterpret_cast<const u32x4*>(packed) + (tile * C + c0) * 64 + lane;
    const float2* sp = reinterpret_cast<const float2*>(packed + L.scales_off()) + (tile * C + c0) * 16 + row;
    const void* zp = MINF ? static_cast<const void*>(reinterpret_cast<const float2*>(packed + L.zeros_off()) +
                                                     (tile * C + c0) * 16 + row)
                          : static_cast<const void*>(reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) +
                                                     (tile * C + c0) * 16 + row);
    const int64_t n_chunks = active ? (c1 - c0) : 0;
    // Tokens past M repeat the last one; their results are not stored.
    const int8_t* xrow = xq + (int64_t)(row < M ? row : M - 1) * L.Kx + kb * 16;
    const int64_t Cx = L.Cx;      // chunk c of the packed axis meets chunk c % Cx of the activation row
    const bool odd_tail = (L.G & 1) != 0;   // the last chunk of a row holds one real group only

    auto load = [&](int64_t i) {
        SkinnyRegs r;
        const int64_t c = c0 + i;
        r.w = __builtin_nontemporal_load(wp + i * 64);
        r.s = sp[i * 16];
        if (MINF) {
            r.mn = static_cast<const float2*>(zp)[i * 16];
            r.z = 0;
        } else {
            r.z = static_cast<const uint16_t*>(zp)[i * 16];
            r.mn = make_float2(0.0f, 0.0f);
        }
        if (!STAGED) {
            r.xa = *reinterpret_cast<const v4i*>(xrow + (c % Cx) * 128);
            r.xb = (odd_tail && c == C - 1) ? v4i{0, 0, 0, 0}
                                            : *reinterpret_cast<const v4i*>(xrow + (c % Cx) * 128 + 64);
        } else {
            r.xa = v4i{0, 0, 0, 0};
            r.xb = v4i{0, 0, 0, 0};
        }
        return r;
    };

    SkinnyRegs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        if (u < n_chunks) cur[u] = load(u);
        else cur[u] = SkinnyRegs{};
    }

    if (STAGED) {
        // The weight loads above are in flight; now the whole workgroup copies the 16 token rows
        // (tokens past M repeat the last one, k past K is zero) in units of 16 bytes: unit (ku, m)
        // holds k = 16 ku .. 16 ku + 15 of token m, and lands at index ku * 16 + m.
        v4i* dst = reinterpret_cast<v4i*>(smem + WAVES * 4 * 64 * 4);
        const int units = (int)C * 8 * 16;
        const int valid_ku = (int)(L.K / 16);
        const int row_ku = (int)(L.Kx / 16);
        for (int u = tid; u < units; u += WAVES * 64) {
            const int m = u & 15, ku = u >> 4;
            v4i v = {0, 0, 0, 0};
            if (ku < valid_ku)
                v = *reinterpret_cast<const v4i*>(xq + (int64_t)(m < M ? m : M - 1) * L.Kx + (ku % row_ku) * 16);
            dst[u] = v;
        }
        __syncthreads();
    }

    const v4i zero = {0, 0, 0, 0};
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t i = 0; i < n_chunks; i += UNROLL) {
        SkinnyRegs nxt[PREFETCH ? UNROLL : 1];
        if (PREFETCH) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                if (i + UNROLL + u < n_chunks) nxt[u] = load(i + UNROLL + u);
                else nxt[u] = SkinnyRegs{};
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (i + u < n_chunks) {
                const SkinnyRegs& r = cur[u];
                v4i xa = r.xa, xb = r.xb;
                if (STAGED) {
                    const int64_t c = c0 + i + u;
                    xa = lds_a[((c * 8 + kb) << 4) + row];
                    xb = lds_a[((c * 8 + 4 + kb) << 4) + row];
                }
                const v4i b0 = unpack_group<MINF>(r.w.x, r.w.y, r.z & 0xffu);
                const v4i b1 = unpack_group<MINF>(r.w.z, r.w.w, r.z >> 8);
                const v4i d0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, b0, zero, 0, 0, 0);
                const v4i d1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xb, b1, zero, 0, 0, 0);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    acc[rr] = fmaf(r.s.x, (float)d0[rr], acc[rr]);
                    acc[rr] = fmaf(r.s.y, (float)d1[rr], acc[rr]);
                }
                if (MINF) {
                    const v4i x0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, ones, zero, 0, 0, 0);
                    const v4i x1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xb, ones, zero, 0, 0, 0);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        acc[rr] = fmaf(r.mn.x, (float)x0[rr], acc[rr]);
                        acc[rr] = fmaf(r.mn.y, (float)x1[rr], acc[rr]);
                    }
                }
            }
        }
        if (!PREFETCH) break;   // the host guarantees n_chunks <= UNROLL
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) cur[u] = nxt[u];
    }

    // Sum over the KSPLIT waves of the row tile, in a fixed order.
    if (KSPLIT > 1) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) lds_part[(wave * 4 + rr) * 64 + lane] = acc[rr];
        __syncthreads();
        if (ks != 0) return;
#pragma unroll
        for (int j = 1; j < KSPLIT; ++j)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[rr] += lds_part[((wave + j) * 4 + rr) * 64 + lane];
    }
    if (!active) return;
    const int64_t n = tile * kTileN + row;
    const float b = bias ? bias[n] : 0.0f;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int m = kb * 4 + rr;
        if (m < M) y[(int64_t)m * L.N + n] = fmaf(acc[rr], sx[m], b);
    }
}

template <int WAVES, int KSPLIT, int UNROLL, bool PREFETCH, bool STAGED>
int launch_cfg(const uint8_t* packed, const Layout& L, int M, const int8_t* xq, const float* sx, const float* bias,
               float* y, hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    const size_t smem = (size_t)WAVES * 4 * 64 * 4 + (STAGED ? (size_t)L.C * 8 * 16 * 16 : 0);
    auto launch = [&](auto kern) -> int {
        if (smem > 64 * 1024) {
            // More than 64 KiB of dynamic LDS has to be allowed once per kernel and device.
            static thread_local int allowed_dev = -1;
            int dev = 0;
            MNNQ_HIP_TRY(hipGetDevice(&dev));
            if (allowed_dev != dev) {
                MNNQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
                allowed_dev = dev;
            }
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WAVES * 64), smem, st, packed, L, M, xq, sx, bias, y);
        MNNQ_HIP_TRY(hipGetLastError());
        return MNNQ_OK;
    };
    if (L.minf) return launch(skinny_kernel<WAVES, KSPLIT, UNROLL, PREFETCH, true, STAGED>);
    return launch(skinny_kernel<WAVES, KSPLIT, UNROLL, PREFETCH, false, STAGED>);
}

}  // namespace

// The smallest number of waves per row tile (up to 8) for which a wave's chunk range fits in
// its registers, so that all loads are issued at once; longer rows use a prefetching loop.
// Large layers with rows of up to 4096 values take the staged variant: 16 waves, i.e.
// 16 / KSPLIT row tiles, share one copy of the activations in LDS.
int launch_skinny(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                  const float* bias, float* y, hipStream_t st)
{
    // At most 8 waves per row tile: without staging a chunk costs 17 registers (weights and
    // activations), which a workgroup of 16 waves could not hold for 8 chunks.
    int ks = 1;
    while (ks < 8 && (L.C + ks - 1) / ks > 8) ks *= 2;
    if (const char* e = getenv("MNNQ_DECODE_KSPLIT")) {   // tests and tuning: force the split
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16) ks = v > 8 ? 8 : v;
    }
    const bool prefetch = (L.C + ks - 1) / ks > 8;
    // Staging pays once the layer is large enough to be bandwidth bound (measured: above ~16 MiB).
    bool staged = L.C <= 32 && !prefetch && L.T * L.C >= 16384;
    if (const char* e = getenv("MNNQ_SKINNY_STAGED")) staged = L.C <= 32 && !prefetch && e[0] == '1';   // tests
    const int m = (int)M;
#define MNNQ_CFG(W, K)                                                                                 \
    if (ks == K) {                                                                                     \
        if (staged) return launch_cfg<16, K, 8, false, true>(packed, L, m, xq, sx, bias, y, st);       \
        return prefetch ? launch_cfg<W, K, 4, true, false>(packed, L, m, xq, sx, bias, y, st)          \
                        : launch_cfg<W, K, 8, false, false>(packed, L, m, xq, sx, bias, y, st);        \
    }
    MNNQ_CFG(4, 1) MNNQ_CFG(4, 2) MNNQ_CFG(4, 4) MNNQ_CFG(8, 8)
#undef MNNQ_CFG
    return MNNQ_ERR_UNSUPPORTED;
}

}  // namespace mnnq
