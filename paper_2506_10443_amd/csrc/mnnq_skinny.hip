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
// LDS.  The activations are small (M * K bytes) and stay in L2: each lane loads its A
// operand - 16 consecutive k of token lane % 16 - straight from there (skinny_kernel),
// or, for large layers whose 16 rows fit in LDS (K <= 4096), a persistent workgroup
// copies them there once and shares them between all its row tiles
// (skinny_persist_kernel).
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

template <int WAVES, int KSPLIT, int UNROLL, bool PREFETCH, bool MINF>
__global__ __launch_bounds__(WAVES * 64) void skinny_kernel(const uint8_t* __restrict__ packed, Layout L, int M,
                                                            const int8_t* __restrict__ xq,
                                                            const float* __restrict__ sx,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ y)
{
    __shared__ float lds_part[WAVES * 4 * 64];   // [wave][r][lane]
    const int64_t C = L.C;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: addresses start in scalar registers
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
        r.xa = *reinterpret_cast<const v4i*>(xrow + (c % Cx) * 128);
        r.xb = (odd_tail && c == C - 1) ? v4i{0, 0, 0, 0} : *reinterpret_cast<const v4i*>(xrow + (c % Cx) * 128 + 64);
        return r;
    };

    SkinnyRegs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        if (u < n_chunks) cur[u] = load(u);
        else cur[u] = SkinnyRegs{};
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
                const v4i xa = r.xa, xb = r.xb;
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
        if (m < M) store_out(y, (int64_t)m * L.N + n, fmaf(acc[rr], sx[m], b), L.out16);
    }
}

// Large layers with rows of up to 4096 values: a persistent workgroup of 8 waves copies the
// 16 token rows into LDS once, in the order the A operand is read, and then walks over its
// share of the row tiles (8 / KSPLIT at a time).  Every wave's chunk range (<= 8 chunks) is
// held in registers; as soon as a chunk has been consumed, the same chunk of the next step is
// fetched into its registers, so a wave keeps its whole range in flight all the time.
struct WeightRegs {
    u32x4 w;
    float2 s;
    uint32_t z;
    float2 mn;
};

template <int KSPLIT, bool MINF>
__global__ __launch_bounds__(512, 2) void skinny_persist_kernel(const uint8_t* __restrict__ packed, Layout L, int M,
                                                             const int8_t* __restrict__ xq,
                                                             const float* __restrict__ sx,
                                                             const float* __restrict__ bias,
                                                             float* __restrict__ y)
{
    constexpr int WAVES = 8, UNROLL = 8;
    extern __shared__ __align__(16) uint8_t smem[];
    float* lds_part = reinterpret_cast<float*>(smem);                                 // [wave][r][lane]
    v4i* lds_a = reinterpret_cast<v4i*>(smem + WAVES * 4 * 64 * 4);                   // [C * 8 units][16 tokens]
    const int64_t C = L.C;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: addresses start in scalar registers
    const int row = lane & 15;
    const int kb = lane >> 4;
    constexpr int TILES_PER_STEP = WAVES / KSPLIT;
    const int ks = wave % KSPLIT;
    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const int n_own = (int)(c1 - c0);
    const int64_t n_steps = (L.T + TILES_PER_STEP - 1) / TILES_PER_STEP;

    // One chunk of this wave's range for the given step (nothing past the last step / tile).
    auto load_chunk = [&](int64_t step, int u) {
        WeightRegs r{};
        const int64_t tile = step * TILES_PER_STEP + wave / KSPLIT;
        if (step < n_steps && tile < L.T && u < n_own) {
            const int64_t ci = (tile * C + c0 + u);
            r.w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(packed) + ci * 64 + lane);
            r.s = (reinterpret_cast<const float2*>(packed + L.scales_off()) + ci * 16)[row];
            if (MINF) r.mn = (reinterpret_cast<const float2*>(packed + L.zeros_off()) + ci * 16)[row];
            else r.z = (reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) + ci * 16)[row];
        }
        return r;
    };

    int64_t step = blockIdx.x;
    WeightRegs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) cur[u] = load_chunk(step, u);

    // The first weights are in flight; copy the token rows (tokens past M repeat the last one,
    // k past K is zero) in units of 16 bytes: unit (ku, m) = k 16 ku .. 16 ku + 15 of token m,
    // stored at index ku * 16 + m.
    {
        const int units = (int)C * 8 * 16;
        const int valid_ku = (int)(L.K / 16);
        const int row_ku = (int)(L.Kx / 16);
        for (int u = tid; u < units; u += WAVES * 64) {
            const int m = u & 15, ku = u >> 4;
            v4i v = {0, 0, 0, 0};
            if (ku < valid_ku)
                v = *reinterpret_cast<const v4i*>(xq + (int64_t)(m < M ? m : M - 1) * L.Kx + (ku % row_ku) * 16);
            lds_a[u] = v;
        }
    }
    __syncthreads();

    const v4i zero = {0, 0, 0, 0};
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    // All waves of a workgroup share `step`, so the workgroup-wide barriers below are uniform.
    for (; step < n_steps; step += gridDim.x) {
        const int64_t tile = step * TILES_PER_STEP + wave / KSPLIT;
        const bool active = tile < L.T;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const WeightRegs r = cur[u];
            // the registers of this chunk are free: fetch the same chunk of the next step into them
            cur[u] = load_chunk(step + gridDim.x, u);
            if (active && u < n_own) {
                const int64_t c = c0 + u;
                const v4i xa = lds_a[((c * 8 + kb) << 4) + row];
                const v4i xb = lds_a[((c * 8 + 4 + kb) << 4) + row];
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
        if (KSPLIT > 1) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) lds_part[(wave * 4 + rr) * 64 + lane] = acc[rr];
            __syncthreads();
            if (ks == 0) {
#pragma unroll
                for (int j = 1; j < KSPLIT; ++j)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) acc[rr] += lds_part[((wave + j) * 4 + rr) * 64 + lane];
            }
            __syncthreads();   // the partial sums are read before the next round overwrites them
        }
        if (active && ks == 0) {
            const int64_t n = tile * kTileN + row;
            const float b = bias ? bias[n] : 0.0f;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int m = kb * 4 + rr;
                if (m < M) store_out(y, (int64_t)m * L.N + n, fmaf(acc[rr], sx[m], b), L.out16);
            }
        }
    }
}

template <int KSPLIT>
int launch_persist(const uint8_t* packed, const Layout& L, int M, const int8_t* xq, const float* sx, const float* bias,
                   float* y, hipStream_t st)
{
    constexpr int tiles_per_step = 8 / KSPLIT;
    const int64_t n_steps = (L.T + tiles_per_step - 1) / tiles_per_step;
    // Two workgroups per CU (LDS: two copies of the activations; registers: 16 waves).
    const int64_t grid = n_steps < 2 * (int64_t)num_cus() ? n_steps : 2 * (int64_t)num_cus();
    const size_t smem = (size_t)8 * 4 * 64 * 4 + (size_t)L.C * 8 * 16 * 16;
    auto launch = [&](auto kern) -> int {
        if (smem > 64 * 1024) {
            // More than 64 KiB of dynamic LDS has to be allowed once per kernel and device.
            static thread_local int allowed_dev = -1;
            int dev = 0;
            MNNQ_HIP_TRY(hipGetDevice(&dev));
            if (allowed_dev != dev) {
                MNNQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024));
                allowed_dev = dev;
            }
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), smem, st, packed, L, M, xq, sx, bias, y);
        MNNQ_HIP_TRY(hipGetLastError());
        return MNNQ_OK;
    };
    if (L.minf) return launch(skinny_persist_kernel<KSPLIT, true>);
    return launch(skinny_persist_kernel<KSPLIT, false>);
}

template <int WAVES, int KSPLIT, int UNROLL, bool PREFETCH>
int launch_cfg(const uint8_t* packed, const Layout& L, int M, const int8_t* xq, const float* sx, const float* bias,
               float* y, hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    if (L.minf)
        hipLaunchKernelGGL((skinny_kernel<WAVES, KSPLIT, UNROLL, PREFETCH, true>), dim3((unsigned)blocks),
                           dim3(WAVES * 64), 0, st, packed, L, M, xq, sx, bias, y);
    else
        hipLaunchKernelGGL((skinny_kernel<WAVES, KSPLIT, UNROLL, PREFETCH, false>), dim3((unsigned)blocks),
                           dim3(WAVES * 64), 0, st, packed, L, M, xq, sx, bias, y);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace

// The smallest number of waves per row tile (up to 8) for which a wave's chunk range fits in
// its registers, so that all loads are issued at once; longer rows use a prefetching loop.
// Large layers with rows of up to 4096 values take the persistent variant, which shares one
// LDS copy of the activations between all the row tiles a workgroup processes.
int launch_skinny(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                  const float* bias, float* y, hipStream_t st)
{
    // At most 8 waves per row tile: without staging a chunk costs 17 registers (weights and
    // activations), which a workgroup of 16 waves could not hold for 8 chunks.
    int ks = 1;
    while (ks < 8 && (L.C + ks - 1) / ks > 8) ks *= 2;
    if (const char* e = debug_option(kDbgDecodeKsplit)) {   // tests and tuning: force the split
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16) ks = v > 8 ? 8 : v;
    }
    const bool prefetch = (L.C + ks - 1) / ks > 8;
    // Staging pays once the layer is large enough to be bandwidth bound (measured: above ~16 MiB).
    bool staged = L.C <= 32 && !prefetch && L.T * L.C >= 16384;
    if (const char* e = debug_option(kDbgSkinnyStaged)) staged = L.C <= 32 && !prefetch && e[0] == '1';   // tests
    const int m = (int)M;
#define MNNQ_CFG(W, K)                                                                                 \
    if (ks == K) {                                                                                     \
        if (staged) return launch_persist<K>(packed, L, m, xq, sx, bias, y, st);                       \
        return prefetch ? launch_cfg<W, K, 4, true>(packed, L, m, xq, sx, bias, y, st)                 \
                        : launch_cfg<W, K, 8, false>(packed, L, m, xq, sx, bias, y, st);               \
    }
    MNNQ_CFG(4, 1) MNNQ_CFG(4, 2) MNNQ_CFG(4, 4) MNNQ_CFG(8, 8)
#undef MNNQ_CFG
    return MNNQ_ERR_UNSUPPORTED;
}

}  // namespace mnnq
