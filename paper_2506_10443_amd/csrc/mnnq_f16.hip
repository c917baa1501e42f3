// W4A16 decode step (Section 4.2: on GPUs the int4 weights are combined with
// fp16 activations to use the floating-point units): same packed weights,
// the activation row stays fp16, accumulation in fp32 with v_dot2_f32_f16.
//
//   y[n] = sum_g scale[n,g] * sum_{k in g} float(x16[k]) * (q[n,k] - zero[n,g]) (+ bias[n])
//
// The integer q - z (|.| <= 15) is exact in fp16, so the weights enter the
// contraction without rounding and the group scale is applied once per group
// in fp32.  Codes become fp16 two at a time: (0x6400 | q) is the half 1024 + q,
// and subtracting the half 1024 + z leaves q - z exactly.
//
// Float-minimum weights (Eq. 1 as printed; also the two 4-bit planes of 8-bit codes):
//   y[n] = sum_g (step[n,g] * sum_{k in g} x[k] q[n,k] + min[n,g] * sum_{k in g} x[k]);
// the codes enter as the halves q (subtract 1024 only) and the fp32 sums of the
// 16-element blocks of x are computed once, when x is staged.
//
// A pair built from one dword with `(w >> 4 s) & 0x000f000f` holds the codes
// j = s/2 + 4 (s%2) and j + 2 of that dword's eight codes, i.e. the eight
// codes come out in the order 0 2 4 6 1 3 5 7.  The activations are put into
// that order once, when they are staged in LDS.
#include "mnnq_common.h"

#include <hip/hip_fp16.h>
#include <stdlib.h>

namespace mnnq {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

union H2Bits {
    uint32_t u;
    h2 h;
};

__device__ __forceinline__ h2 as_h2(uint32_t u)
{
    H2Bits b;
    b.u = u;
    return b.h;
}

__device__ __forceinline__ uint32_t as_u32(h2 h)
{
    H2Bits b;
    b.h = h;
    return b.u;
}

// The s-th pair of (q - z) halves of dword w; zb = the half 1024 + z twice.
__device__ __forceinline__ h2 code_pair(uint32_t w, int s, h2 zb)
{
    return as_h2(((w >> (4 * s)) & 0x000f000fu) | 0x64006400u) - zb;
}

// Natural order (h0 h1)(h2 h3)(h4 h5)(h6 h7) -> (h0 h2)(h4 h6)(h1 h3)(h5 h7).
__device__ __forceinline__ uint4 permute8(uint4 v)
{
    uint4 o;
    o.x = __builtin_amdgcn_perm(v.y, v.x, 0x05040100u);
    o.y = __builtin_amdgcn_perm(v.w, v.z, 0x05040100u);
    o.z = __builtin_amdgcn_perm(v.y, v.x, 0x07060302u);
    o.w = __builtin_amdgcn_perm(v.w, v.z, 0x07060302u);
    return o;
}

// ---------------------------------------------------------------- decode

struct ChunkRegs {
    u32x4 w;
    float2 s;
    uint32_t z;    // zero points of both groups (integer zero point form)
    float2 mn;     // group minima of both groups (float minimum form)
};

template <bool MINF>
__device__ __forceinline__ ChunkRegs load_chunk(const u32x4* wp, const float2* sp, const void* zp, int64_t i)
{
    ChunkRegs r;
    r.w = __builtin_nontemporal_load(wp + i * 64);
    r.s = sp[i * 16];
    if (MINF) {
        r.mn = static_cast<const float2*>(zp)[i * 16];
        r.z = 0;
    } else {
        r.z = static_cast<const uint16_t*>(zp)[i * 16];
        r.mn = make_float2(0.0f, 0.0f);
    }
    return r;
}

__device__ __forceinline__ float dot16_f16(uint32_t w0, uint32_t w1, uint32_t z, const uint4& xa,
                                           const uint4& xb)
{
    const _Float16 zh = (_Float16)(float)(1024u + z);
    const h2 zb = {zh, zh};
    float p = 0.0f;
    p = __builtin_amdgcn_fdot2(code_pair(w0, 0, zb), as_h2(xa.x), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w0, 1, zb), as_h2(xa.y), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w0, 2, zb), as_h2(xa.z), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w0, 3, zb), as_h2(xa.w), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w1, 0, zb), as_h2(xb.x), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w1, 1, zb), as_h2(xb.y), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w1, 2, zb), as_h2(xb.z), p, false);
    p = __builtin_amdgcn_fdot2(code_pair(w1, 3, zb), as_h2(xb.w), p, false);
    return p;
}

// A wave owns one row tile and a contiguous chunk range; KSPLIT waves share a row
// tile and add their partial sums in a fixed order through LDS.  As in the W4A8
// decode kernel the host picks KSPLIT so that a wave's whole chunk range fits in
// registers: all weight loads are issued before the activations are touched, and
// each wave stages only the slice of x it consumes into a private LDS region (no
// barrier).
//
// EARLY (whole chunk range in registers): the wave's slice of x is requested ahead of the weights
// and every wave issues all UNROLL chunk loads without a branch, a wave with fewer chunks repeating
// its first one.  Loads return in order, and only for straight-line code does the compiler count
// how many younger loads may still be in flight when x is first used (behind conditional loads it
// waits for the whole weight stream before x is staged).  Used where it pays: small layers, and
// layers whose waves all have exactly UNROLL chunks.
template <int WAVES, int KSPLIT, int UNROLL, bool PREFETCH, bool MINF, bool EARLY = false>
__global__ __launch_bounds__(WAVES * 64) void decode_f16_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                                const uint16_t* __restrict__ x16,
                                                                const float* __restrict__ bias,
                                                                float* __restrict__ y, int PW)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int64_t C = L.C;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane & 15;
    const int kb = lane >> 4;
    // per wave: PW * 128 halves (permuted by 8), then the fp32 sums of their 16-element blocks
    // stored as [chunk][half][kb] (used by the float minimum form only)
    constexpr int kPerChunk = MINF ? 256 + 32 : 256;
    uint4* lds_x = reinterpret_cast<uint4*>(smem + (size_t)wave * PW * kPerChunk);
    float* lds_xs = reinterpret_cast<float*>(smem + (size_t)wave * PW * kPerChunk + (size_t)PW * 256);
    float* lds_part = reinterpret_cast<float*>(smem + (size_t)WAVES * PW * kPerChunk);  // [WAVES][16]

    constexpr int TILES_PER_WG = WAVES / KSPLIT;
    const int64_t tile = (int64_t)blockIdx.x * TILES_PER_WG + wave / KSPLIT;
    const int ks = wave % KSPLIT;
    const bool active = tile < L.T;
    static_assert(!EARLY || !PREFETCH, "EARLY: no prefetch loop");
    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const int64_t n_chunks = active ? (c1 - c0) : 0;
    // (EARLY: a wave without chunks - a row tile past the matrix, an empty share of a short row -
    // points at chunk 0 of the last row tile; what it loads is discarded)
    const int64_t first = (!EARLY || n_chunks > 0) ? tile * C + c0 : (L.T - 1) * C;
    const u32x4* wp = reinterpret_cast<const u32x4*>(packed) + first * 64 + lane;
    const float2* sp = reinterpret_cast<const float2*>(packed + L.scales_off()) + first * 16 + row;
    const void* zp = MINF ? static_cast<const void*>(reinterpret_cast<const float2*>(packed + L.zeros_off()) +
                                                     first * 16 + row)
                          : static_cast<const void*>(reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) +
                                                     first * 16 + row);

    // This wave's slice of x in units of 8 halves (16 B): unit u of the region is unit
    // c0 * 16 + u of the packed reduction axis, which runs over the activation row once
    // (twice for 8-bit codes: one 4-bit plane after the other); units past K are zero.
    constexpr int XP = (UNROLL * 16 + 63) / 64;
    const int64_t own = n_chunks * 16;
    const int64_t valid = L.K / 8;
    const int64_t row_units = L.Kx / 8;
    uint4 xv[XP];
    if (EARLY) {
#pragma unroll
        for (int j = 0; j < XP; ++j) {
            const int64_t u = lane + 64 * j, gu = c0 * 16 + u;
            const bool ok = u < own && gu < valid;
            xv[j] = reinterpret_cast<const uint4*>(x16)[ok ? (gu >= row_units ? gu - row_units : gu) : 0];
            if (!ok) xv[j] = make_uint4(0, 0, 0, 0);
        }
    }

    ChunkRegs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        if (EARLY) {
            // (a repeated chunk: all lanes on its first 16 bytes, one cache line instead of sixteen)
            cur[u] = load_chunk<MINF>(u < n_chunks ? wp : wp - lane, sp, zp, u < n_chunks ? u : 0);
        } else if (u < n_chunks) {
            cur[u] = load_chunk<MINF>(wp, sp, zp, u);
        } else {
            cur[u] = ChunkRegs{};
        }
    }

    {
        auto put = [&](int64_t u, const uint4 v) {
            lds_x[u] = permute8(v);
            if (MINF) {
                // sum of the 16-element block: its two units sit in neighbouring lanes
                const h2 one = {(_Float16)1.0f, (_Float16)1.0f};
                float sum = __builtin_amdgcn_fdot2(as_h2(v.x), one, 0.0f, false);
                sum = __builtin_amdgcn_fdot2(as_h2(v.y), one, sum, false);
                sum = __builtin_amdgcn_fdot2(as_h2(v.z), one, sum, false);
                sum = __builtin_amdgcn_fdot2(as_h2(v.w), one, sum, false);
                sum += __shfl_xor(sum, 1, 64);
                // unit 8 h + 2 kb + e of the chunk -> block [h][kb]
                if ((u & 1) == 0) lds_xs[(u / 16) * 8 + ((u % 16) / 8) * 4 + ((u % 8) / 2)] = sum;
            }
        };
        if (EARLY) {   // at most UNROLL chunks: all of them were requested above
#pragma unroll
            for (int j = 0; j < XP; ++j)
                if (lane + 64 * j < own) put(lane + 64 * j, xv[j]);
        } else {
            for (int64_t u = lane; u < own; u += 64) {
                const int64_t gu = c0 * 16 + u;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (gu < valid) v = reinterpret_cast<const uint4*>(x16)[gu >= row_units ? gu - row_units : gu];
                put(u, v);
            }
        }
        // The region is private to the wave; LDS operations of one wave complete in order.
    }

    float accf = 0.0f;
    for (int64_t i = 0; i < n_chunks; i += UNROLL) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const ChunkRegs& r = cur[u];
            if (i + u < n_chunks) {
                // 16-byte unit of x[128 c + 64 h + 16 kb] inside the region: 16 (i + u) + 8 h + 2 kb
                const uint4* xp = lds_x + (i + u) * 16 + kb * 2;
                const float p0 = dot16_f16(r.w.x, r.w.y, r.z & 0xffu, xp[0], xp[1]);
                const float p1 = dot16_f16(r.w.z, r.w.w, r.z >> 8, xp[8], xp[9]);
                accf = fmaf(r.s.x, p0, accf);
                accf = fmaf(r.s.y, p1, accf);
                if (MINF) {
                    accf = fmaf(r.mn.x, lds_xs[(i + u) * 8 + kb], accf);
                    accf = fmaf(r.mn.y, lds_xs[(i + u) * 8 + 4 + kb], accf);
                }
            }
            if (PREFETCH) {
                // Rolling window: the registers of the chunk just consumed are refilled with the chunk
                // UNROLL further on, without a branch around the load (past the wave's range all lanes
                // read the first 16 bytes of its first chunk; the copy is never used), so that the
                // compiler waits by count and the refills stay in flight.
                const bool have = i + UNROLL + u < n_chunks;
                cur[u] = load_chunk<MINF>(have ? wp : wp - lane, sp, zp, have ? i + UNROLL + u : 0);
            }
        }
        if (!PREFETCH) break;   // the host guarantees n_chunks <= UNROLL
    }

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
        float r = accf;
        if (bias) r += bias[n];
        store_out(y, n, r, L.out16);
    }
}

template <int WAVES, int KSPLIT, int UNROLL, bool PREFETCH, bool EARLY = false>
int launch_decode_cfg(const uint8_t* packed, const Layout& L, const uint16_t* x16, const float* bias,
                      float* y, hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    const int PW = (int)((L.C + KSPLIT - 1) / KSPLIT);
    const size_t smem = (size_t)WAVES * PW * (L.minf ? 256 + 32 : 256) + WAVES * 16 * sizeof(float);
    // Rows beyond about 30000 values need more than the 64 KiB of LDS a kernel gets by default.
    static thread_local int allowed_minf = -1, allowed_zp = -1;
    if (L.minf) {
        auto kern = decode_f16_kernel<WAVES, KSPLIT, UNROLL, PREFETCH, true, EARLY>;
        if (int s = allow_large_lds(kern, smem, allowed_minf)) return s;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WAVES * 64), smem, st, packed, L, x16, bias, y, PW);
    } else {
        auto kern = decode_f16_kernel<WAVES, KSPLIT, UNROLL, PREFETCH, false, EARLY>;
        if (int s = allow_large_lds(kern, smem, allowed_zp)) return s;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WAVES * 64), smem, st, packed, L, x16, bias, y, PW);
    }
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace

// The smallest number of waves per row tile for which a wave's chunk range fits in
// its registers (8, else 12 chunks); very long rows fall back to a prefetching loop.
int launch_decode_f16(const uint8_t* packed, const Layout& L, const uint16_t* x16, const float* bias,
                      float* y, hipStream_t st)
{
    int ks = 1;
    while (ks < 16 && (L.C + ks - 1) / ks > 8) ks *= 2;
    int unroll = 8, prefetch = 0;
    if ((L.C + ks - 1) / ks > 8) {
        if ((L.C + 15) / 16 <= 12) unroll = 12;
        else prefetch = 1;
    }
    if (const char* e = debug_option(kDbgDecodeKsplit)) {   // tests and tuning: force the split
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16) {
            ks = v;
            const int64_t pw = (L.C + ks - 1) / ks;
            unroll = pw <= 8 ? 8 : (pw <= 12 && ks == 16 ? 12 : 8);
            prefetch = pw > unroll;
        }
    }
    // Rows of 28 chunks (K = 3584) on four waves: seven chunks each, with no register left unused
    if (ks == 4 && L.C == 28 && !prefetch && !debug_option(kDbgDecodeKsplit)) unroll = 7;
    // x staged under the weight stream: small layers whose waves have at most two chunks fewer than `unroll`,
    // and those whose waves all have exactly `unroll` chunks
    const bool exact = L.C % ks == 0 && L.C / ks == unroll;
    bool early = !prefetch && (((int64_t)L.total() <= (16 << 20) && L.C / ks >= unroll - 2) || exact);
    if (const char* e = debug_option(kDbgDecodeEarly)) early = !prefetch && e[0] == '1';   // tests and tuning
#define MNNQ_CFG(W, K, U, P)                                                              \
    if (ks == K && unroll == U && prefetch == P) {                                        \
        if constexpr (P == 0) {                                                           \
            if (early) return launch_decode_cfg<W, K, U, false, true>(packed, L, x16, bias, y, st); \
        }                                                                                 \
        return launch_decode_cfg<W, K, U, (P != 0)>(packed, L, x16, bias, y, st);         \
    }
    MNNQ_CFG(4, 1, 8, 0) MNNQ_CFG(4, 2, 8, 0) MNNQ_CFG(4, 4, 8, 0) MNNQ_CFG(4, 4, 7, 0) MNNQ_CFG(8, 8, 8, 0)
    MNNQ_CFG(16, 16, 8, 0) MNNQ_CFG(16, 16, 12, 0)
    MNNQ_CFG(4, 1, 8, 1) MNNQ_CFG(4, 2, 8, 1) MNNQ_CFG(4, 4, 8, 1) MNNQ_CFG(8, 8, 8, 1) MNNQ_CFG(16, 16, 8, 1)
#undef MNNQ_CFG
    return MNNQ_ERR_UNSUPPORTED;
}

}  // namespace mnnq
