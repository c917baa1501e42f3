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
// A layer is a few MB to a few tens of MB, i.e. microseconds of HBM time, so
// the kernel is built to have every byte in flight as early as possible: the
// host picks KSPLIT so that a wave's whole chunk range fits in registers, and
// the wave issues all its loads before it touches the activations.
//
// The activation row takes one of two routes into the workgroup's LDS:
//   XQ    - already quantized int8 (mnnq_quant_act ran before);
//   FUSED - fp32 input, quantized here: per-token symmetric int8 (Section 4.2),
//           scale = max|x| / 127, the same IEEE operations as mnnq_quant_act.
//           Every workgroup repeats this for the whole row; the rounding is done
//           with a multiply and falls back to the division only next to a tie
//           (see quant4_fast), which gives the same codes at a fraction of the cost.
// This file is compiled with -ffp-contract=off for that reason.
#include "mnnq_common.h"

#include <stdio.h>
#include <stdlib.h>

namespace mnnq {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Mode { kXQ = 0, kFused = 1, kAcc = 2 };

struct ChunkRegs {
    u32x4 w;      // 32 codes: .x,.y group 2c ; .z,.w group 2c+1
    float2 s;     // scales of the lane's row for both groups
    uint32_t z;   // zero points, low byte group 2c, next byte group 2c+1      (integer zero point form)
    float2 mn;    // group minima of the lane's row for both groups          (float minimum form)
};

// MINF: the packed matrix holds fp32 group minima where the zero points would be.
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

__device__ __forceinline__ int dot16(uint32_t wa, uint32_t wb, const int4& x)
{
    int d = __builtin_amdgcn_sdot4((int)(wa & 0x0f0f0f0fu), x.x, 0, false);
    d = __builtin_amdgcn_sdot4((int)((wa >> 4) & 0x0f0f0f0fu), x.y, d, false);
    d = __builtin_amdgcn_sdot4((int)(wb & 0x0f0f0f0fu), x.z, d, false);
    d = __builtin_amdgcn_sdot4((int)((wb >> 4) & 0x0f0f0f0fu), x.w, d, false);
    return d;
}

// Fused activation quantizer: per-token symmetric int8 (Section 4.2) of the fp32 row x into the
// workgroup's LDS image - the row as dwords of four codes over the padded packed reduction axis
// (which runs over the row twice for int8 weights) and the sums of its 16-byte blocks as
// [chunk][kb][half].  Returns the scale max|x| / 127; the same IEEE operations as mnnq_quant_act.
// All WAVES * 64 threads of the workgroup call it; it ends with a barrier.
//
// Loads return in the order they were issued, so a row that is read after the weight stream has
// been started cannot be touched before all those weights have arrived.  The caller therefore
// reads the first XR float4 per thread (elements tid + j * THREADS) before it starts the weights
// and passes them in; rows that fit (K <= 4 * XR * THREADS) are then quantized without another
// load, longer ones read the rest from memory.
constexpr int kRowRegs = 2;

template <int WAVES>
__device__ __forceinline__ void preload_row(const float* __restrict__ x, const Layout& L, float4 (&xr)[kRowRegs])
{
    constexpr int THREADS = WAVES * 64;
    const int row_dw = (int)(L.Kx / 4);     // (a row the GEMV can stage has fewer than 2^17 values: 32-bit indices)
    const float4* x4 = reinterpret_cast<const float4*>(x);
#pragma unroll
    for (int j = 0; j < kRowRegs; ++j) {
        const int i = (int)threadIdx.x + j * THREADS;
        xr[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (i < row_dw) xr[j] = x4[i];
    }
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() carries a release fence, for which
// the compiler waits for every outstanding global load too - here the weight stream, which may
// stay in flight while the row is quantized.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Maximum over the workgroup (one barrier) -> quantization scale max|x| / 127.
template <int WAVES>
__device__ __forceinline__ float workgroup_scale(float amax, float* lds_amax)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    amax = wave_max_nonneg(amax);            // (max_abs4 drops NaNs and signs)
    if (lane == 0) lds_amax[wave] = amax;
    lds_barrier();
    amax = lds_amax[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) amax = fmaxf(amax, lds_amax[w]);
    return (amax == 0.0f) ? 0.0f : amax / 127.0f;
}

__device__ __forceinline__ float max_abs4(float amax, const float4 v)
{
    return fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
}

// One dword i of the padded row: quantize, store, and add up its 16-byte block (the four dwords
// of a block sit in four neighbouring lanes, which all call this together).
struct RowQuantizer {
    float scale, inv, lim;
    int valid;
    int* lds_xd;
    int* lds_xs;
    __device__ __forceinline__ explicit RowQuantizer(float s, int valid_, int* xd, int* xs)
        : scale(s), inv(s == 0.0f ? 0.0f : 1.0f / s), valid(valid_), lds_xd(xd), lds_xs(xs)
    {
        lim = quant_fast_limit(scale, inv);
    }
    __device__ __forceinline__ void put(int i, const float4 xv) const
    {
        int v = 0;
        if (i < valid && scale != 0.0f) v = quant4_fast(xv, scale, inv, lim);
        lds_xd[i] = v;
        int sum = __builtin_amdgcn_sdot4(v, 0x01010101, 0, false);
        sum += row_exchange<0xB1>(sum);      // the four dwords of a block: one quad of lanes
        sum += row_exchange<0x4E>(sum);
        if ((threadIdx.x & 3) == 0) {
            const int u = i >> 2;                       // 16-byte block; chunk u / 8
            lds_xs[(u & ~7) + (u & 3) * 2 + ((u >> 2) & 1)] = sum;
        }
    }
};

template <int WAVES>
__device__ __forceinline__ float quantize_row_to_lds(const float* __restrict__ x, const float4 (&xr)[kRowRegs],
                                                     const Layout& L, int* lds_xd, int* lds_xs, float* lds_amax)
{
    constexpr int THREADS = WAVES * 64;
    const int tid = threadIdx.x;
    const int dwords = (int)(L.C * 32);                  // padded row of the packed reduction axis
    const int valid = (int)(L.K / 4);
    const int row_dw = (int)(L.Kx / 4);                  // the activation row itself
    const float4* x4 = reinterpret_cast<const float4*>(x);

    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < kRowRegs; ++j) amax = max_abs4(amax, xr[j]);   // zeros past the row do not change the maximum
    for (int i = tid + kRowRegs * THREADS; i < row_dw; i += THREADS) amax = max_abs4(amax, x4[i]);
    const RowQuantizer q(workgroup_scale<WAVES>(amax, lds_amax), valid, lds_xd, lds_xs);
    // The row itself: first the elements already in registers, then the rest from memory.  (No
    // conditional between a register value and a load: it would select between two addresses and
    // force the registers into scratch memory.)  The row length is a multiple of 16 dwords, so the
    // four lanes of a block always take the same branch.
#pragma unroll
    for (int j = 0; j < kRowRegs; ++j) {
        const int i = tid + j * THREADS;
        if (i < row_dw) q.put(i, xr[j]);
    }
    for (int i = tid + kRowRegs * THREADS; i < row_dw; i += THREADS) q.put(i, x4[i]);
    // Past the row: its second pass (int8 weights) and the zero padding of the last chunk.
    for (int i = row_dw + tid; i < dwords; i += THREADS) {
        float4 xv = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (i < valid) xv = x4[i - row_dw];              // (the packed axis runs over the row at most twice)
        q.put(i, xv);
    }
    lds_barrier();
    return q.scale;
}

// LDS of a workgroup: the activation row (K int8, zero padded to C * 128 bytes),
// the sums of its 16-byte blocks stored as [chunk][kb][half], the partial sums
// of the split rows and the per-wave maxima of the fused quantizer.
//
// EARLY (whole chunk range in registers): the wave's part of the activation row is requested ahead
// of the weights, and every wave issues all UNROLL chunk loads without a branch, a wave with fewer
// chunks repeating its first one.  Loads return in order, and only for straight-line code does the
// compiler count how many younger loads may still be in flight when the row elements are first
// used; behind conditional loads it waits for all of them, so that the row is quantized and staged
// only when the whole weight stream has arrived.  The launches of small layers, which are bound by
// latency, gain 7 - 9 % from the overlap; layers whose waves hold clearly fewer chunks than UNROLL
// lose (3 - 13 % measured) and keep the conditional form: the host decides (decode_config).
template <int WAVES, int KSPLIT, int UNROLL, int MODE, bool PREFETCH, bool MINF, bool EARLY = false>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                            const void* __restrict__ xin,
                                                            const float* __restrict__ sx,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ y,
                                                            int32_t* __restrict__ acc, int PW)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int64_t C = L.C;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // Fused quantizer: the wave index is made uniform, so that the wave's addresses start in scalar
    // registers - 7 vector registers fewer, i.e. one more wave per SIMD (decode pass -4.7 %).  The
    // plain GEMV is faster without (+3 % with): its launches wait on the scalar address arithmetic.
    const int wave = (MODE == kFused) ? __builtin_amdgcn_readfirstlane(tid >> 6) : (tid >> 6);
    const int row = lane & 15;
    const int kb = lane >> 4;
    constexpr int TILES_PER_WG = WAVES / KSPLIT;
    const int64_t tile = (int64_t)blockIdx.x * TILES_PER_WG + wave / KSPLIT;
    const int ks = wave % KSPLIT;
    const int64_t m = (MODE == kAcc) ? blockIdx.y : 0;
    const bool active = tile < L.T;

    // Fused mode: one image of the whole row per workgroup.  Otherwise every wave
    // stages just the chunk range it consumes into a private region (PW chunks),
    // which needs no barrier.
    constexpr bool SHARED = (MODE == kFused);
    const size_t x_bytes = SHARED ? (size_t)C * 160 : (size_t)WAVES * PW * 160;
    uint8_t* xbase = SHARED ? smem : smem + (size_t)wave * PW * 160;
    const size_t xs_off = SHARED ? (size_t)C * 128 : (size_t)PW * 128;
    int* lds_xd = reinterpret_cast<int*>(xbase);                        // row as dwords
    const int4* lds_x = reinterpret_cast<const int4*>(xbase);           // row as 16-byte units
    int* lds_xs = reinterpret_cast<int*>(xbase + xs_off);
    float* lds_part = reinterpret_cast<float*>(smem + x_bytes);         // [WAVES][16]
    float* lds_amax = lds_part + WAVES * 16;                            // [WAVES]

    static_assert(!EARLY || (MODE != kAcc && !PREFETCH), "EARLY: no prefetch loop");
    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const int64_t n_chunks = active ? (c1 - c0) : 0;
    // (EARLY: a wave without chunks - a row tile past the matrix, an empty share of a short row -
    // points at chunk 0 of the last row tile; what it loads is discarded)
    const int64_t first = (!EARLY || n_chunks > 0) ? tile * C + c0 : (L.T - 1) * C;
    const u32x4* wp = reinterpret_cast<const u32x4*>(packed) + first * 64 + lane;
    const float2* sp = reinterpret_cast<const float2*>(packed + L.scales_off()) + first * 16 + row;
    // zero points (2 x u8 per row and chunk) or group minima (2 x fp32)
    const void* zp = MINF ? static_cast<const void*>(reinterpret_cast<const float2*>(packed + L.zeros_off()) +
                                                     first * 16 + row)
                          : static_cast<const void*>(reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) +
                                                     first * 16 + row);

    // Fused quantizer: the first elements of the row are requested ahead of the weights, so that
    // they arrive first (see quantize_row_to_lds).
    float4 xr[kRowRegs];
    if (MODE == kFused) preload_row<WAVES>(static_cast<const float*>(xin), L, xr);
    // Quantized row given: the wave's own chunks of it in 16-byte units (unit u of its LDS region is unit
    // c0 * 8 + u of the row; the packed axis runs over the row at most twice); EARLY: requested here.
    constexpr int XP = (UNROLL * 8 + 63) / 64;
    const int64_t valid = L.K / 4;                       // dwords of the packed reduction axis that carry data
    const int4* xq16 = reinterpret_cast<const int4*>(static_cast<const int8_t*>(xin) + m * L.Kx);
    const int64_t row_units = L.Kx / 16;
    const int64_t own = n_chunks * 8;
    int4 xv[XP];
    if (EARLY && MODE != kFused) {
#pragma unroll
        for (int j = 0; j < XP; ++j) {
            const int64_t u = lane + 64 * j, gu = c0 * 8 + u;
            const bool ok = u < own && gu * 4 < valid;
            xv[j] = xq16[ok ? (gu >= row_units ? gu - row_units : gu) : 0];   // (no branch: as for the weights)
            if (!ok) xv[j] = make_int4(0, 0, 0, 0);
        }
    }
    // Start the weight stream before the activation row is touched: it does not depend on x.
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

    // ---- activation row -> LDS
    float scale = 0.0f;
    if (MODE == kFused) {
        scale = quantize_row_to_lds<WAVES>(static_cast<const float*>(xin), xr, L, lds_xd, lds_xs, lds_amax);
    } else {
        // This wave's chunks only.
        int4* lds_xw = reinterpret_cast<int4*>(xbase);
        auto put = [&](int64_t u, const int4 v) {
            lds_xw[u] = v;
            int sum = __builtin_amdgcn_sdot4(v.x, 0x01010101, 0, false);
            sum = __builtin_amdgcn_sdot4(v.y, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4(v.z, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4(v.w, 0x01010101, sum, false);
            lds_xs[(u / 8) * 8 + (int)(u % 4) * 2 + (int)(u % 8) / 4] = sum;
        };
        if (EARLY) {   // at most UNROLL chunks: all of them were requested above
#pragma unroll
            for (int j = 0; j < XP; ++j)
                if (lane + 64 * j < own) put(lane + 64 * j, xv[j]);
        } else {
            for (int64_t u = lane; u < own; u += 64) {
                const int64_t gu = c0 * 8 + u;
                int4 v = make_int4(0, 0, 0, 0);
                if (gu * 4 < valid) v = xq16[gu >= row_units ? gu - row_units : gu];
                put(u, v);
            }
        }
        // The region is private to the wave; LDS operations of one wave complete in order.
    }
    const int64_t cbase = SHARED ? c0 : 0;    // chunk index of the wave's first chunk inside its LDS image

    float accf = 0.0f;
    for (int64_t i = 0; i < n_chunks; i += UNROLL) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const ChunkRegs& r = cur[u];
            if (i + u < n_chunks) {
                const int64_t c = c0 + i + u;
                const int64_t cl = cbase + i + u;
                const int4 xa = lds_x[cl * 8 + kb];
                const int4 xb = lds_x[cl * 8 + 4 + kb];
                const int2 xs = *reinterpret_cast<const int2*>(lds_xs + cl * 8 + kb * 2);
                // integer zero point: sum x (q - z) = sum x q - z sum x; float minimum: sum x q, the
                // minimum enters below with the same block sum
                int i0 = dot16(r.w.x, r.w.y, xa) - (MINF ? 0 : (int)(r.z & 0xffu) * xs.x);
                int i1 = dot16(r.w.z, r.w.w, xb) - (MINF ? 0 : (int)(r.z >> 8) * xs.y);
                if (MODE == kAcc) {
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
                    if (MINF) {
                        accf = fmaf(r.mn.x, (float)xs.x, accf);
                        accf = fmaf(r.mn.y, (float)xs.y, accf);
                    }
                }
            }
            if (PREFETCH) {
                // Rows longer than the registers hold: a rolling window.  The registers of the chunk just
                // consumed are refilled with the chunk UNROLL further on, so that a wave keeps UNROLL
                // chunks in flight all the time.  No branch around the load (past the wave's range all
                // lanes read the first 16 bytes of its first chunk, and the copy is never used): only
                // then does the compiler wait by count for the chunk it consumes next, with the refills
                // issued since still in flight.
                const bool have = i + UNROLL + u < n_chunks;
                cur[u] = load_chunk<MINF>(have ? wp : wp - lane, sp, zp, have ? i + UNROLL + u : 0);
            }
        }
        if (!PREFETCH) break;   // the host guarantees n_chunks <= UNROLL
    }
    if (MODE == kAcc) return;

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
        float r = accf * ((MODE == kFused) ? scale : sx[0]);
        if (bias) r += bias[n];
        store_out(y, n, r, L.out16);
    }
}

// ---------------------------------------------------------------------------------------------
// Byte form of int8 weights (Layout::native8): a chunk is two kilobytes, one per group, lane l
// holding the 16 bytes q8 - 128 of row l % 16 and k-block l / 16 - four v_dot4_i32_i8 against the
// int8 row per group, no unpacking.  With D = sum xq (q8 - 128) and xs = sum xq (the block sums
// staged with the row) a group's term is  s (D + 128 xs) + min xs.  Same work split, same LDS image
// of the activation row and same order of operations as decode_kernel: all of a wave's loads
// first (UNROLL chunks; a rolling window for longer ranges), then the row, then the dot products.
struct Chunk8Regs {
    u32x4 w0, w1;   // groups 2c and 2c + 1
    float2 s, mn;   // steps and minima of the lane's row for both groups
};

__device__ __forceinline__ Chunk8Regs load_chunk8(const u32x4* wp, const float2* sp, const float2* mp, int64_t i)
{
    Chunk8Regs r;
    r.w0 = __builtin_nontemporal_load(wp + i * 128);
    r.w1 = __builtin_nontemporal_load(wp + i * 128 + 64);
    r.s = sp[i * 16];
    r.mn = mp[i * 16];
    return r;
}

__device__ __forceinline__ int dot16_bytes(const u32x4 w, const int4& x)
{
    int d = __builtin_amdgcn_sdot4((int)w.x, x.x, 0, false);
    d = __builtin_amdgcn_sdot4((int)w.y, x.y, d, false);
    d = __builtin_amdgcn_sdot4((int)w.z, x.z, d, false);
    d = __builtin_amdgcn_sdot4((int)w.w, x.w, d, false);
    return d;
}

template <int WAVES, int KSPLIT, int UNROLL, int MODE, bool PREFETCH>
__global__ __launch_bounds__(WAVES * 64) void decode8_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                             const void* __restrict__ xin,
                                                             const float* __restrict__ sx,
                                                             const float* __restrict__ bias,
                                                             float* __restrict__ y, int PW)
{
    static_assert(MODE == kXQ || MODE == kFused, "no accumulator dump in the byte form");
    extern __shared__ __align__(16) uint8_t smem[];
    const int64_t C = L.C;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = (MODE == kFused) ? __builtin_amdgcn_readfirstlane(tid >> 6) : (tid >> 6);
    const int row = lane & 15;
    const int kb = lane >> 4;
    constexpr int TILES_PER_WG = WAVES / KSPLIT;
    const int64_t tile = (int64_t)blockIdx.x * TILES_PER_WG + wave / KSPLIT;
    const int ks = wave % KSPLIT;
    const bool active = tile < L.T;

    constexpr bool SHARED = (MODE == kFused);
    const size_t x_bytes = SHARED ? (size_t)C * 160 : (size_t)WAVES * PW * 160;
    uint8_t* xbase = SHARED ? smem : smem + (size_t)wave * PW * 160;
    const size_t xs_off = SHARED ? (size_t)C * 128 : (size_t)PW * 128;
    int* lds_xd = reinterpret_cast<int*>(xbase);
    const int4* lds_x = reinterpret_cast<const int4*>(xbase);
    int* lds_xs = reinterpret_cast<int*>(xbase + xs_off);
    float* lds_part = reinterpret_cast<float*>(smem + x_bytes);         // [WAVES][16]
    float* lds_amax = lds_part + WAVES * 16;                            // [WAVES]

    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const int64_t n_chunks = active ? (c1 - c0) : 0;
    // (a wave without chunks points at the first chunk of the matrix and loads nothing)
    const int64_t first = n_chunks > 0 ? tile * C + c0 : 0;
    const u32x4* wp = reinterpret_cast<const u32x4*>(packed) + first * 128 + lane;
    const float2* sp = reinterpret_cast<const float2*>(packed + L.scales_off()) + first * 16 + row;
    const float2* mp = reinterpret_cast<const float2*>(packed + L.zeros_off()) + first * 16 + row;

    float4 xr[kRowRegs];
    if (MODE == kFused) preload_row<WAVES>(static_cast<const float*>(xin), L, xr);
    // Start the weight stream before the activation row is touched: it does not depend on x.
    Chunk8Regs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        if (u < n_chunks) cur[u] = load_chunk8(wp, sp, mp, u);
        else cur[u] = Chunk8Regs{};
    }

    // ---- activation row -> LDS (the image of decode_kernel)
    float scale = 0.0f;
    if (MODE == kFused) {
        scale = quantize_row_to_lds<WAVES>(static_cast<const float*>(xin), xr, L, lds_xd, lds_xs, lds_amax);
    } else {
        // This wave's chunks only; the region is private to the wave, whose LDS operations complete in order.
        const int4* xq16 = reinterpret_cast<const int4*>(static_cast<const int8_t*>(xin));
        const int64_t valid = L.K / 4;
        const int64_t own = n_chunks * 8;
        int4* lds_xw = reinterpret_cast<int4*>(xbase);
        for (int64_t u = lane; u < own; u += 64) {
            const int64_t gu = c0 * 8 + u;
            int4 v = make_int4(0, 0, 0, 0);
            if (gu * 4 < valid) v = xq16[gu];
            lds_xw[u] = v;
            int sum = __builtin_amdgcn_sdot4(v.x, 0x01010101, 0, false);
            sum = __builtin_amdgcn_sdot4(v.y, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4(v.z, 0x01010101, sum, false);
            sum = __builtin_amdgcn_sdot4(v.w, 0x01010101, sum, false);
            lds_xs[(u / 8) * 8 + (int)(u % 4) * 2 + (int)(u % 8) / 4] = sum;
        }
    }
    const int64_t cbase = SHARED ? c0 : 0;    // chunk index of the wave's first chunk inside its LDS image

    float accf = 0.0f;
    for (int64_t i = 0; i < n_chunks; i += UNROLL) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const Chunk8Regs& r = cur[u];
            if (i + u < n_chunks) {
                const int64_t cl = cbase + i + u;
                const int4 xa = lds_x[cl * 8 + kb];
                const int4 xb = lds_x[cl * 8 + 4 + kb];
                const int2 xs = *reinterpret_cast<const int2*>(lds_xs + cl * 8 + kb * 2);
                // sum xq q8 = D + 128 xs as an integer (below 2^22: exact in fp32), then the group's two terms as
                // the definition has them - folding the 128 into the minimum instead would add and subtract
                // 128 s xs in fp32, which cancels badly where s is large against min (a constant group: s = 1)
                const int i0 = dot16_bytes(r.w0, xa) + (xs.x << 7);
                const int i1 = dot16_bytes(r.w1, xb) + (xs.y << 7);
                accf = fmaf(r.s.x, (float)i0, accf);
                accf = fmaf(r.s.y, (float)i1, accf);
                accf = fmaf(r.mn.x, (float)xs.x, accf);
                accf = fmaf(r.mn.y, (float)xs.y, accf);
            }
            if (PREFETCH) {
                // a rolling window: the registers of the chunk just consumed take the chunk UNROLL further on
                // (past the wave's range its first chunk again, never used - no branch around the load, so that
                // the compiler waits by count)
                const bool have = i + UNROLL + u < n_chunks;
                cur[u] = load_chunk8(have ? wp : wp - lane, sp, mp, have ? i + UNROLL + u : 0);
            }
        }
        if (!PREFETCH) break;   // the host guarantees n_chunks <= UNROLL
    }

    // Sum over the four k-blocks of the row, then over the KSPLIT waves (fixed order).
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
        float r = accf * ((MODE == kFused) ? scale : sx[0]);
        if (bias) r += bias[n];
        store_out(y, n, r, L.out16);
    }
}

template <int WAVES, int KSPLIT, int UNROLL, int MODE, bool PREFETCH>
int launch_cfg8(const uint8_t* packed, const Layout& L, const void* xin, const float* sx, const float* bias, float* y,
                hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    const int PW = (int)((L.C + KSPLIT - 1) / KSPLIT);
    const size_t smem = (MODE == kFused ? (size_t)L.C * 160 : (size_t)WAVES * PW * 160) + WAVES * 17 * sizeof(float);
    static thread_local int allowed = -1;
    auto kern = decode8_kernel<WAVES, KSPLIT, UNROLL, MODE, PREFETCH>;
    if (int s = allow_large_lds(kern, smem, allowed)) return s;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WAVES * 64), smem, st, packed, L, xin, sx, bias, y, PW);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

template <int WAVES, int KSPLIT, int UNROLL, int MODE, bool PREFETCH, bool EARLY = false>
int launch_cfg(const uint8_t* packed, const Layout& L, int64_t M, const void* xin, const float* sx,
               const float* bias, float* y, int32_t* acc, hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    const int PW = (int)((L.C + KSPLIT - 1) / KSPLIT);
    const size_t smem = (MODE == kFused ? (size_t)L.C * 160 : (size_t)WAVES * PW * 160) + WAVES * 17 * sizeof(float);
    // Rows beyond about 50000 values need more than the 64 KiB of LDS a kernel gets by default.
    static thread_local int allowed_minf = -1, allowed_zp = -1;
    if (L.minf) {
        auto kern = decode_kernel<WAVES, KSPLIT, UNROLL, MODE, PREFETCH, true, EARLY>;
        if (int s = allow_large_lds(kern, smem, allowed_minf)) return s;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks, (unsigned)M), dim3(WAVES * 64), smem, st, packed, L, xin, sx,
                           bias, y, acc, PW);
    } else {
        auto kern = decode_kernel<WAVES, KSPLIT, UNROLL, MODE, PREFETCH, false, EARLY>;
        if (int s = allow_large_lds(kern, smem, allowed_zp)) return s;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks, (unsigned)M), dim3(WAVES * 64), smem, st, packed, L, xin, sx,
                           bias, y, acc, PW);
    }
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

// Configuration: the smallest number of waves per row tile for which a wave's
// chunk range fits in its registers (8, else 12 chunks), so that all loads of
// the layer are issued at once; very long rows fall back to a prefetching loop.
// WAVES is the workgroup size: larger workgroups repeat the staging of the
// activation row less often.
struct DecodeCfg {
    int waves, ks, unroll, prefetch;
    int early;   // activation row handled under the weight stream (see decode_kernel): small layers
};

constexpr int64_t kEarlyMaxBytes = 16 << 20;

DecodeCfg decode_config(const Layout& L, bool fused)
{
    int ks = 1;
    while (ks < 16 && (L.C + ks - 1) / ks > 8) ks *= 2;
    int unroll = 8, prefetch = 0;
    if ((L.C + ks - 1) / ks > 8) {
        if ((L.C + 15) / 16 <= 12) unroll = 12;
        else prefetch = 1;
    }
    // Fused quantizer (eight-wave workgroups) on a layer with at most one row tile per CU: all eight
    // waves on one row tile, so that every tile has a workgroup of its own (o of Qwen2-7B: 6.1 -> 5.3 us).
    if (fused && ks < 8 && L.T <= num_cus() && L.C >= 8) ks = 8;
    if (const char* e = debug_option(kDbgDecodeKsplit)) {   // tests and tuning: force the split
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16) {
            ks = v;
            const int64_t pw = (L.C + ks - 1) / ks;
            unroll = pw <= 8 ? 8 : (pw <= 12 && ks == 16 ? 12 : 8);
            prefetch = pw > unroll;
        }
    }
    // Rows of 28 chunks (K = 3584) on four waves or of 112 (K = 14336) on sixteen: seven chunks each, with no
    // register left unused
    if ((ks == 4 || ks == 16) && L.C == 7 * ks && !prefetch && !debug_option(kDbgDecodeKsplit)) unroll = 7;
    // ... and eight waves on a row tile with at most four chunks each (the fused form of small layers)
    if (fused && ks == 8 && (L.C + 7) / 8 <= 4 && !debug_option(kDbgDecodeKsplit)) unroll = 4;
    int waves = fused ? (ks > 8 ? 16 : 8) : (ks > 4 ? ks : 4);
    if (const char* e = debug_option(kDbgDecodeWaves)) {    // tuning only
        const int v = atoi(e);
        if ((v == 4 || v == 8 || v == 16) && v >= ks) waves = v;
    }
    if (waves < ks) waves = ks;
    // small layers whose waves have at most two chunks fewer than `unroll` (with fewer chunks per wave the
    // form is slower: down of Qwen2-1.5B, 4 - 5 chunks on sixteen waves, 5.1 -> 5.7 us), and those whose
    // waves all have exactly `unroll` chunks (nothing is loaded twice)
    const bool exact = L.C % ks == 0 && L.C / ks == unroll;
    int early = !prefetch && (((int64_t)L.total() <= kEarlyMaxBytes && L.C / ks >= unroll - 2) || exact);
    if (const char* e = debug_option(kDbgDecodeEarly)) early = !prefetch && e[0] == '1';   // tests and tuning
    return DecodeCfg{waves, ks, unroll, prefetch, early};
}

size_t decode_lds_bytes(const Layout& L, const DecodeCfg& c, bool fused)
{
    const int64_t pw = (L.C + c.ks - 1) / c.ks;
    return (fused ? (size_t)L.C * 160 : (size_t)c.waves * pw * 160) + c.waves * 17 * sizeof(float);
}

// Byte form of int8 weights: seven chunks (of two kilobytes) per wave in registers - the smallest power of
// two of waves per row tile that gets there; beyond sixteen waves a rolling window of seven.
DecodeCfg decode8_config(const Layout& L, bool fused)
{
    int ks = 1;
    while (ks < 16 && (L.C + ks - 1) / ks > 7) ks *= 2;
    if (const char* e = debug_option(kDbgDecodeKsplit)) {   // tests and tuning: force the split
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4 || v == 8 || v == 16) ks = v;
    }
    const int prefetch = (L.C + ks - 1) / ks > 7;
    const int waves = fused ? (ks > 8 ? 16 : 8) : (ks > 4 ? ks : 4);
    return DecodeCfg{waves, ks, 7, prefetch, 0};
}

template <int MODE>
int dispatch8(const uint8_t* packed, const Layout& L, const void* xin, const float* sx, const float* bias, float* y,
              hipStream_t st)
{
    const DecodeCfg c = decode8_config(L, MODE == kFused);
#define MNNQ_CFG8(W, K)                                                                                   \
    if (c.waves == W && c.ks == K) {                                                                      \
        if (c.prefetch) return launch_cfg8<W, K, 7, MODE, true>(packed, L, xin, sx, bias, y, st);         \
        return launch_cfg8<W, K, 7, MODE, false>(packed, L, xin, sx, bias, y, st);                        \
    }
    if constexpr (MODE == kFused) {
        MNNQ_CFG8(8, 1) MNNQ_CFG8(8, 2) MNNQ_CFG8(8, 4) MNNQ_CFG8(8, 8) MNNQ_CFG8(16, 16)
    } else {
        MNNQ_CFG8(4, 1) MNNQ_CFG8(4, 2) MNNQ_CFG8(4, 4) MNNQ_CFG8(8, 8) MNNQ_CFG8(16, 16)
    }
#undef MNNQ_CFG8
    return MNNQ_ERR_UNSUPPORTED;
}

template <int MODE>
int dispatch(const uint8_t* packed, const Layout& L, int64_t M, const void* xin, const float* sx,
             const float* bias, float* y, int32_t* acc, hipStream_t st)
{
    if (L.native8) {
        if constexpr (MODE == kAcc) return MNNQ_ERR_UNSUPPORTED;
        else return dispatch8<MODE>(packed, L, xin, sx, bias, y, st);
    }
    const DecodeCfg c = decode_config(L, MODE == kFused);
    const int waves = c.waves, ks = c.ks, unroll = c.unroll, prefetch = c.prefetch;
#define MNNQ_CFG(W, K, U, P)                                                    \
    if (waves == W && ks == K && unroll == U && prefetch == P) {                \
        if constexpr (MODE != kAcc && P == 0) {                                 \
            if (c.early) return launch_cfg<W, K, U, MODE, false, true>(packed, L, M, xin, sx, bias, y, acc, st); \
        }                                                                       \
        return launch_cfg<W, K, U, MODE, (P != 0)>(packed, L, M, xin, sx, bias, y, acc, st); \
    }
#define MNNQ_CFG_W(K, U, P) MNNQ_CFG(4, K, U, P) MNNQ_CFG(8, K, U, P) MNNQ_CFG(16, K, U, P)
    MNNQ_CFG_W(1, 8, 0) MNNQ_CFG_W(2, 8, 0) MNNQ_CFG_W(4, 8, 0) MNNQ_CFG_W(4, 7, 0)
    MNNQ_CFG(8, 8, 8, 0) MNNQ_CFG(8, 8, 4, 0) MNNQ_CFG(16, 8, 8, 0) MNNQ_CFG(16, 16, 8, 0) MNNQ_CFG(16, 16, 7, 0) MNNQ_CFG(16, 16, 12, 0)
    MNNQ_CFG_W(1, 8, 1) MNNQ_CFG_W(2, 8, 1) MNNQ_CFG_W(4, 8, 1)
    MNNQ_CFG(8, 8, 8, 1) MNNQ_CFG(16, 8, 8, 1) MNNQ_CFG(16, 16, 8, 1)
#undef MNNQ_CFG_W
#undef MNNQ_CFG
    return MNNQ_ERR_UNSUPPORTED;
}

}  // namespace

void describe_decode(const Layout& L, bool fused, int32_t out[8])
{
    const DecodeCfg c = L.native8 ? decode8_config(L, fused) : decode_config(L, fused);
    const int tiles_per_wg = c.waves / c.ks;
    out[0] = c.waves;
    out[1] = c.ks;
    out[2] = c.unroll;
    out[3] = c.prefetch;
    out[4] = (int32_t)decode_lds_bytes(L, c, fused);
    out[5] = (int32_t)((L.T + tiles_per_wg - 1) / tiles_per_wg);   // workgroups
    out[6] = tiles_per_wg;
    out[7] = c.early;
}

int launch_decode(const uint8_t* packed, const Layout& L, const int8_t* xq, const float* sx,
                  const float* bias, float* y, hipStream_t st)
{
    return dispatch<kXQ>(packed, L, 1, xq, sx, bias, y, nullptr, st);
}

int launch_decode_fused(const uint8_t* packed, const Layout& L, const float* x, const float* bias, float* y,
                        hipStream_t st)
{
    return dispatch<kFused>(packed, L, 1, x, nullptr, bias, y, nullptr, st);
}

int launch_decode_acc(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, int32_t* acc,
                      hipStream_t st)
{
    // Same inner loop as the decode kernel, one grid row per token.
    return dispatch<kAcc>(packed, L, M, xq, nullptr, nullptr, nullptr, acc, st);
}

}  // namespace mnnq
