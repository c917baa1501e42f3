// W4A16 variants (Section 4.2: on GPUs the int4 weights are combined with
// fp16 activations to use the floating-point units): same packed weights,
// activations stay fp16, accumulation in fp32.
//
//   y[m,n] = sum_g scale[n,g] * sum_{k in g} float(x16[m,k]) * (q[n,k] - zero[n,g]) (+ bias[n])
//
// The integer q - z (|.| <= 15) is exact in fp16, so the weights enter the
// contraction without rounding and the group scale is applied once per group
// in fp32.  Codes become fp16 two at a time: (0x6400 | q) is the half 1024 + q,
// and subtracting the half 1024 + z leaves q - z exactly.
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
    uint32_t z;
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

template <int WAVES, int KSPLIT, int UNROLL>
__global__ __launch_bounds__(WAVES * 64) void decode_f16_kernel(const uint8_t* __restrict__ packed, Layout L,
                                                                const uint16_t* __restrict__ x16,
                                                                const float* __restrict__ bias,
                                                                float* __restrict__ y)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int64_t C = L.C;
    uint4* lds_x = reinterpret_cast<uint4*>(smem);                 // C * 128 halves, permuted by 8
    float* lds_part = reinterpret_cast<float*>(smem + C * 256);    // [WAVES][16]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane & 15;
    const int kb = lane >> 4;
    constexpr int TILES_PER_WG = WAVES / KSPLIT;
    const int64_t tile = (int64_t)blockIdx.x * TILES_PER_WG + wave / KSPLIT;
    const int ks = wave % KSPLIT;
    const bool active = tile < L.T;
    const int64_t c0 = C * ks / KSPLIT;
    const int64_t c1 = C * (ks + 1) / KSPLIT;
    const u32x4* wp = reinterpret_cast<const u32x4*>(packed) + (tile * C + c0) * 64 + lane;
    const float2* sp = reinterpret_cast<const float2*>(packed + L.scales_off()) + (tile * C + c0) * 16 + row;
    const uint16_t* zp = reinterpret_cast<const uint16_t*>(packed + L.zeros_off()) + (tile * C + c0) * 16 + row;
    const int64_t n_chunks = active ? (c1 - c0) : 0;

    ChunkRegs cur[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        if (u < n_chunks) cur[u] = load_chunk(wp, sp, zp, u);
        else cur[u] = ChunkRegs{};
    }

    // Stage x: units of 8 halves (16 B), zero padded to C * 16 units.
    {
        const int64_t units = C * 16;
        const int64_t valid = L.K / 8;
        for (int64_t u = tid; u < units; u += WAVES * 64) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (u < valid) v = reinterpret_cast<const uint4*>(x16)[u];
            lds_x[u] = permute8(v);
        }
    }
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
                // 16-byte unit index of x[128 c + 64 h + 16 kb]: (128 c + 64 h + 16 kb) / 8
                const uint4* xp = lds_x + c * 16 + kb * 2;
                const ChunkRegs& r = cur[u];
                const float p0 = dot16_f16(r.w.x, r.w.y, r.z & 0xffu, xp[0], xp[1]);
                const float p1 = dot16_f16(r.w.z, r.w.w, r.z >> 8, xp[8], xp[9]);
                accf = fmaf(r.s.x, p0, accf);
                accf = fmaf(r.s.y, p1, accf);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) cur[u] = nxt[u];
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
        y[n] = r;
    }
}

template <int WAVES, int KSPLIT, int UNROLL>
int launch_decode_cfg(const uint8_t* packed, const Layout& L, const uint16_t* x16, const float* bias,
                      float* y, hipStream_t st)
{
    constexpr int tiles_per_wg = WAVES / KSPLIT;
    const int64_t blocks = (L.T + tiles_per_wg - 1) / tiles_per_wg;
    const size_t smem = (size_t)L.C * 256 + WAVES * 16 * sizeof(float);
    hipLaunchKernelGGL((decode_f16_kernel<WAVES, KSPLIT, UNROLL>), dim3((unsigned)blocks), dim3(WAVES * 64),
                       smem, st, packed, L, x16, bias, y);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

// ---------------------------------------------------------------- prefill

constexpr int kAStride = 144;  // bytes per LDS row: 64 halves + 16 B padding

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(WGM * WGN * 64) void prefill_f16_kernel(const uint8_t* __restrict__ packed,
                                                                     Layout L, int64_t M,
                                                                     const uint16_t* __restrict__ x16,
                                                                     const float* __restrict__ bias,
                                                                     float* __restrict__ y, int MT, int NT)
{
    constexpr int THREADS = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int A_UNITS = BM * 8;  // one stage = one group: 64 halves = 8 units of 16 B per row
    constexpr int A_PER_THREAD = A_UNITS / THREADS;
    static_assert(A_UNITS % THREADS == 0, "A tile must split evenly");

    __shared__ __align__(16) uint8_t lds_a[2][BM * kAStride];

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
    const int64_t S = 2 * C;  // stages (groups, including a padding group)

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

    auto load_a = [&](int64_t s) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            const int u = tid + i * THREADS;
            const int r = u / 8, cu = u % 8;
            const int64_t m = m0 + r;
            const int64_t k = s * 64 + cu * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m < M && k < L.K) v = *reinterpret_cast<const uint4*>(x16 + m * L.K + k);
            areg[i] = permute8(v);
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

    for (int64_t s = 0; s < S; ++s) {
        const int buf = (int)(s & 1);
        const int h = buf;
        __syncthreads();
        const bool more = s + 1 < S;
        if (more) load_a(s + 1);
        if (h == 1 && more) load_b((s + 1) / 2, bw_n, bs_n, bz_n);

        h8 b0[TN], b1[TN];
        float sc[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const uint32_t zz = h ? (bz[j] >> 8) : (bz[j] & 0xffu);
            const _Float16 zh = (_Float16)(float)(1024u + zz);
            const h2 zb = {zh, zh};
            const uint32_t w0 = h ? bw[j].z : bw[j].x;
            const uint32_t w1 = h ? bw[j].w : bw[j].y;
            h2 p;
            p = code_pair(w0, 0, zb); b0[j][0] = p[0]; b0[j][1] = p[1];
            p = code_pair(w0, 1, zb); b0[j][2] = p[0]; b0[j][3] = p[1];
            p = code_pair(w0, 2, zb); b0[j][4] = p[0]; b0[j][5] = p[1];
            p = code_pair(w0, 3, zb); b0[j][6] = p[0]; b0[j][7] = p[1];
            p = code_pair(w1, 0, zb); b1[j][0] = p[0]; b1[j][1] = p[1];
            p = code_pair(w1, 1, zb); b1[j][2] = p[0]; b1[j][3] = p[1];
            p = code_pair(w1, 2, zb); b1[j][4] = p[0]; b1[j][5] = p[1];
            p = code_pair(w1, 3, zb); b1[j][6] = p[0]; b1[j][7] = p[1];
            sc[j] = h ? bs[j].y : bs[j].x;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = wm * WM + i * 16 + col;
            // The lane's 16 activations of this group: halves 16 kb .. 16 kb + 15.
            const h8 a0 = *reinterpret_cast<const h8*>(&lds_a[buf][r * kAStride + kb * 32]);
            const h8 a1 = *reinterpret_cast<const h8*>(&lds_a[buf][r * kAStride + kb * 32 + 16]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                v4f d = {0.0f, 0.0f, 0.0f, 0.0f};
                d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, b0[j], d, 0, 0, 0);
                d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, b1[j], d, 0, 0, 0);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) yacc[i][j][rr] = fmaf(sc[j], d[rr], yacc[i][j][rr]);
            }
        }
        if (more) store_a(buf ^ 1);
        if (h == 1 && more) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                bw[j] = bw_n[j];
                bs[j] = bs_n[j];
                bz[j] = bz_n[j];
            }
        }
    }

#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int64_t m = m0 + wm * WM + i * 16 + kb * 4 + rr;
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (!b_ok[j]) continue;
                const int64_t n = (rt0 + j) * 16 + col;
                float v = yacc[i][j][rr];
                if (bias) v += bias[n];
                y[m * L.N + n] = v;
            }
        }
    }
}

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

int launch_decode_f16(const uint8_t* packed, const Layout& L, const uint16_t* x16, const float* bias,
                      float* y, hipStream_t st)
{
    switch (pick_ksplit(L)) {
        case 1:  return launch_decode_cfg<4, 1, 4>(packed, L, x16, bias, y, st);
        case 2:  return launch_decode_cfg<4, 2, 4>(packed, L, x16, bias, y, st);
        case 4:  return launch_decode_cfg<4, 4, 4>(packed, L, x16, bias, y, st);
        case 8:  return launch_decode_cfg<8, 8, 4>(packed, L, x16, bias, y, st);
        default: return launch_decode_cfg<16, 16, 4>(packed, L, x16, bias, y, st);
    }
}

int launch_prefill_f16(const uint8_t* packed, const Layout& L, int64_t M, const uint16_t* x16,
                       const float* bias, float* y, hipStream_t st)
{
    constexpr int BM = 128, BN = 128;
    const int MT = (int)((M + BM - 1) / BM);
    const int NT = (int)((L.N + BN - 1) / BN);
    const int64_t blocks = (int64_t)MT * ((NT + 7) / 8) * 8;
    hipLaunchKernelGGL((prefill_f16_kernel<BM, BN, 2, 2>), dim3((unsigned)blocks), dim3(256), 0, st, packed, L,
                       M, x16, bias, y, MT, NT);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

}  // namespace mnnq
