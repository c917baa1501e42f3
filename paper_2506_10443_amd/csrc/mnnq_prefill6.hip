// Prefill (M tokens) on the fp6 matrix instructions of gfx950 (Section 2.1: the compute-bound phase;
// Section 5.1: operands rearranged once so that the inner loop reads what one instruction consumes).
//
//   y[m,n] = sx[m] * sum_g scale[n,g] * I[m,n,g] (+ bias[n]),   I = sum_{k in g} xq[m,k] (q[n,k] - zero[n,g])
//
// Why not the int8 instruction: its int32 result needs two vector operations per output and group
// (to fp32, multiply-add with the group's scale), and on this chip a SIMD issues vector and matrix
// instructions one after the other, not side by side - the epilogue, not the matrix pipe, sets the
// pace.  v_mfma_scale_f32_32x32x64_f8f6f4 with fp6 (e2m3) operands runs at the same rate per group as the
// int8 form and delivers the group sum in fp32, which leaves one multiply-add per output and group:
//   * an e2m3 number is (-1)^s * m / 8 for m = 0..15 (and coarser above), so every integer of
//     magnitude <= 15 is exact: the weight operand is (q - zero) / 8, its code the sign-magnitude
//     form of q - zero;
//   * an int8 activation is split as xq = sign(xq) (16 hi + lo) with hi = |xq| >> 4 (0..8) and
//     lo = |xq| & 15, both parts signed like xq and exact as well (the split by magnitude rather than
//     by two's-complement bits leaves the high part of every small value - nearly all of them, once a
//     token has an outlier - an all-zero code: fewer bits toggle in the matrix pipe, and the chip,
//     which runs this kernel against its power limit, clocks higher); one instruction contracts the 64 high parts of a group with the
//     weights, a second one the low parts, accumulating on the first; the instruction's power-of-two
//     operand scale (2^10 resp. 2^6 on the activation side) puts back the 16 and the two divisions by 8;
//   * all products and the sums (|I| <= 64 * 127 * 15 < 2^17) are integers, exact in fp32, so the
//     result is the int32 group accumulator, bit for bit (the accumulator dump of this kernel is
//     compared with the oracle's integers).
// Both operands are prepared ahead: the weights at load time (the matrix-core plane of the packed
// buffer, see mnnq_common.h), the activations by a small kernel per call (planes_kernel below), so
// the GEMM's loop holds nothing but LDS reads, matrix instructions and the multiply-adds.
//
// Lane mapping of the 32x32x64 instruction as used here (A: 32 x 64, B: 64 x 32, D: 32 x 32):
//   A / B operand: lane l holds row / column l % 32 and the 32 values of k-block l / 32, value j at
//                  bits [6 j, 6 j + 6) of six registers; one scale byte per lane covers its 32 values;
//   D: lane l holds column l % 32, rows 8 (r / 4) + 4 (l / 32) + r % 4 for r = 0..15.
#include "mnnq_common.h"

#include <type_traits>

namespace mnnq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define MNNQ_LDS(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int kBufFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)
constexpr int kOutOfRange = 0x7ffffff0; // a byte offset beyond every buffer: loads give 0, stores are dropped

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---------------------------------------------------------------------------------------------
// fp6 packing.  c[0..7]: 32 six-bit codes, one per byte, code j in byte j % 4 of c[j / 4].
// out[0..5]: the same codes at bits [6 j, 6 j + 6).
__device__ __forceinline__ uint32_t pack24(uint32_t c)
{
    return (c & 0x3fu) | ((c >> 2) & 0xfc0u) | ((c >> 4) & 0x3f000u) | ((c >> 6) & 0xfc0000u);
}

__device__ __forceinline__ void pack_fp6(const uint32_t (&c)[8], uint32_t (&out)[6])
{
    const uint32_t p0 = pack24(c[0]), p1 = pack24(c[1]), p2 = pack24(c[2]), p3 = pack24(c[3]);
    const uint32_t p4 = pack24(c[4]), p5 = pack24(c[5]), p6 = pack24(c[6]), p7 = pack24(c[7]);
    out[0] = p0 | (p1 << 24);
    out[1] = (p1 >> 8) | (p2 << 16);
    out[2] = (p2 >> 16) | (p3 << 8);
    out[3] = p4 | (p5 << 24);
    out[4] = (p5 >> 8) | (p6 << 16);
    out[5] = (p6 >> 16) | (p7 << 8);
}

// Sign-magnitude six-bit codes of four small integers held as bytes 0x80 + v (|v| <= 15).
__device__ __forceinline__ uint32_t signmag_from_biased(uint32_t b)
{
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int v = (int)((b >> (8 * i)) & 0xffu) - 0x80;
        const uint32_t code = v < 0 ? (32u | (uint32_t)(-v)) : (uint32_t)v;
        r |= code << (8 * i);
    }
    return r;
}

// One block (1536 B) of a plane: six dwords per lane, dwords 0..3 of lane l at 16 l, dwords 4..5 at
// 1024 + 8 l - a kilobyte of 16-byte units and half a kilobyte of 8-byte units, both read without
// bank conflicts.
__device__ __forceinline__ void store_block(uint8_t* block, int lane, const uint32_t (&d)[6])
{
    *reinterpret_cast<uint4*>(block + lane * 16) = make_uint4(d[0], d[1], d[2], d[3]);
    *reinterpret_cast<uint2*>(block + 1024 + lane * 8) = make_uint2(d[4], d[5]);
}

// ---------------------------------------------------------------------------------------------
// Load time: the matrix-core plane from the chunk layout in front of it (one wave per group and
// column tile of 32).
__global__ __launch_bounds__(256) void plane_build_kernel(uint8_t* __restrict__ packed, Layout L)
{
    const int lane = threadIdx.x & 63;
    const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (blk >= L.Gx * L.T32p) return;
    // (the few bytes between the chunk layout and the plane's 256-byte boundary: zero, so that equal
    // weights give equal buffers)
    if (blk == 0)
        for (size_t i = L.total() + lane; i < L.plane_off(); i += 64) packed[i] = 0;
    const int64_t g = blk / L.T32p, tn = blk % L.T32p;
    const int col = lane & 31, kb = lane >> 5;
    const int64_t n = tn * 32 + col;
    uint32_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float scale = 0.0f;
    if (n < L.N) {
        const int64_t t16 = n / 16, chunk = g / 2;
        const int r16 = (int)(n % 16), h = (int)(g & 1);
        const int64_t cell = t16 * L.C + chunk;
        const uint32_t z = packed[L.zeros_off() + (cell * 16 + r16) * 2 + h];
        scale = *reinterpret_cast<const float*>(packed + L.scales_off() + (cell * 16 + r16) * 8 + h * 4);
        const uint32_t bias4 = 0x80808080u - z * 0x01010101u;     // 0x80 - zero in every byte
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int lane16 = r16 + 16 * (2 * kb + half);
            const uint2 w = *reinterpret_cast<const uint2*>(packed + (cell * 64 + lane16) * 16 + 8 * h);
            c[half * 4 + 0] = signmag_from_biased((w.x & 0x0f0f0f0fu) + bias4);
            c[half * 4 + 1] = signmag_from_biased(((w.x >> 4) & 0x0f0f0f0fu) + bias4);
            c[half * 4 + 2] = signmag_from_biased((w.y & 0x0f0f0f0fu) + bias4);
            c[half * 4 + 3] = signmag_from_biased(((w.y >> 4) & 0x0f0f0f0fu) + bias4);
        }
    }
    uint32_t d[6];
    pack_fp6(c, d);
    uint8_t* plane = packed + L.plane_off();
    store_block(plane + blk * kPlaneBlockBytes, lane, d);
    if (lane < 32) *reinterpret_cast<float*>(plane + L.plane_codes_bytes() + blk * 128 + lane * 4) = scale;
}

// ---------------------------------------------------------------------------------------------
// Per call: the activation planes [Gx][TMp][2][1536 B] from the int8 codes [M, K] - block (g, tm, 0)
// the high parts, block (g, tm, 1) the low parts of xq = sign(xq) (16 hi + lo), hi = |xq| >> 4,
// lo = |xq| & 15, both carrying the sign of xq (so that small values have an all-zero high part), of rows 32 tm .. 32 tm + 31
// and group g, lane l holding row l % 32 and k = 64 g + 32 (l / 32) + j.  Rows past M are zero.
// One wave per (tm, g); consecutive waves take consecutive groups of the same rows, so that the
// 128-byte lines of xq (two groups each) are fetched once.
__global__ __launch_bounds__(256) void planes_kernel(const int8_t* __restrict__ xq, int64_t M, int64_t K, int Gx,
                                                     int TMp, uint8_t* __restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (int64_t)Gx * TMp) return;
    const int64_t tm = wid / Gx, g = wid % Gx;
    const int64_t m = tm * 32 + (lane & 31);
    uint32_t x[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (m < M) {
        const uint4* p = reinterpret_cast<const uint4*>(xq + m * K + g * 64 + (lane >> 5) * 32);
        const uint4 a = p[0], b = p[1];
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    uint32_t hi[8], lo[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // byte-wise: xq = s (16 hi + lo) with s = +-1, hi = |xq| >> 4 (0..8), lo = |xq| & 15; the code of a
        // part is its magnitude with the sign in bit 5, zero parts stay all-zero codes
        const uint32_t neg = (x[i] >> 7) & 0x01010101u;           // 1 in the bytes with xq < 0
        const uint32_t mag = (x[i] ^ (neg * 255u)) + neg;         // |xq| (at most 128: no carry between bytes)
        const uint32_t ml = mag & 0x0f0f0f0fu, mh = (mag >> 4) & 0x0f0f0f0fu;
        const uint32_t nzl = ((ml + 0x0f0f0f0fu) >> 4) & 0x01010101u, nzh = ((mh + 0x0f0f0f0fu) >> 4) & 0x01010101u;
        lo[i] = ml | ((neg & nzl) << 5);
        hi[i] = mh | ((neg & nzh) << 5);
    }
    uint32_t dh[6], dl[6];
    pack_fp6(hi, dh);
    pack_fp6(lo, dl);
    uint8_t* block = out + ((g * TMp + tm) * 2) * (int64_t)kPlaneBlockBytes;
    store_block(block, lane, dh);
    store_block(block + kPlaneBlockBytes, lane, dl);
}

// ---------------------------------------------------------------------------------------------
// The GEMM.  Workgroup tile BM x BN, K range in KS parts of WM x WN waves each; a wave owns
// TMW x TNW tiles of 32 x 32.  Per group (stage): BM * 96 bytes of activation planes, BN * 48 bytes
// of weight plane and BN scales travel verbatim from memory to LDS with direct 128-bit loads, two
// stages per K part.  The loop is software pipelined over the groups: while group g is contracted,
// every fragment (six registers per lane) is refilled from the stage of group g + 1 right after the
// matrix instruction that used it last, so the LDS reads run between the matrix instructions; at the
// top of a group one barrier makes the stage of g + 1 visible and frees the stage of g for the direct
// loads of g + 2.
template <int BM, int BN, int NS = 2>
struct Stage {
    static constexpr int A_BYTES = BM * 96;
    static constexpr int B_BYTES = BN * 48;
    static constexpr int S_BYTES = (BN * 4 + 1023) / 1024 * 1024;   // BN scales in whole wave-wide loads
    static constexpr int W_BYTES = B_BYTES + S_BYTES;                // weight side of a stage: codes, then scales
    // The activation side is a ring of NS stages (NS - 1 groups in flight or ready beside the one whose
    // fragments are in registers), the weight side a ring of NS or - for wave tiles of more than four column
    // tiles, whose weight fragments are still read while their group is contracted - of NS + 1.
    static constexpr int NRING_A = NS;
    static constexpr int NRING_W = (BN / 32 > 8) ? NS + 1 : NS;
    static constexpr int W_RING_OFF = NRING_A * A_BYTES;
    static constexpr int BYTES = NRING_A * A_BYTES + NRING_W * W_BYTES;    // all stages of one K part
    static constexpr int NA = A_BYTES / 1024, NB = B_BYTES / 1024, NSC = S_BYTES / 1024;
    static_assert(A_BYTES % 1024 == 0 && B_BYTES % 1024 == 0, "whole wave-wide loads");
};

// LDS of a workgroup: two stages per K part and the junk kilobyte, or the K parts' sums when those
// need more (they are exchanged after the last stage is dead).
template <int BM, int BN, int KS, int NS = 2>
constexpr size_t lds_bytes6()
{
    const size_t stages = (size_t)KS * Stage<BM, BN, NS>::BYTES + 1024;
    const size_t sums = KS > 1 ? (size_t)(BM / 32) * (BN / 32) * 16 * 64 * 4 : 0;
    return stages > sums ? stages : sums;
}

// A fragment (six registers) from a block in LDS; off16 = 16 lane, off8 = 8 lane.  Neighbouring blocks
// are read with two copies of off8 that the compiler cannot tell to be equal: it would otherwise merge
// their 8-byte reads into one instruction whose four result registers belong to two fragments, and
// pay for that with register copies in the loop.
__device__ __forceinline__ v8i frag6(const uint8_t* block, int off16, int off8)
{
    const v4i p0 = *reinterpret_cast<const v4i*>(block + off16);
    const v2i p1 = *reinterpret_cast<const v2i*>(block + 1024 + off8);
    return v8i{p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, 0, 0};
}

// D = A x B + C on fp6 (e2m3) operands with per-lane power-of-two operand scales.
__device__ __forceinline__ v16f mfma6(v8i a, v8i b, v16f c, int scale_a, int scale_b)
{
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 2, 2, 0, scale_a, 0, scale_b);
}

template <int BM, int BN, int WM, int WN, int KS, bool ACC, int NS = 2>
__global__ __launch_bounds__(64 * WM * WN * KS, 2) void prefill6_kernel(
    const uint8_t* __restrict__ plane, const uint8_t* __restrict__ a6, Layout L, int64_t M, int TMp,
    const float* __restrict__ sx, const float* __restrict__ bias, float* __restrict__ y,
    int32_t* __restrict__ acc_out, int MT, int NT)
{
    using St = Stage<BM, BN, NS>;
    constexpr int W = WM * WN;                        // waves per K part
    constexpr int TMW = BM / WM / 32, TNW = BN / WN / 32;
    constexpr int NL = (St::NA + St::NB + St::NSC + W - 1) / W;   // direct loads per wave and stage
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "whole 32 x 32 tiles per wave");

    extern __shared__ __align__(16) uint8_t lds_all[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = uniform(tid >> 6);
    const int part = wave_id / W;                    // K part of this wave
    const int w = wave_id % W;
    const int wm = w / WN, wn = w % WN;
    uint8_t* const lds = lds_all + part * St::BYTES;
    uint8_t* const junk = lds_all + KS * St::BYTES;
    // stage of group k (counted from this part's first group): activation side, weight side
    auto stage_a = [&](int k) { return lds + (k % St::NRING_A) * St::A_BYTES; };
    auto stage_w = [&](int k) { return lds + St::W_RING_OFF + (k % St::NRING_W) * St::W_BYTES; };
    // s_waitcnt for "at most n of this wave's vector-memory operations outstanding, no LDS operation":
    // vmcnt in bits 3:0 and 15:14, lgkmcnt(0), expcnt left alone - the loads of the NS - 2 youngest stages
    // may stay in flight at the top of a group
    constexpr int kInFlight = (NS - 2) * NL;
    static_assert(kInFlight < 64, "six bits of vmcnt");
    constexpr int kWaitTop = 0x0070 | (kInFlight & 15) | ((kInFlight >> 4) << 14);
    constexpr int kFirst = (NS - 1) * NL;             // prologue: all but the first stage may still be in flight
    static_assert(kFirst < 64, "six bits of vmcnt");
    constexpr int kWaitFirst = 0x0F70 | (kFirst & 15) | ((kFirst >> 4) << 14);

    // Workgroups are dealt to the 8 XCDs round-robin by their linear id: each XCD gets whole columns
    // of output tiles, so that a block of weights is fetched into one L2 only.
    const int xcd = blockIdx.x % 8;
    const int seq = blockIdx.x / 8;
    const int tile_m = seq % MT;
    const int tile_n = (seq / MT) * 8 + xcd;
    if (tile_n >= NT) return;
    const int G = (int)L.Gx;
    const int gb = G * part / KS, ge = G * (part + 1) / KS;      // this part's groups
    const int n_iter = (G + KS - 1) / KS;                        // the longest share: every wave runs the same barriers

    const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(a6), 0, (int)((int64_t)G * TMp * 2 * kPlaneBlockBytes), kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(plane), 0, (int)L.plane_bytes(), kBufFlags);

    const int a_base = tile_m * (BM / 32) * 2 * kPlaneBlockBytes, a_step = TMp * 2 * kPlaneBlockBytes;
    const int w_base = tile_n * (BN / 32) * kPlaneBlockBytes, w_step = (int)L.T32p * kPlaneBlockBytes;
    const int s_base = (int)L.plane_codes_bytes() + tile_n * (BN / 32) * 128, s_step = (int)L.T32p * 128;
    const int voff = lane * 16;

    // Stage of the part's group k <- group gb + k: this wave's NL pieces of 1 KiB (with more than two stages,
    // whose waits count loads, slots past the stage's pieces go to a junk kilobyte with an out-of-range
    // source, so that every wave issues the same number of loads).  Groups past the end of the matrix lie outside the buffers and arrive as zeros.
    auto issue_stage = [&](int k) {
        const int g = gb + k;
        uint8_t* sta = stage_a(k);
        uint8_t* stw = stage_w(k);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int s = w + W * i;   // wave-uniform
            // (the offsets are named before the calls: with the expressions written into a 128-bit direct
            // load's argument list this toolchain's host pass drops the kernel without a message)
            const int so_a = uniform(a_base + g * a_step + s * 1024);
            const int so_w = uniform(w_base + g * w_step + (s - St::NA) * 1024);
            // (scales: a kilobyte past the tile's own columns holds the next tiles' scales or lies outside the
            // buffer; nobody reads that part of the stage)
            const int so_s = uniform(s_base + g * s_step + (s - St::NA - St::NB) * 1024);
            const int so_ws = s < St::NA + St::NB ? so_w : so_s;
            if (s < St::NA)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, MNNQ_LDS(sta + s * 1024), 16, voff, so_a, 0, 0);
            else if (s < St::NA + St::NB + St::NSC)   // codes, then scales: consecutive in the stage
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(stw + (s - St::NA) * 1024), 16, voff, so_ws, 0, 0);
            else if (NS > 2)   // (two stages: the waits are for all loads, nothing is counted)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(junk), 16, voff, kOutOfRange, 0, 0);
        }
    };

    float yacc[TMW * TNW][16];
#pragma unroll
    for (int t = 0; t < TMW * TNW; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) yacc[t][r] = 0.0f;

    // operand scales (one byte per lane, 2^(b - 127)): operands are value / 8 each, the high parts weigh 16
    int scale_hi = 127 + 10, scale_lo = 127 + 6, scale_b = 127;
    asm volatile("" : "+v"(scale_hi), "+v"(scale_lo), "+v"(scale_b));
    const v16f zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // this wave's fragments inside a stage
    const int a_frag = (wm * TMW) * 2 * kPlaneBlockBytes;                    // in the activation side
    const int b_frag = (wn * TNW) * kPlaneBlockBytes;                        // in the weight side
    const int s_frag = St::B_BYTES + (wn * TNW) * 128 + (lane & 31) * 4;

    const int off16 = lane * 16, off8 = lane * 8;
    int off8x = off8;
    asm volatile("" : "+v"(off8x));   // the same value, unknown to the compiler (see frag6)

    // Wide wave tiles (more than four column tiles): the column-major loop below, which holds two weight
    // fragments at a time instead of all TNW - all of them plus the accumulators would not fit 256 registers.
    constexpr bool JO = TNW > 4;
    static_assert(!JO || (KS == 1 && !ACC), "the column-major loop is built for one K part");
    v8i ahi[TMW], alo[TMW], b[JO ? 2 : TNW];
    float sc[JO ? 2 : TNW], scn[JO ? 1 : TNW];
    auto read_a = [&](const uint8_t* st, int i) {
        ahi[i] = frag6(st + a_frag + i * 2 * kPlaneBlockBytes, off16, off8);
        alo[i] = frag6(st + a_frag + i * 2 * kPlaneBlockBytes + kPlaneBlockBytes, off16, off8x);
    };
    auto read_b = [&](const uint8_t* st, int j) {
        b[j] = frag6(st + b_frag + j * kPlaneBlockBytes, off16, (j & 1) ? off8x : off8);
    };

    if constexpr (JO) {
        // Column-major order over the wave's tiles: column j's fragment sits in slot (j + PAR) & 1 and is
        // replaced, after its last use, by the fragment two columns further on - of this group or of the next
        // one (stage g + 1).  With an odd TNW the slot of column 0 alternates from group to group, hence two
        // copies of the group body (PAR = 0, 1).  The multiply-adds of a tile run behind the matrix
        // instructions of the next one, so a column's scale is replaced only after the multiply-adds of its
        // last tile.
        auto read_bs = [&](const uint8_t* st, int j, int slot) {
            b[slot] = frag6(st + b_frag + j * kPlaneBlockBytes, off16, (slot & 1) ? off8x : off8);
        };
        auto read_sc = [&](const uint8_t* st, int j) { return *reinterpret_cast<const float*>(st + s_frag + j * 128); };
        if (NS > 2) {
            // all NS stages are requested at once; the first one is waited for (by count: every wave issues NL
            // loads per stage)
#pragma unroll
            for (int s = 0; s < NS; ++s) issue_stage(s);
            __builtin_amdgcn_s_waitcnt(kWaitFirst);
            __builtin_amdgcn_s_barrier();
        } else {
            issue_stage(0);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __builtin_amdgcn_s_barrier();
            issue_stage(1);
        }
        read_bs(stage_w(0), 0, 0);
        read_bs(stage_w(0), 1, 1);
        sc[0] = read_sc(stage_w(0), 0);
        sc[1] = read_sc(stage_w(0), 1);
#pragma unroll
        for (int i = 0; i < TMW; ++i) read_a(stage_a(0), i);

        auto group = [&](auto par_c, int it) {
            constexpr int PAR = decltype(par_c)::value;
            __builtin_amdgcn_s_waitcnt(kWaitTop);   // stage it + 1 has landed; no LDS read of this wave is open
            __builtin_amdgcn_s_barrier();
            // Top of group `it`: its activation fragments and the weight fragments of its first two columns
            // are in registers (or on their way); its other columns are read from its weight stage as it
            // goes, which therefore stays untouched until the next barrier - the loads of group it + NS go to the
            // extra stage of the weight ring and to the activation stage this group has been read out of.
            issue_stage(it + NS);
            const uint8_t* cu = stage_w(it);          // weight side of this group
            const uint8_t* nx = stage_w(it + 1);      // ... and of the next one
            const uint8_t* nxa = stage_a(it + 1);
            v16f d[2];
#pragma unroll
            for (int t = 0; t < TMW * TNW; ++t) {
                const int j = t / TMW, i = t % TMW;
                const int slot = (j + PAR) & 1;
                d[t & 1] = mfma6(ahi[i], b[slot], zero16, scale_hi, scale_b);
                d[t & 1] = mfma6(alo[i], b[slot], d[t & 1], scale_lo, scale_b);
                if (j == TNW - 1) read_a(nxa, i);
                if (i == TMW - 1) {
                    if (j + 2 < TNW) read_bs(cu, j + 2, slot);
                    else read_bs(nx, j + 2 - TNW, slot);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (t > 0) {
                    const int tp = t - 1, jp = tp / TMW, ip = tp % TMW, sp = (jp + PAR) & 1;
#pragma unroll
                    for (int r = 0; r < 16; ++r) yacc[ip * TNW + jp][r] = fmaf(sc[sp], d[tp & 1][r], yacc[ip * TNW + jp][r]);
                    if (ip == TMW - 1) sc[sp] = (jp + 2 < TNW) ? read_sc(cu, jp + 2) : read_sc(nx, jp + 2 - TNW);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            {
                constexpr int tp = TMW * TNW - 1, jp = tp / TMW, ip = tp % TMW, sp = (jp + PAR) & 1;
#pragma unroll
                for (int r = 0; r < 16; ++r) yacc[ip * TNW + jp][r] = fmaf(sc[sp], d[tp & 1][r], yacc[ip * TNW + jp][r]);
                sc[sp] = read_sc(nx, jp + 2 - TNW);
            }
        };
        for (int it = 0; it < n_iter; it += 2) {
            group(std::integral_constant<int, 0>{}, it);
            if (it + 1 < n_iter) group(std::integral_constant<int, (TNW & 1)>{}, it + 1);
        }
    } else {
        if (NS > 2) {
            // all NS stages are requested at once; the first one is waited for (by count: every wave issues NL
            // loads per stage)
#pragma unroll
            for (int s = 0; s < NS; ++s) issue_stage(s);
            __builtin_amdgcn_s_waitcnt(kWaitFirst);
            __builtin_amdgcn_s_barrier();
        } else {
            issue_stage(0);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __builtin_amdgcn_s_barrier();
            issue_stage(1);
        }
#pragma unroll
        for (int j = 0; j < TNW; ++j) {
            read_b(stage_w(0), j);
            sc[j] = *reinterpret_cast<const float*>(stage_w(0) + s_frag + j * 128);
        }
#pragma unroll
        for (int i = 0; i < TMW; ++i) read_a(stage_a(0), i);

        for (int it = 0; it < n_iter; ++it) {
            const int g = gb + it;
            // Top of group g: its fragments are in registers (or on their way).  Once this wave's reads of
            // the stage they came from and its pieces of the next stage are complete, and every other
            // wave's too, the old stage can be loaded over (with group g + NS) and the next one read.
            __builtin_amdgcn_s_waitcnt(kWaitTop);   // all but the loads of the NS - 2 youngest stages, and the LDS reads
            __builtin_amdgcn_s_barrier();
            issue_stage(it + NS);
            if (KS > 1 && g >= ge) continue;      // the shorter share idles through the last round
            const uint8_t* nx = stage_w(it + 1);   // stage of group g + 1: weight side
            const uint8_t* nxa = stage_a(it + 1);  // ... and activation side

            v16f d[2];
#pragma unroll
            for (int t = 0; t < TMW * TNW; ++t) {
                const int i = t / TNW, j = t % TNW;
                d[t & 1] = mfma6(ahi[i], b[j], zero16, scale_hi, scale_b);
                d[t & 1] = mfma6(alo[i], b[j], d[t & 1], scale_lo, scale_b);
                // fragments used for the last time in this group: fetch their successors
                if (j == TNW - 1) read_a(nxa, i);
                if (i == TMW - 1) {
                    read_b(nx, j);
                    scn[j] = *reinterpret_cast<const float*>(nx + s_frag + j * 128);
                }
                __builtin_amdgcn_sched_barrier(0);
                // the multiply-adds of the tile before, behind this tile's matrix instructions
                if (t > 0) {
                    const int tp = t - 1, jp = (t - 1) % TNW;
                    if (ACC) {
                        const int ip = tp / TNW;
                        const int64_t n = (int64_t)tile_n * BN + (wn * TNW + jp) * 32 + (lane & 31);
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int64_t m = (int64_t)tile_m * BM + (wm * TMW + ip) * 32 + 8 * (r / 4) + 4 * (lane >> 5) + r % 4;
                            if (m < M && n < L.N) acc_out[(m * L.N + n) * G + g] = (int32_t)d[tp & 1][r];
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) yacc[tp][r] = fmaf(sc[jp], d[tp & 1][r], yacc[tp][r]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            {
                constexpr int tp = TMW * TNW - 1, jp = tp % TNW, ip = tp / TNW;
                if (ACC) {
                    const int64_t n = (int64_t)tile_n * BN + (wn * TNW + jp) * 32 + (lane & 31);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int64_t m = (int64_t)tile_m * BM + (wm * TMW + ip) * 32 + 8 * (r / 4) + 4 * (lane >> 5) + r % 4;
                        if (m < M && n < L.N) acc_out[(m * L.N + n) * G + g] = (int32_t)d[tp & 1][r];
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) yacc[tp][r] = fmaf(sc[jp], d[tp & 1][r], yacc[tp][r]);
                }
            }
#pragma unroll
            for (int j = 0; j < TNW; ++j) sc[j] = scn[j];
        }
    }
    if (ACC) return;

    if (KS > 1) {
        // Add the K parts in a fixed order: part p > 0 leaves its sums in LDS, part 0 adds them.
        float* red = reinterpret_cast<float*>(lds_all);
        const int slot = w * (TMW * TNW * 16 * 64) + lane;
#pragma unroll
        for (int p = 1; p < KS; ++p) {
            __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0): no direct load may still land in LDS
            __builtin_amdgcn_s_barrier();
            if (part == p) {
#pragma unroll
                for (int t = 0; t < TMW * TNW; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[slot + (t * 16 + r) * 64] = yacc[t][r];
            }
            __builtin_amdgcn_s_waitcnt(0x0070);
            __builtin_amdgcn_s_barrier();
            if (part == 0) {
#pragma unroll
                for (int t = 0; t < TMW * TNW; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) yacc[t][r] += red[slot + (t * 16 + r) * 64];
            }
        }
        if (part != 0) return;
    }

    // Output: y = yacc * sx[m] + bias[n].  Buffer accesses: rows past M fall outside the buffers (loads
    // give 0, stores are dropped), columns past N are sent out of range, a NULL bias is an empty buffer.
    // A wave's 8 rows x 32 TNW columns at a time go through a private LDS patch (rows padded by four floats)
    // and leave as 128-bit stores of whole row segments: a quarter of the store instructions of the direct
    // form, whose lanes hold single columns.  The patch lies where the stages were (one K part: after every
    // wave's loads have landed and every wave has left the loop) or in the wave's own slots of the K parts'
    // sums (which it has read by then; LDS operations of one wave complete in order).
    const __amdgpu_buffer_rsrc_t rs_sx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(sx), 0, (int)(M * 4), kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_bias =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (int)(L.N * 4) : 0, kBufFlags);
    const int y_bytes = (int)(uint32_t)(M * L.N * (L.out16 ? 2 : 4));
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, kBufFlags);
    const int N = (int)L.N;
    const int row0 = tile_m * BM + wm * TMW * 32;
    const int col0 = tile_n * BN + wn * TNW * 32;
    const int esz = L.out16 ? 2 : 4;
    constexpr int RS = TNW * 32 + 4;                  // floats per patch row
    constexpr int UPR = TNW * 8;                      // 16-byte units per row segment
    constexpr int PATCH_STRIDE = KS > 1 ? TMW * TNW * 16 * 64 : 8 * RS;   // floats between the waves' patches
    static_assert(8 * RS <= PATCH_STRIDE, "the patch fits the wave's slots");
    if (KS == 1) {
        __builtin_amdgcn_s_waitcnt(0x0070);           // vmcnt(0) lgkmcnt(0): this wave's direct loads have landed
        __builtin_amdgcn_s_barrier();                 // ... and everybody's; nobody reads a stage any more
    }
    float* patch = reinterpret_cast<float*>(lds_all) + w * PATCH_STRIDE;
    float* wr = patch + (4 * (lane >> 5)) * RS + (lane & 31);
    float bj[TNW];
#pragma unroll
    for (int j = 0; j < TNW; ++j)
        bj[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_bias, (lane & 31) * 4, (col0 + j * 32) * 4, 0));
#pragma unroll
    for (int i = 0; i < TMW; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int mrow = row0 + i * 32 + 8 * q;   // the patch's first row; this lane wrote rows + 4 (lane / 32) + rr
            const v4i s4 = __builtin_amdgcn_raw_buffer_load_b128(rs_sx, (lane >> 5) * 16, mrow * 4, 0);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int j = 0; j < TNW; ++j)
                    wr[rr * RS + j * 32] = fmaf(yacc[i * TNW + j][q * 4 + rr], __int_as_float(s4[rr]), bj[j]);
#pragma unroll
            for (int p = 0; p < TNW; ++p) {
                const int u = p * 64 + lane;          // unit of the patch: row u / UPR, columns 4 (u % UPR) ..
                const int r = u / UPR, c4 = u % UPR;
                // (read as a struct of floats: the same scalar type as the writes for alias analysis)
                const float4 f = *reinterpret_cast<const float4*>(patch + r * RS + c4 * 4);
                const int n = col0 + c4 * 4;          // N is a multiple of 16: a unit lies inside the row or past it
                const int voff = n < N ? (r * N + c4 * 4) * esz : kOutOfRange;
                const int soff = (mrow * N + col0) * esz;
                if (L.out16) {
                    const _Float16 h0 = (_Float16)f.x, h1 = (_Float16)f.y, h2 = (_Float16)f.z, h3 = (_Float16)f.w;
                    const v2i v = {(int)((uint32_t) * reinterpret_cast<const uint16_t*>(&h0) |
                                         ((uint32_t) * reinterpret_cast<const uint16_t*>(&h1) << 16)),
                                   (int)((uint32_t) * reinterpret_cast<const uint16_t*>(&h2) |
                                         ((uint32_t) * reinterpret_cast<const uint16_t*>(&h3) << 16))};
                    __builtin_amdgcn_raw_buffer_store_b64(v, rs_y, voff, soff, 0);
                } else {
                    const v4i v = {(int)__float_as_uint(f.x), (int)__float_as_uint(f.y), (int)__float_as_uint(f.z),
                                   (int)__float_as_uint(f.w)};
                    __builtin_amdgcn_raw_buffer_store_b128(v, rs_y, voff, soff, 0);
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int KS, bool ACC, int NS = 2>
int launch6(const uint8_t* packed, const Layout& L, int64_t M, const uint8_t* a6, int TMp, const float* sx,
            const float* bias, float* y, int32_t* acc, hipStream_t st)
{
    const int MT = (int)((M + BM - 1) / BM);
    const int NT = (int)((L.N + BN - 1) / BN);
    constexpr size_t smem = lds_bytes6<BM, BN, KS, NS>();
    static_assert(smem <= kLdsPerWorkgroup, "LDS of a workgroup");
    auto kern = prefill6_kernel<BM, BN, WM, WN, KS, ACC, NS>;
    static thread_local int allowed_dev = -1;
    if (int s = allow_large_lds(kern, smem, allowed_dev)) return s;
    const int64_t blocks = (int64_t)MT * ((NT + 7) / 8) * 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * WM * WN * KS), smem, st, packed + L.plane_off(), a6, L, M,
                       TMp, sx, bias, y, acc, MT, NT);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

int tmp_tiles(int64_t M) { return (int)(((M + 31) / 32 + kPlaneTilePad - 1) / kPlaneTilePad * kPlaneTilePad); }

// Tile plans (all waves own 64 rows): 0 = 128 x 128 tiles of four waves (two workgroups per CU),
// 1 = 128 x 128 with the K range in two parts (eight waves), 2 = 128 x 256 of four waves (64 x 128
// outputs per wave, two workgroups per CU), 3 = 128 x 256 with two K parts, 4 = 256 x 256 of eight waves,
// 5 = 128 x 320 of four waves (64 x 160 outputs per wave, the column-major loop, two workgroups per CU).
int choose_plan6(const Layout& L, int64_t M)
{
    if (const char* e = debug_option(kDbgPrefill6Plan))   // tests and tuning
        if (e[0] >= '0' && e[0] <= '5') return e[0] - '0';
    const int64_t cus = num_cus();
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((L.N + bn - 1) / bn); };
    auto rounds = [&](int64_t t, int64_t slots) { return (double)((t + slots - 1) / slots); };
    // Fewer 128 x 128 tiles than CUs: one tile per CU with its K range in two parts keeps every SIMD busy
    // (measured on Qwen2-7B's o and down at 1024 tokens: 1.3 and 1.5 times faster than one part).
    const int64_t t0 = tiles(128, 128);
    if (t0 <= cus) return 1;
    // Else two workgroups of four waves per CU.  A 128 x 256 tile takes 1.54 times as long as a 128 x 128
    // one (measured at K = 3584) for twice the outputs; what decides is how many rounds of workgroups
    // each form needs.  With a single round the larger tile loses (its writes of 128 KiB per workgroup
    // all come at the end, with nothing left to overlap them).
    // (The K-split forms of these sizes lost everywhere they were measured: their loops are short and the
    // exchange of the sums is a fixed cost per tile.)
    // A 128 x 320 tile (column-major loop) takes 2.21 times a 128 x 128 one for 2.5 times the outputs:
    // worth it where it saves a round (Qwen2-7B's gate|up: two rounds instead of three of 128 x 256).
    const double r2 = rounds(tiles(128, 256), 2 * cus), r5 = rounds(tiles(128, 320), 2 * cus);
    const double c0 = rounds(t0, 2 * cus) * 1.0;
    const double c2 = r2 >= 2 ? r2 * 1.54 : 1e30;
    const double c5 = r5 >= 2 ? r5 * 2.21 : 1e30;
    if (c5 < c2 && c5 < c0) return 5;
    return c2 < c0 ? 2 : 0;
}

// Stages of the LDS rings for a plan (groups in flight or ready beside the one being contracted, plus one):
// the small tiles spend little time per group and need their loads issued further ahead.
int choose_stages6(int plan, const Layout& L, int64_t M)
{
    // measured on the Qwen2-7B shapes (two -> four stages): down 129 -> 107 us, o 31.6 -> 28.0, q|k|v 44.1 -> 41.6;
    // the 128 x 256 tiles gain nothing from a third stage (a group keeps them busy for longer than a load takes).
    // Four stages of the four-wave 128 x 128 form leave room for two workgroups per CU where two stages
    // leave room for three: with more tiles than two per CU the third workgroup is worth more than the
    // deeper ring (Llama-3-8B's q|k|v, 768 tiles: 82.6 us with two stages, 92.8 with four).
    const int64_t t0 = ((M + 127) / 128) * ((L.N + 127) / 128);
    int ns = plan == 1 ? 4 : (plan == 0 && t0 <= 2 * (int64_t)num_cus()) ? 4 : 2;
    if (const char* e = debug_option(kDbgPrefill6Stages)) {   // tests and tuning
        const int v = e[0] - '0';
        if (v >= 2 && v <= 4) ns = v;
    }
    if (plan >= 4 || (plan >= 2 && ns > 3)) ns = 2;   // what fits the LDS: 4 for the 128 x 128 tiles, 3 for 128 x 256
    return ns;
}

struct Plan6Info {
    int BM, BN, KS, waves;
    size_t lds;
};

Plan6Info plan6_info(int plan, const Layout& L, int64_t M)
{
    const int ns = choose_stages6(plan, L, M);
    switch (plan) {
        case 1: return {128, 128, 2, 8, ns == 4 ? lds_bytes6<128, 128, 2, 4>() : ns == 3 ? lds_bytes6<128, 128, 2, 3>() : lds_bytes6<128, 128, 2>()};
        case 2: return {128, 256, 1, 4, ns == 3 ? lds_bytes6<128, 256, 1, 3>() : lds_bytes6<128, 256, 1>()};
        case 3: return {128, 256, 2, 8, ns == 3 ? lds_bytes6<128, 256, 2, 3>() : lds_bytes6<128, 256, 2>()};
        case 4: return {256, 256, 1, 8, lds_bytes6<256, 256, 1>()};
        case 5: return {128, 320, 1, 4, lds_bytes6<128, 320, 1>()};
        default: return {128, 128, 1, 4, ns == 4 ? lds_bytes6<128, 128, 1, 4>() : ns == 3 ? lds_bytes6<128, 128, 1, 3>() : lds_bytes6<128, 128, 1>()};
    }
}

}  // namespace

size_t prefill6_ws_bytes(int64_t M, int64_t K) { return (size_t)(K / kGroup) * tmp_tiles(M) * 2 * kPlaneBlockBytes; }

bool prefill6_possible(const Layout& L, int64_t M)
{
    const int64_t lim = ((int64_t)1 << 31) - 1;
    return L.plane && L.mode == MNNQ_W4_ZP_INT && M > 32 && (int64_t)L.plane_bytes() <= lim &&
           (int64_t)prefill6_ws_bytes(M, L.Kx) <= lim;
}

bool prefill6_wanted(const Layout& L, int64_t M)
{
    if (!prefill6_possible(L, M)) return false;
    if (debug_option(kDbgPrefill6Plan)) return true;   // a forced plan: tests and tuning
    // fewer 128 x 128 tiles than a quarter of the CUs and a long K: the int8 GEMM, which splits K four
    // ways, fills the chip better than this one's two parts
    const int64_t t0 = ((M + 127) / 128) * ((L.N + 127) / 128);
    return 4 * t0 >= num_cus() || L.Kx < 4096;
}

void describe_prefill6(const Layout& L, int64_t M, int32_t out[8])
{
    const Plan6Info p = plan6_info(choose_plan6(L, M), L, M);
    const int64_t MT = (M + p.BM - 1) / p.BM, NT = (L.N + p.BN - 1) / p.BN;
    out[0] = p.BM;
    out[1] = p.BN;
    out[2] = p.KS;
    out[3] = 1;
    out[4] = p.waves;
    out[5] = (int32_t)p.lds;
    out[6] = (int32_t)(MT * ((NT + 7) / 8) * 8);
    out[7] = 6;   // operands in fp6
}

int launch_plane_build(uint8_t* packed, const Layout& L, hipStream_t st)
{
    const int64_t blocks = (L.Gx * L.T32p + 3) / 4;
    hipLaunchKernelGGL(plane_build_kernel, dim3((unsigned)blocks), dim3(256), 0, st, packed, L);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

int launch_act_planes(const int8_t* xq, int64_t M, int64_t K, void* planes, hipStream_t st)
{
    const int TMp = tmp_tiles(M);
    const int Gx = (int)(K / kGroup);
    const int64_t waves = (int64_t)Gx * TMp;
    hipLaunchKernelGGL(planes_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, xq, M, K, Gx, TMp,
                       static_cast<uint8_t*>(planes));
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

int launch_prefill6(const uint8_t* packed, const Layout& L, int64_t M, const void* planes, const float* sx,
                    const float* bias, float* y, int32_t* acc_debug, hipStream_t st)
{
    const int TMp = tmp_tiles(M);
    const uint8_t* a6 = static_cast<const uint8_t*>(planes);
    if (acc_debug) return launch6<128, 128, 2, 2, 1, true, 4>(packed, L, M, a6, TMp, sx, bias, y, acc_debug, st);   // plan 0 as it runs
    const int plan = choose_plan6(L, M), ns = choose_stages6(plan, L, M);
#define MNNQ_ARGS6 packed, L, M, a6, TMp, sx, bias, y, nullptr, st
    if (ns == 4) {
        if (plan == 1) return launch6<128, 128, 2, 2, 2, false, 4>(MNNQ_ARGS6);
        if (plan == 0) return launch6<128, 128, 2, 2, 1, false, 4>(MNNQ_ARGS6);
    }
    if (ns == 3) {
        if (plan == 0) return launch6<128, 128, 2, 2, 1, false, 3>(MNNQ_ARGS6);
        if (plan == 1) return launch6<128, 128, 2, 2, 2, false, 3>(MNNQ_ARGS6);
        if (plan == 2) return launch6<128, 256, 2, 2, 1, false, 3>(MNNQ_ARGS6);
        if (plan == 3) return launch6<128, 256, 2, 2, 2, false, 3>(MNNQ_ARGS6);
    }
#undef MNNQ_ARGS6
    switch (plan) {
        case 1: return launch6<128, 128, 2, 2, 2, false>(packed, L, M, a6, TMp, sx, bias, y, nullptr, st);
        case 2: return launch6<128, 256, 2, 2, 1, false>(packed, L, M, a6, TMp, sx, bias, y, nullptr, st);
        case 3: return launch6<128, 256, 2, 2, 2, false>(packed, L, M, a6, TMp, sx, bias, y, nullptr, st);
        case 4: return launch6<256, 256, 4, 2, 1, false>(packed, L, M, a6, TMp, sx, bias, y, nullptr, st);
        case 5: return launch6<128, 320, 2, 2, 1, false>(packed, L, M, a6, TMp, sx, bias, y, nullptr, st);
        default: return launch6<128, 128, 2, 2, 1, false>(packed, L, M, a6, TMp, sx, bias, y, nullptr, st);
    }
}

}  // namespace mnnq
