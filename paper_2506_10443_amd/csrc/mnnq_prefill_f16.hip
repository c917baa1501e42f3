// Prefill GEMM with fp16 activations on the gfx950 fp16 matrix cores (Section 4.2:
// on GPUs the int4 weights are combined with fp16 activations, W4A16).
//
//   y[m,n] = rs[m] * sum_g scale[n,g] * sum_{k in g} float(x16[m,k]) * (q[n,k] - zero[n,g]) (+ bias[n])
//
// rs is an optional per-row factor (1 when absent).  The integer q - z (|.| <= 15)
// is exact in fp16, so the weights enter the contraction unrounded and the group
// scale is applied once per group in fp32: two v_mfma_f32_16x16x32_f16 with a
// zero C operand contract one quantization group (K = 64) of a 16 x 16 tile, and
// four fused multiply-adds per lane fold the fp32 group sum into the running sum.
//
// When the activations are integer codes |x| <= 127 stored as fp16, every product
// (<= 1905) and every partial sum of a group (<= 121920) is an integer below 2^24
// and therefore exact in fp32 whatever the summation order: the group sums equal
// the int32 accumulators of the int8 kernel, and no int -> float conversion is
// needed in the epilogue.
//
// Float-minimum weights (Eq. 1 as printed; also the two 4-bit planes of 8-bit codes, whose
// reduction axis runs over the activation row twice):
//   y[m,n] = rs[m] * sum_g (step[n,g] * sum_{k in g} x[m,k] q[n,k] + min[n,g] * sum_{k in g} x[m,k]);
// the B operand is the code itself, and one more MFMA pair per 16 rows and group with an
// all-ones B operand yields the group sums of x in the D layout, i.e. for exactly the four
// rows a lane holds.
//
// The structure is that of the int8 prefill kernel: operands reach LDS with
// direct buffer loads, an A stage is one group (BM rows x 64 halves = 128 B per
// row, 16-byte units XOR-swizzled by the row), a B chunk (two groups) is copied
// verbatim and held in registers while it is used, and the epilogue of one tile
// is issued behind the MFMAs of the next.
//
// Lane mapping of the 16x16x32 fp16 MFMA (A: 16 x 32, B: 32 x 16, D: 16 x 16):
//   A operand: lane l holds row l % 16, 8 consecutive k of block l / 16;
//   B operand: lane l holds column l % 16, the same 8 k;
//   D:         lane l holds column l % 16, rows 4 (l / 16) + r, r = 0..3.
// The packed layout gives lane l the 16 codes k = 16 (l / 16) + j of a group.  The
// first MFMA of a group takes j = 0..7 and the second j = 8..15 on both operands;
// which k meets which MFMA slot does not matter as long as A and B agree.
#include "mnnq_common.h"

#include <stdlib.h>

namespace mnnq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

#define MNNQ_LDS(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int kBufFlags = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)

union H8Bits {
    uint32_t u[4];
    h8 h;
};

union H2Bits {
    uint32_t u;
    h2 h;
};

// Two codes (bytes b0, b1 of v, each 0..15) -> the halves (c0 - z, c1 - z).
// A byte c under the high byte 0x64 is the half 1024 + c; subtracting the half
// 1024 + z (zb, twice) leaves c - z exactly.
template <uint32_t SEL>
__device__ __forceinline__ uint32_t code_pair(uint32_t v, h2 zb)
{
    H2Bits p;
    p.u = __builtin_amdgcn_perm(0x64646464u, v, SEL);
    p.h = p.h - zb;
    return p.u;
}

// The eight codes of dword w in natural order (low nibbles of bytes 0..3 are codes
// 0..3, high nibbles codes 4..7) as eight halves q - z.
__device__ __forceinline__ h8 unpack8(uint32_t w, h2 zb)
{
    const uint32_t lo = w & 0x0f0f0f0fu;
    const uint32_t hi = (w >> 4) & 0x0f0f0f0fu;
    H8Bits r;
    r.u[0] = code_pair<0x04010400u>(lo, zb);
    r.u[1] = code_pair<0x04030402u>(lo, zb);
    r.u[2] = code_pair<0x04010400u>(hi, zb);
    r.u[3] = code_pair<0x04030402u>(hi, zb);
    return r.h;
}

template <int BM, int BN, bool MINF>
struct Lds {
    static constexpr int NT16 = BN / 16;                 // row tiles of B per workgroup
    static constexpr int A_BYTES = BM * 128;             // [BM][64] halves, swizzled
    static constexpr int A_OFF = 0;                      // two A buffers (even / odd group)
    static constexpr int B_OFF = 2 * A_BYTES;            // [NT16][1024] packed codes
    static constexpr int S_OFF = B_OFF + NT16 * 1024;    // [NT16][16][2] fp32 scales
    static constexpr int Z_OFF = S_OFF + NT16 * 128;     // [NT16][16][2] u8 zeros, or fp32 group minima (MINF)
    static constexpr int BYTES = Z_OFF + NT16 * (MINF ? 128 : 32);
};

// KS: K parts inside the workgroup (as in the int8 kernel): with KS = 2 the workgroup has eight waves,
// each half takes one half of the chunks with staging buffers of its own, and the halves' sums are
// added through LDS in a fixed order - for shapes with at most one tile per CU.
template <int BM, int BN, bool MINF, int KS = 1>
__global__ __launch_bounds__(256 * KS, KS > 1 ? 1 : 2) void prefill_f16_kernel(const uint8_t* __restrict__ packed, Layout L, int64_t M,
                                                             const uint16_t* __restrict__ x16,
                                                             const float* __restrict__ rs,
                                                             const float* __restrict__ bias, float* __restrict__ y,
                                                             int MT, int NT)
{
    using St = Lds<BM, BN, MINF>;
    constexpr int WM = BM / 2, WN = BN / 2;      // 2 x 2 waves
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int NT16 = St::NT16;
    constexpr int A_INSTR = BM / 8 / 4;          // 1 KiB direct loads of A per wave and stage
    static_assert(NT16 == 8, "B side is written for 8 row tiles per workgroup");
    static_assert(KS == 1 || 4 * TM * TN * 4 * 64 * 4 <= KS * St::BYTES, "the K parts' sums must fit in LDS");

    extern __shared__ __align__(16) uint8_t lds_all[];   // KS * St::BYTES

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave = wave_id & 3;                // position in the 2 x 2 wave grid of its K part
    const int kh = wave_id >> 2;                 // K part of this wave (0 .. KS-1)
    uint8_t* const lds = lds_all + kh * St::BYTES;
    const int wm = wave >> 1, wn = wave & 1;
    const int col = lane & 15;
    const int kb = lane >> 4;
    const int C = (int)L.C;
    const int K2 = (int)L.Kx * 2;                // bytes per activation row
    const int Gx = (int)L.Kx / 64;               // group g of the packed axis meets group g % Gx of the row

    // Each XCD gets whole columns of output tiles, so that a weight block is fetched
    // into one L2 only.
    const int xcd = blockIdx.x % 8;
    const int seq = blockIdx.x / 8;
    const int tile_m = seq % MT;
    const int tile_n = (seq / MT) * 8 + xcd;
    if (tile_n >= NT) return;
    const int64_t m0 = (int64_t)tile_m * BM;
    const int rt0 = tile_n * NT16;

    // Out-of-range reads (rows past M, row tiles past N) return zero.
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x16), 0, (int)(M * L.Kx * 2), kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(packed), 0, (int)L.total(), kBufFlags);

    // A zero the compiler cannot see through: casting a compile-time-constant LDS
    // address to the LDS address space trips a code generation error in this toolchain.
    int opaque_zero = 0;
    asm volatile("" : "+s"(opaque_zero));

    const int a_voff = (lane >> 3) * K2 + (((lane & 7) ^ (lane >> 3)) << 4);
    const int b_voff = lane * 16;
    const int s_voff = (lane >> 5) * C * 128 + (lane & 31) * 4;
    const int z_voff = (lane >> 3) * C * 32 + (lane & 7) * 4;
    const int scales_off = (int)L.scales_off();
    const int zeros_off = (int)L.zeros_off();

    const int a_row_off = St::A_OFF + (wm * WM + col) * 128;   // + i * 2048 per m-tile
    const int a_sw = col & 7;
    const int a_u0 = ((2 * kb) ^ a_sw) << 4;                    // unit of halves 16 kb .. 16 kb + 7
    const int a_u1 = ((2 * kb + 1) ^ a_sw) << 4;                // unit of halves 16 kb + 8 .. 16 kb + 15
    const int b_frag_off = St::B_OFF + wn * TN * 1024 + lane * 16;
    const int s_frag_off = St::S_OFF + wn * TN * 128 + col * 8;
    const int z_frag_off = St::Z_OFF + (MINF ? wn * TN * 128 + col * 8 : wn * TN * 32 + col * 2);

    // A stage: group g of this workgroup's BM rows.
    auto issue_a = [&](int g, int buf) {
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) {
            const int q = wave * A_INSTR + i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, MNNQ_LDS(lds + St::A_OFF + buf * St::A_BYTES + q * 1024),
                                                     16, a_voff, ((int)m0 + q * 8) * K2 + (g % Gx) * 128, 0, 0);
        }
    };
    auto issue_b = [&](int c) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = wave * 2 + i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::B_OFF + j * 1024), 16, b_voff,
                                                     ((rt0 + j) * C + c) * 1024, 0, 0);
        }
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::S_OFF + wave * 256), 4, s_voff,
                                                 scales_off + ((rt0 + wave * 2) * C + c) * 128, 0, 0);
        if (MINF)   // group minima: fp32, laid out like the scales
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::Z_OFF + wave * 256), 4, s_voff,
                                                     zeros_off + ((rt0 + wave * 2) * C + c) * 128, 0, 0);
        else if (wave == 0)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::Z_OFF + opaque_zero), 4, z_voff,
                                                     zeros_off + (rt0 * C + c) * 32, 0, 0);
    };

    float yacc[TM][TN][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) yacc[i][j][r] = 0.0f;

    v4i bw[TN];
    v2i bsv[TN];
    uint32_t bz[TN];      // zero points of both groups (integer zero point form)
    v2i bmn[TN];          // group minima of both groups, fp32 bits (float minimum form)
    auto read_b = [&]() {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            bw[j] = *reinterpret_cast<const v4i*>(lds + b_frag_off + j * 1024);
            bsv[j] = *reinterpret_cast<const v2i*>(lds + s_frag_off + j * 128);
            if (MINF) bmn[j] = *reinterpret_cast<const v2i*>(lds + z_frag_off + j * 128);
            else bz[j] = *reinterpret_cast<const uint16_t*>(lds + z_frag_off + j * 32);
        }
    };

    // One group of the wave's TM x TN tiles: MFMA pair (t+1) < epilogue (t) < MFMA pair (t+2).
    // The empty asm statements emit nothing; they tie values together so that this
    // order survives the compiler's schedulers.
    auto compute = [&](int h, int buf) {
        h8 b0[TN], b1[TN];
        float sc[TN];
        float mnv[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            H2Bits zb;   // the half 1024 + zero point, twice (float minimum form: 1024, the codes stay as they are)
            if (MINF) zb.u = 0x64006400u;
            else zb.u = __builtin_amdgcn_perm(0x64646464u, bz[j], h ? 0x04010401u : 0x04000400u);
            b0[j] = unpack8((uint32_t)(h ? bw[j].z : bw[j].x), zb.h);
            b1[j] = unpack8((uint32_t)(h ? bw[j].w : bw[j].y), zb.h);
            sc[j] = __int_as_float(h ? bsv[j].y : bsv[j].x);
            mnv[j] = MINF ? __int_as_float(h ? bmn[j].y : bmn[j].x) : 0.0f;
        }
        const uint8_t* ap = lds + buf * St::A_BYTES + a_row_off;
        const v4f zero = {0.0f, 0.0f, 0.0f, 0.0f};
        h8 a0 = *reinterpret_cast<const h8*>(ap + a_u0);
        h8 a1 = *reinterpret_cast<const h8*>(ap + a_u1);
        h8 a0_nxt = a0, a1_nxt = a1;
        if (TM > 1) {
            a0_nxt = *reinterpret_cast<const h8*>(ap + 2048 + a_u0);
            a1_nxt = *reinterpret_cast<const h8*>(ap + 2048 + a_u1);
        }
        v4f d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, b0[0], zero, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, b1[0], d, 0, 0, 0);
        // float minimum form: group sums of x for the lane's four rows of this and the next m-tile
        H8Bits ones;
        ones.u[0] = ones.u[1] = ones.u[2] = ones.u[3] = 0x3c003c00u;
        v4f xs_cur = zero, xs_nxt = zero;
        if (MINF) {
            xs_cur = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, ones.h, zero, 0, 0, 0);
            xs_cur = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, ones.h, xs_cur, 0, 0, 0);
        }
#pragma unroll
        for (int tt = 0; tt < TM * TN; ++tt) {
            const int i = tt / TN, j = tt % TN;
            v4f d_nxt = d;
            if (tt + 1 < TM * TN) {
                const int i1 = (tt + 1) / TN, j1 = (tt + 1) % TN;
                if (j1 == 0) {
                    a0 = a0_nxt;
                    a1 = a1_nxt;
                    if (i1 + 1 < TM) {
                        a0_nxt = *reinterpret_cast<const h8*>(ap + (i1 + 1) * 2048 + a_u0);
                        a1_nxt = *reinterpret_cast<const h8*>(ap + (i1 + 1) * 2048 + a_u1);
                    }
                }
                d_nxt = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, b0[j1], zero, 0, 0, 0);
                d_nxt = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, b1[j1], d_nxt, 0, 0, 0);
                if (MINF && j1 == 0) {
                    xs_nxt = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, ones.h, zero, 0, 0, 0);
                    xs_nxt = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, ones.h, xs_nxt, 0, 0, 0);
                }
                asm volatile("" : "+v"(d), "+v"(d_nxt));
            }
            if (MINF && j == 0 && i > 0) xs_cur = xs_nxt;   // issued with the first MFMA pair of this row of tiles
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                yacc[i][j][rr] = fmaf(sc[j], d[rr], yacc[i][j][rr]);
                if (MINF) yacc[i][j][rr] = fmaf(mnv[j], xs_cur[rr], yacc[i][j][rr]);
            }
            if (tt + 2 < TM * TN) {
                const int j2 = (tt + 2) % TN;
                asm volatile(""
                             : "+v"(b0[j2]), "+v"(yacc[i][j][0]), "+v"(yacc[i][j][1]), "+v"(yacc[i][j][2]),
                               "+v"(yacc[i][j][3]));
            } else {
                asm volatile("" : "+v"(yacc[i][j][0]), "+v"(yacc[i][j][1]), "+v"(yacc[i][j][2]), "+v"(yacc[i][j][3]));
            }
            d = d_nxt;
        }
    };

    // This K part's chunks; all waves run the longest share's barriers, the shorter share idles
    // through the last round.
    const int cb = C * kh / KS, ce = C * (kh + 1) / KS;
    const int n_iter = (C + KS - 1) / KS;
    if (cb < ce) {
        issue_a(2 * cb, 0);
        issue_b(cb);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (cb < ce) read_b();

    for (int it = 0; it < n_iter; ++it) {
        const int c = cb + it;
        const bool live = c < ce;
        const bool more = c + 1 < ce;
        // Every wave has finished group 2c - 1 and holds chunk c's B fragments in
        // registers: the odd A buffer and the B tile may be overwritten.
        __syncthreads();
        // The padding group of an odd G is skipped: its activations would be the next
        // row's, and 0 * x is not 0 for every x.
        const bool odd_group = live && 2 * c + 1 < (int)L.G;
        if (odd_group) issue_a(2 * c + 1, 1);
        if (more) issue_b(c + 1);
        if (live) compute(0, 0);
        // Group 2c + 1 (and chunk c + 1's B tile) has landed for every wave, and every
        // wave has finished reading the even A buffer.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (more) issue_a(2 * c + 2, 0);
        if (odd_group) compute(1, 1);
        if (more) {
            read_b();
            __builtin_amdgcn_s_waitcnt(0x0F70);
        }
    }

    if (KS > 1) {
        // Add the K parts in a fixed order: part kh > 0 leaves its sums in LDS (one conflict-free
        // float per lane and accumulator), part 0 adds them.
        float* red = reinterpret_cast<float*>(lds_all);
        const int slot = wave * (TM * TN * 4 * 64) + lane;
#pragma unroll
        for (int p = 1; p < KS; ++p) {
            __syncthreads();                 // staging buffers (or the previous part's sums) are dead
            if (kh == p) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) red[slot + ((i * TN + j) * 4 + r) * 64] = yacc[i][j][r];
            }
            __syncthreads();
            if (kh == 0) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) yacc[i][j][r] += red[slot + ((i * TN + j) * 4 + r) * 64];
            }
        }
        __syncthreads();                     // part 0 has read the sums: LDS is free for the output stage
        if (kh != 0) return;
    }

    // Output: y = yacc * rs[m] + bias[n].  Buffer accesses keep this free of branches
    // and 64-bit address arithmetic: rows past M fall outside the buffers (loads give 0,
    // stores are dropped), a NULL bias is an empty buffer.
    const __amdgpu_buffer_rsrc_t rs_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(rs), 0, rs ? (int)(M * 4) : 0, kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_bias =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (int)(L.N * 4) : 0, kBufFlags);
    const int y_bytes = (int)(uint32_t)(M * L.N * 4);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, kBufFlags);
    const int Nb = (int)L.N * 4;                       // bytes per output row
    const int row0 = (int)m0 + wm * WM;                // first row of this wave
    const int nt0 = rt0 + wn * TN;                     // first row tile (16 outputs) of this wave
    float bj[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
        bj[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_bias, col * 4, (nt0 + j) * 64, 0));
    // The 16 x (16 TN) block of one m-tile goes through a private LDS patch of the wave (rows
    // padded by 4 floats: conflict-free both ways) and leaves as 128-bit stores of whole row
    // segments.  LDS operations of one wave complete in order, so the patch needs no barrier of
    // its own; the barrier in front makes sure no wave still reads operands where it lies.
    static_assert(TN == 4, "a lane stores one 16-byte unit of a 64-column row segment");
    constexpr int RS = 16 * TN + 4;                    // floats per patch row
    if (KS == 1) __syncthreads();
    float* patch = reinterpret_cast<float*>(lds_all) + wave * (16 * RS);
    float* wr = patch + (kb * 4) * RS + col;
    const float* rd = patch + kb * RS + col * 4;       // + 4 p rows
    // a lane's 16-byte unit lies in row tile nt0 + col / 4; units past N are sent out of range
    const bool unit_ok = nt0 + (col >> 2) < (int)L.T;
    const int y_voff = unit_ok ? kb * Nb + col * 16 : y_bytes;
    // binary16 output: the same unit is four halves, rows are half as long
    const __amdgpu_buffer_rsrc_t rs_y16 = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes / 2, kBufFlags);
    const int y_voff16 = unit_ok ? kb * (Nb / 2) + col * 8 : y_bytes / 2;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        float rsr[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            rsr[rr] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_rs, kb * 16, (row0 + i * 16 + rr) * 4, 0));
            if (!rs) rsr[rr] = 1.0f;
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
#pragma unroll
            for (int j = 0; j < TN; ++j) wr[rr * RS + j * 16] = fmaf(yacc[i][j][rr], rsr[rr], bj[j]);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            // (read as a struct of floats: the same scalar type as the writes for alias analysis)
            const float4 f = *reinterpret_cast<const float4*>(rd + p * 4 * RS);
            if (L.out16) {
                H2Bits lo, hi;
                lo.h = h2{(_Float16)f.x, (_Float16)f.y};
                hi.h = h2{(_Float16)f.z, (_Float16)f.w};
                const v2i v = {(int)lo.u, (int)hi.u};
                __builtin_amdgcn_raw_buffer_store_b64(v, rs_y16, y_voff16, (row0 + i * 16 + p * 4) * (Nb / 2) + nt0 * 32, 0);
                continue;
            }
            const v4i v = {(int)__float_as_uint(f.x), (int)__float_as_uint(f.y), (int)__float_as_uint(f.z),
                           (int)__float_as_uint(f.w)};
            __builtin_amdgcn_raw_buffer_store_b128(v, rs_y, y_voff, (row0 + i * 16 + p * 4) * Nb + nt0 * 64, 0);
        }
    }
}

template <int BM, int BN, bool MINF, int KS = 1>
int launch_tiles_m(const uint8_t* packed, const Layout& L, int64_t M, const uint16_t* x16, const float* rs,
                   const float* bias, float* y, hipStream_t st)
{
    const int MT = (int)((M + BM - 1) / BM);
    const int NT = (int)((L.N + BN - 1) / BN);
    constexpr size_t smem = (size_t)KS * Lds<BM, BN, MINF>::BYTES;
    auto kern = prefill_f16_kernel<BM, BN, MINF, KS>;
    if (smem > 64 * 1024) {
        // More than 64 KiB of dynamic LDS has to be allowed once per kernel and device.
        static thread_local int allowed_dev = -1;
        int dev = 0;
        MNNQ_HIP_TRY(hipGetDevice(&dev));
        if (allowed_dev != dev) {
            MNNQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            allowed_dev = dev;
        }
    }
    const int64_t blocks = (int64_t)MT * ((NT + 7) / 8) * 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256 * KS), smem, st, packed, L, M, x16, rs, bias, y, MT, NT);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

template <int BM, int BN, int KS = 1>
int launch_tiles(const uint8_t* packed, const Layout& L, int64_t M, const uint16_t* x16, const float* rs,
                 const float* bias, float* y, hipStream_t st)
{
    if (L.minf) return launch_tiles_m<BM, BN, true, KS>(packed, L, M, x16, rs, bias, y, st);
    return launch_tiles_m<BM, BN, false, KS>(packed, L, M, x16, rs, bias, y, st);
}

}  // namespace

int launch_prefill_f16(const uint8_t* packed, const Layout& L, int64_t M, const uint16_t* x16, const float* rs,
                       const float* bias, float* y, hipStream_t st)
{
    const int cus = num_cus();
    const int64_t tiles_big = ((M + 255) / 256) * ((L.N + 127) / 128);
    const int64_t tiles_small = ((M + 127) / 128) * ((L.N + 127) / 128);
    bool big = M > 128 && tiles_big >= 2 * (int64_t)cus;
    // at most one 128-row tile per CU: split the chunks over the two halves of an eight-wave workgroup
    int ks = (!big && tiles_small <= (int64_t)cus && L.C >= 4) ? 2 : 1;
    if (const char* e = debug_option(kDbgPrefillTile)) {   // tuning and tests: "b"/"s" tile, third letter "k" = K parts
        if (e[0] == 'b') big = true;
        if (e[0] == 's') big = false;
        if (e[0]) ks = (e[1] && e[2] == 'k') ? 2 : 1;
    }
    if (big && ks == 2) return launch_tiles<256, 128, 2>(packed, L, M, x16, rs, bias, y, st);
    if (big) return launch_tiles<256, 128>(packed, L, M, x16, rs, bias, y, st);
    if (ks == 2) return launch_tiles<128, 128, 2>(packed, L, M, x16, rs, bias, y, st);
    return launch_tiles<128, 128>(packed, L, M, x16, rs, bias, y, st);
}

}  // namespace mnnq
