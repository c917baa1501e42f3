// Prefill (M tokens): W4A8 GEMM on the gfx950 int8 matrix cores, compute-bound
// (Section 2.1).  One v_mfma_i32_16x16x64_i8 contracts exactly one quantization
// group (K = 64) of a 16 x 16 output tile, so its result (above the constant in
// its C operand) is the int32 group accumulator I[m, n, g]; the fused epilogue
// turns it into fp32 and adds scale[n, g] * I to the running sum:
//
//   y[m,n] = sx[m] * sum_g scale[n,g] * I[m,n,g] (+ bias[n])
//
// The epilogue needs two VALU operations (int32 -> fp32, fused multiply-add) per
// output and group - 8 per MFMA and lane, which take longer to issue than the
// MFMA occupies the matrix pipe - so the kernel is bound by the vector ALU, not
// by the MFMA rate.  Everything else is arranged to add as little VALU work as
// possible and to let it overlap the MFMAs:
//   * all operands reach LDS with direct buffer loads (buffer_load ... lds): no
//     staging registers, no address arithmetic in the vector pipe (the buffer
//     resource and the per-chunk offsets are scalar), out-of-range rows read 0;
//   * a wave owns TM x TN tiles of 16 x 16 (TM = 8 where M allows), so the
//     nibble -> int8 unpack of a B fragment is shared by TM MFMAs;
//   * the chunk layout of the weights already is the MFMA B-operand order, so a
//     weight chunk is copied to LDS verbatim and read back with one conflict
//     free 128-bit read per lane;
//   * A rows are 128 B in LDS with their 16-byte units XOR-swizzled by the row,
//     which makes the 128-bit fragment reads conflict free without padding;
//   * the epilogue of one tile is issued behind the MFMA of the next;
//   * a tile is worked on by four or eight waves per K part (template parameter
//     WNW); the eight-wave forms need at most 128 registers, which puts four waves
//     on every SIMD.
//
// Lane mapping of the 16x16x64 int8 MFMA (A: 16 x 64, B: 64 x 16, D: 16 x 16):
//   A operand: lane l holds row l % 16, 16 consecutive k of block l / 16;
//   B operand: lane l holds column l % 16, the same 16 k of block l / 16;
//   D:         lane l holds column l % 16, rows 4 (l / 16) + r, r = 0..3.
#include "mnnq_common.h"

#include <stdlib.h>

namespace mnnq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t h2_bits(h2v h)
{
    union {
        h2v h;
        uint32_t u;
    } b;
    b.h = h;
    return b.u;
}

#define MNNQ_LDS(p) ((__attribute__((address_space(3))) void*)(p))

// A value that is the same in every lane, said so to the compiler: as the scalar offset of a
// buffer load it then needs no loop over the distinct values of a vector register.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

constexpr int kBufFlags = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)

// q - z per byte for four codes (0..15) in the bytes of v.  c4 holds 0x80 - z in
// every byte: adding it keeps each byte in [0x71, 0x8f], so no carry or borrow
// crosses a byte, and flipping bit 7 afterwards leaves q - z as a signed byte.
__device__ __forceinline__ int sub_zero(uint32_t v, uint32_t c4)
{
    return (int)((v + c4) ^ 0x80808080u);
}

__device__ __forceinline__ v4i unpack_b(uint32_t w0, uint32_t w1, uint32_t c4)
{
    v4i b;
    b.x = sub_zero(w0 & 0x0f0f0f0fu, c4);
    b.y = sub_zero((w0 >> 4) & 0x0f0f0f0fu, c4);
    b.z = sub_zero(w1 & 0x0f0f0f0fu, c4);
    b.w = sub_zero((w1 >> 4) & 0x0f0f0f0fu, c4);
    return b;
}

// LDS map of a workgroup: the A tile is double buffered, the B tile (codes, scales,
// zeros of one chunk) is single buffered - it is copied into registers before
// the next chunk is loaded over it.
// W8: the packed matrix holds 8-bit codes as two nibble planes; the low plane's chunk gets a B
// tile of its own behind the high plane's.
template <int BM, int BN, bool MINF, int W8 = 0>
struct Lds {
    static constexpr int NT16 = BN / 16;                 // row tiles of B per workgroup
    static constexpr int A_BYTES = BM * 128;             // [BM][128] int8, swizzled
    static constexpr int A_OFF = 0;                      // two A buffers
    static constexpr int B_OFF = 2 * A_BYTES;            // [NT16][1024] packed codes
    static constexpr int B2_OFF = B_OFF + NT16 * 1024;   // W8: [NT16][1024] codes of the low nibble plane
    static constexpr int S_OFF = B2_OFF + (W8 ? NT16 * 1024 : 0);   // [NT16][16][2] fp32 scales
    static constexpr int Z_OFF = S_OFF + NT16 * 128;     // [NT16][16][2] u8 zeros, or fp32 group minima (MINF)
    // (the zero points arrive with one load of 8 x 32 B whatever NT16 is: lanes past the tile bring zeros)
    static constexpr int BYTES = Z_OFF + (MINF ? NT16 * 128 : 8 * 32);
};

// Work distribution: one workgroup per output tile and K split.  Shapes with few
// output tiles and a long K (e.g. N = 3584, K = 18944 at M = 1024) cannot fill 256
// CUs with whole tiles, so their K range is cut in two; both halves add their part
// to a zeroed y with fp32 atomics.  Two addends commute, so the result does not
// depend on which half arrives first.
//
// W8 (8-bit weights, float minimum form): a code q8 = 16 hi + lo lies in two nibble planes, chunk c
// of the high plane and chunk c + Cx of the low one.  Both are fetched, merged in registers into
// the signed byte q8 - 128 and contracted with one MFMA per group; with D = sum xq (q8 - 128) and
// xs = sum xq the group's term  s (D + 128 xs) + min xs  is  s D + (min + 128 s) xs, so only the
// minimum that enters the epilogue changes.  The stored scale of the high plane is 16 s.
//
// WNW: waves along N per K part (2 x WNW waves work on a tile).  With WNW = 4 a wave owns 128 x 32
// outputs of a 256 x 128 tile: half the accumulators, so that four waves fit on a SIMD (two
// workgroups of eight waves per CU) while a B unpack is still shared by eight MFMAs.
template <int BM, int BN, int KS, bool ACC, bool MINF, int W8 = 0, int WNW = 2>
__global__ __launch_bounds__(128 * WNW * KS, (ACC || KS > 1) ? 1 : 2) void prefill_kernel(const uint8_t* __restrict__ packed, Layout L, int64_t M,
                                                         const int8_t* __restrict__ xq,
                                                         const float* __restrict__ sx,
                                                         const float* __restrict__ bias, float* __restrict__ y,
                                                         int32_t* __restrict__ acc_out, int MT, int NT, int S)
{
    using St = Lds<BM, BN, MINF, W8>;
    static_assert(!W8 || (MINF && !ACC), "8-bit weights come in the float minimum form; the accumulator dump stays per plane");
    constexpr int WPK = 2 * WNW;                 // waves per K part: 2 x WNW
    constexpr int WM = BM / 2, WN = BN / WNW;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int NT16 = St::NT16;
    constexpr int A_INSTR = BM / 8 / WPK;        // 1 KiB direct loads of A per wave and stage
    constexpr int B_INSTR = NT16 / WPK;          // row tiles of B codes per wave and stage
    static_assert(NT16 == 8 || NT16 == 4, "B side: 8 row tiles per workgroup, or 4 (64-column tiles for few tokens)");
    static_assert(NT16 % WPK == 0 && (NT16 == 8 || (!ACC && !W8)), "64-column tiles: plain GEMM, four waves per K part");
    static_assert(WNW == 2 || WNW == 4, "four or eight waves per K part");
    static_assert(KS == 1 || WPK * TM * TN * 4 * 64 * 4 <= KS * St::BYTES, "the K parts' sums must fit in LDS");
    static_assert(KS == 1 || !ACC, "the accumulator dump runs unsplit");

    extern __shared__ __align__(16) uint8_t lds_all[];   // KS * St::BYTES

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave = wave_id % WPK;              // position in the 2 x WNW wave grid of its K part
    const int kh = wave_id / WPK;                // K part of this wave (0 .. KS-1)
    uint8_t* const lds = lds_all + kh * St::BYTES;
    const int wm = wave / WNW, wn = wave % WNW;
    const int col = lane & 15;
    const int kb = lane >> 4;
    const int C = (int)L.C;     // chunks per row tile in the packed matrix
    const int K = (int)L.Kx;    // activation row length
    const int Cx = (int)L.Cx;   // chunk c of the packed axis meets chunk c % Cx of the activation row
    const int CL = W8 ? Cx : C; // chunks this kernel walks over (merged planes: those of the activation row)

    // Workgroups are dealt to the 8 XCDs round-robin by their linear id.  Give each
    // XCD whole columns of output tiles (one weight row block, all token blocks and
    // K splits), so that a weight block is fetched into one L2 only.
    const int xcd = blockIdx.x % 8;
    const int seq = blockIdx.x / 8;
    const int split = seq % S;
    const int tile_m = (seq / S) % MT;
    const int tile_n = (seq / (S * MT)) * 8 + xcd;
    if (tile_n >= NT) return;
    const int wcb = CL * split / S, wce = CL * (split + 1) / S;   // this workgroup's chunks
    // ... of which each K part of the workgroup takes a contiguous share
    const int cb = wcb + (wce - wcb) * kh / KS, ce = wcb + (wce - wcb) * (kh + 1) / KS;
    const int n_iter = (wce - wcb + KS - 1) / KS;                // the longest share: all waves run the same barriers
    const int64_t m0 = (int64_t)tile_m * BM;
    const int rt0 = tile_n * NT16;               // first row tile of this output tile

    // Buffer resources: out-of-range reads (rows past M, row tiles past N) return zero.
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(xq), 0, (int)(M * L.Kx), kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(packed), 0, (int)L.total(), kBufFlags);

    // A zero the compiler cannot see through: casting a compile-time-constant LDS
    // address to the LDS address space trips a code generation error in this toolchain.
    int opaque_zero = 0;
    asm volatile("" : "+s"(opaque_zero));

    // Per-lane offsets of the direct loads (constant over the whole kernel).
    const int a_voff = (lane >> 3) * K + (((lane & 7) ^ (lane >> 3)) << 4);
    const int b_voff = lane * 16;
    const int s_voff = (lane >> 5) * C * 128 + (lane & 31) * 4;
    // (lanes past the tile's row tiles are sent out of the buffer's range and bring zeros)
    const int z_voff = (lane >> 3) < NT16 ? (lane >> 3) * C * 32 + (lane & 7) * 4 : 0x7ffffff0;
    const int scales_off = (int)L.scales_off();
    const int zeros_off = (int)L.zeros_off();

    // Fragment read offsets.
    const int a_row_off = St::A_OFF + (wm * WM + col) * 128;   // + i * 2048 per m-tile
    const int a_sw = col & 7;                                   // swizzle key: row & 7 == col & 7
    const int b_frag_off = St::B_OFF + wn * TN * 1024 + lane * 16;
    const int s_frag_off = St::S_OFF + wn * TN * 128 + col * 8;
    const int z_frag_off = St::Z_OFF + (MINF ? wn * TN * 128 + col * 8 : wn * TN * 32 + col * 2);

    {
        auto issue_stage = [&](int c, int buf) {
            // A: this wave's A_INSTR blocks of 8 rows x 128 B.
#pragma unroll
            for (int i = 0; i < A_INSTR; ++i) {
                const int q = wave * A_INSTR + i;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rs_x, MNNQ_LDS(lds + St::A_OFF + buf * St::A_BYTES + q * 1024), 16, a_voff,
                    ((int)m0 + q * 8) * K + (c % Cx) * 128, 0, 0);
            }
            // B codes: B_INSTR row tiles per wave, one chunk block (1 KiB) each.
#pragma unroll
            for (int i = 0; i < B_INSTR; ++i) {
                const int j = wave * B_INSTR + i;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::B_OFF + j * 1024), 16, b_voff,
                                                         uniform(((rt0 + j) * C + c) * (W8 == 2 ? 2048 : 1024)), 0, 0);
                if (W8)   // the low nibble plane of the same weights (byte form: the chunk's second group)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::B2_OFF + j * 1024), 16, b_voff,
                                                             uniform(W8 == 2 ? ((rt0 + j) * C + c) * 2048 + 1024
                                                                             : ((rt0 + j) * C + c + Cx) * 1024), 0, 0);
            }
            // Scales: one load covers two row tiles (2 x 128 B), four loads in all; zeros: one load covers
            // all eight row tiles (8 x 32 B).  (wave is uniform: these are scalar branches.)
            if ((WPK == 4 && NT16 == 8) || wave < NT16 / 2)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::S_OFF + wave * 256), 4, s_voff,
                                                         uniform(scales_off + ((rt0 + wave * 2) * C + c) * 128), 0, 0);
            if (MINF) {   // group minima: fp32, laid out like the scales
                if ((WPK == 4 && NT16 == 8) || wave < NT16 / 2)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::Z_OFF + wave * 256), 4, s_voff,
                                                             uniform(zeros_off + ((rt0 + wave * 2) * C + c) * 128), 0, 0);
            } else if (wave == 0)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, MNNQ_LDS(lds + St::Z_OFF + opaque_zero), 4, z_voff,
                                                         uniform(zeros_off + (rt0 * C + c) * 32), 0, 0);
        };

        float yacc[TM][TN][4];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) yacc[i][j][r] = 0.0f;

        // C operand of the MFMAs whose results go to the fp32 epilogue (see there)
        constexpr int kFloatBiasBits = 0x4B400000;
        constexpr float kFloatBias = 12582912.0f;
        v4i fbias = {kFloatBiasBits, kFloatBiasBits, kFloatBiasBits, kFloatBiasBits};
        asm volatile("" : "+v"(fbias));

        v4i bw[TN];
        v4i bw2[W8 ? TN : 1];   // low nibble plane (W8)
        v2i bsv[TN];
        uint32_t bz[TN];      // zero points of both groups (integer zero point form)
        v2i bmn[TN];          // group minima of both groups, fp32 bits (float minimum form)
        auto read_b = [&]() {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                bw[j] = *reinterpret_cast<const v4i*>(lds + b_frag_off + j * 1024);
                if (W8) bw2[j] = *reinterpret_cast<const v4i*>(lds + b_frag_off + (St::B2_OFF - St::B_OFF) + j * 1024);
                bsv[j] = *reinterpret_cast<const v2i*>(lds + s_frag_off + j * 128);
                if (MINF) bmn[j] = *reinterpret_cast<const v2i*>(lds + z_frag_off + j * 128);
                else bz[j] = *reinterpret_cast<const uint16_t*>(lds + z_frag_off + j * 32);
            }
        };

        if (cb < ce) issue_stage(cb, 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        read_b();

        for (int it = 0; it < n_iter; ++it) {
            const int c = cb + it;
            const int buf = it & 1;
            // Every wave holds the B fragments of chunk c in registers and has finished
            // chunk c - 1: the B tile and the other A buffer may be overwritten.
            __syncthreads();
            if (c + 1 < ce) issue_stage(c + 1, buf ^ 1);

            const uint8_t* st = lds + buf * St::A_BYTES;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (KS > 1 && c >= ce) break;   // the shorter share idles through the last round
                v4i b[TN];
                float sc[TN];
                float mnv[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const uint32_t w0 = (uint32_t)(h ? bw[j].z : bw[j].x), w1 = (uint32_t)(h ? bw[j].w : bw[j].y);
                    if (W8 == 2) {
                        // byte form: the sixteen bytes q8 - 128 are the operand
                        b[j] = h ? bw2[j] : bw[j];
                        mnv[j] = __int_as_float(h ? bmn[j].y : bmn[j].x);
                    } else if (W8) {
                        // q8 - 128 per byte: high plane nibble above low plane nibble, top bit flipped
                        const uint32_t l0 = (uint32_t)(h ? bw2[j].z : bw2[j].x), l1 = (uint32_t)(h ? bw2[j].w : bw2[j].y);
                        b[j].x = (int)((((w0 << 4) & 0xf0f0f0f0u) | (l0 & 0x0f0f0f0fu)) ^ 0x80808080u);
                        b[j].y = (int)(((w0 & 0xf0f0f0f0u) | ((l0 >> 4) & 0x0f0f0f0fu)) ^ 0x80808080u);
                        b[j].z = (int)((((w1 << 4) & 0xf0f0f0f0u) | (l1 & 0x0f0f0f0fu)) ^ 0x80808080u);
                        b[j].w = (int)(((w1 & 0xf0f0f0f0u) | ((l1 >> 4) & 0x0f0f0f0fu)) ^ 0x80808080u);
                        mnv[j] = __int_as_float(h ? bmn[j].y : bmn[j].x);
                    } else if (MINF) {
                        // the codes themselves (0..15) are the B operand; the minimum enters in the epilogue
                        b[j].x = (int)(w0 & 0x0f0f0f0fu);
                        b[j].y = (int)((w0 >> 4) & 0x0f0f0f0fu);
                        b[j].z = (int)(w1 & 0x0f0f0f0fu);
                        b[j].w = (int)((w1 >> 4) & 0x0f0f0f0fu);
                        mnv[j] = __int_as_float(h ? bmn[j].y : bmn[j].x);
                    } else {
                        // 0x80 - zero point of this group in each of the four bytes
                        const uint32_t c4 = 0x80808080u - __builtin_amdgcn_perm(bz[j], bz[j], h ? 0x01010101u : 0u);
                        b[j] = unpack_b(w0, w1, c4);
                        mnv[j] = 0.0f;
                    }
                    sc[j] = __int_as_float(h ? bsv[j].y : bsv[j].x);
                    if (W8) {
                        if (W8 == 1) sc[j] *= 0.0625f;            // the high plane stores 16 s (exact)
                        mnv[j] = fmaf(sc[j], 128.0f, mnv[j]);     // min + 128 s
                    }
                }
                const int g = 2 * c + h;
                const uint8_t* ap = st + a_row_off + (((h * 4 + kb) ^ a_sw) << 4);
                const v4i zero = {0, 0, 0, 0};
                if (ACC) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const v4i a = *reinterpret_cast<const v4i*>(ap + i * 2048);
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const v4i d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[j], zero, 0, 0, 0);
                            const int64_t n = (int64_t)(rt0 + wn * TN + j) * 16 + col;
                            if (n < L.N && g < L.G) {
#pragma unroll
                                for (int rr = 0; rr < 4; ++rr) {
                                    const int64_t m = m0 + wm * WM + i * 16 + kb * 4 + rr;
                                    if (m < M) acc_out[(m * L.N + n) * L.G + g] = d[rr];
                                }
                            }
                        }
                    }
                } else {
                    // Software pipeline over the TM x TN tiles of this group: the MFMA of
                    // tile t + 1 is issued before the eight VALU operations that fold tile
                    // t into the running sums.  The empty asm statements emit nothing; they
                    // only tie values together so that this order survives the compiler's
                    // schedulers: MFMA(t+1) < epilogue(t) < MFMA(t+2).
                    // Float minimum form: one more MFMA per 16 rows with an all-ones B operand gives
                    // xs[m] = sum_{k in g} xq[m,k] in the D layout, i.e. for exactly the four rows of
                    // this lane; the epilogue adds min[n,g] * xs[m,g].
                    // int32 -> fp32 without a convert instruction (it runs at a fraction of the rate of the
                    // other vector instructions): the C operand carries the bit pattern of 1.5 * 2^23, so the
                    // MFMA's integer result I + 0x4B400000 is, read as a float, exactly 12582912 + I for
                    // |I| < 2^22 (here |I| <= 64 * 127 * 15), and one exact subtraction gives float(I).
                    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
                    v4i a = *reinterpret_cast<const v4i*>(ap);
                    v4i a_nxt = a;
                    if (TM > 1) a_nxt = *reinterpret_cast<const v4i*>(ap + 2048);
                    v4i d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[0], fbias, 0, 0, 0);
                    v4i xs_cur = zero, xs_nxt = zero;
                    if (MINF) xs_cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, ones, fbias, 0, 0, 0);
                    float xsf[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int tt = 0; tt < TM * TN; ++tt) {
                        const int i = tt / TN, j = tt % TN;
                        v4i d_nxt = d;
                        if (tt + 1 < TM * TN) {
                            const int i1 = (tt + 1) / TN, j1 = (tt + 1) % TN;
                            if (j1 == 0) {
                                a = a_nxt;
                                if (i1 + 1 < TM) a_nxt = *reinterpret_cast<const v4i*>(ap + (i1 + 1) * 2048);
                            }
                            d_nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[j1], fbias, 0, 0, 0);
                            if (MINF && j1 == 0) xs_nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, ones, fbias, 0, 0, 0);
                            asm volatile("" : "+v"(d), "+v"(d_nxt));
                        }
                        if (MINF && j == 0) {
                            if (i > 0) xs_cur = xs_nxt;      // issued with the first MFMA of this row of tiles
#pragma unroll
                            for (int rr = 0; rr < 4; ++rr) xsf[rr] = __int_as_float(xs_cur[rr]) - kFloatBias;
                        }
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            yacc[i][j][rr] = fmaf(sc[j], __int_as_float(d[rr]) - kFloatBias, yacc[i][j][rr]);
                            if (MINF) yacc[i][j][rr] = fmaf(mnv[j], xsf[rr], yacc[i][j][rr]);
                        }
                        if (tt + 2 < TM * TN) {
                            const int j2 = (tt + 2) % TN;
                            asm volatile(""
                                         : "+v"(b[j2]), "+v"(yacc[i][j][0]), "+v"(yacc[i][j][1]),
                                           "+v"(yacc[i][j][2]), "+v"(yacc[i][j][3]));
                        } else {
                            asm volatile(""
                                         : "+v"(yacc[i][j][0]), "+v"(yacc[i][j][1]), "+v"(yacc[i][j][2]),
                                           "+v"(yacc[i][j][3]));
                        }
                        d = d_nxt;
                    }
                }
            }
            if (it + 1 < n_iter) {
                // The loads of chunk c + 1 were issued before this chunk's arithmetic; wait for
                // this wave's part, make every wave's part visible, fetch the B fragments.
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
                __syncthreads();
                if (c + 1 < ce) read_b();
            }
        }
        if (KS > 1) {
            // Add the K parts in a fixed order: part kh > 0 leaves its sums in LDS (one
            // conflict-free float per lane and accumulator), part 0 adds them.
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
        if (!ACC) {
            // Output: y = yacc * sx[m] + bias[n].  Buffer accesses keep this free of
            // branches and 64-bit address arithmetic: rows past M fall outside the
            // buffers (loads give 0, stores are dropped), a NULL bias is an empty buffer.
            const __amdgpu_buffer_rsrc_t rs_sx =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(sx), 0, (int)(M * 4), kBufFlags);
            const __amdgpu_buffer_rsrc_t rs_bias = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(bias), 0, (bias && split == 0) ? (int)(L.N * 4) : 0, kBufFlags);
            const int y_bytes = (int)(uint32_t)(M * L.N * 4);
            const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, kBufFlags);
            const int Nb = (int)L.N * 4;                       // bytes per output row
            const int row0 = (int)m0 + wm * WM;                // first row of this wave
            const int nt0 = rt0 + wn * TN;                     // first row tile (16 outputs) of this wave
            float bj[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bj[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_bias, col * 4, (nt0 + j) * 64, 0));
            if (S == 1) {
                // The 16 x (16 TN) block of one m-tile goes through a private LDS patch of the wave
                // (rows padded by 4 floats: conflict-free both ways) and leaves as 128-bit stores of
                // whole row segments - a quarter of the store instructions and full cache lines.
                // LDS operations of one wave complete in order, so the patch needs no barrier of its
                // own; the barrier in front makes sure no wave still reads operands where it lies.
                static_assert(TN == 4 || TN == 2, "a lane stores one 16-byte unit of a row segment of 64 or 32 columns");
                constexpr int RS = 16 * TN + 4;                // floats per patch row
                constexpr int LPR = 4 * TN;                    // lanes (16-byte units) per row segment
                constexpr int RPP = 64 / LPR;                  // rows a wave stores per instruction
                if (KS == 1) __syncthreads();
                float* patch = reinterpret_cast<float*>(lds_all) + wave * (16 * RS);
                float* wr = patch + (kb * 4) * RS + col;
                const int lr = lane / LPR, lu = lane % LPR;    // this lane's row within a pass and unit within the row
                const float* rd = patch + lr * RS + lu * 4;    // + RPP p rows
                // a lane's 16-byte unit lies in row tile nt0 + lu / 4; units past N are sent out of range
                const bool unit_ok = nt0 + (lu >> 2) < (int)L.T;
                const int y_voff = unit_ok ? lr * Nb + lu * 16 : y_bytes;
                // binary16 output: the same unit is four halves, rows are half as long
                const __amdgpu_buffer_rsrc_t rs_y16 = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes / 2, kBufFlags);
                const int y_voff16 = unit_ok ? lr * (Nb / 2) + lu * 8 : y_bytes / 2;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    float sxr[4];
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        sxr[rr] = __uint_as_float(
                            __builtin_amdgcn_raw_buffer_load_b32(rs_sx, kb * 16, (row0 + i * 16 + rr) * 4, 0));
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                        for (int j = 0; j < TN; ++j) wr[rr * RS + j * 16] = fmaf(yacc[i][j][rr], sxr[rr], bj[j]);
#pragma unroll
                    for (int p = 0; p < 16 / RPP; ++p) {
                        // (read as a struct of floats: the same scalar type as the writes for alias analysis)
                        const float4 f = *reinterpret_cast<const float4*>(rd + p * RPP * RS);
                        if (L.out16) {
                            const h2v lo = {(_Float16)f.x, (_Float16)f.y}, hi = {(_Float16)f.z, (_Float16)f.w};
                            const v2i v = {(int)h2_bits(lo), (int)h2_bits(hi)};
                            __builtin_amdgcn_raw_buffer_store_b64(v, rs_y16, y_voff16,
                                                                  (row0 + i * 16 + p * RPP) * (Nb / 2) + nt0 * 32, 0);
                            continue;
                        }
                        const v4i v = {(int)__float_as_uint(f.x), (int)__float_as_uint(f.y), (int)__float_as_uint(f.z),
                                       (int)__float_as_uint(f.w)};
                        __builtin_amdgcn_raw_buffer_store_b128(v, rs_y, y_voff,
                                                               (row0 + i * 16 + p * RPP) * Nb + nt0 * 64, 0);
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    float sxr[4];
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        sxr[rr] = __uint_as_float(
                            __builtin_amdgcn_raw_buffer_load_b32(rs_sx, kb * 16, (row0 + i * 16 + rr) * 4, 0));
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            if (nt0 + j >= (int)L.T) continue;     // wave-uniform
                            const float v = fmaf(yacc[i][j][rr], sxr[rr], bj[j]);
                            const int64_t m = (int64_t)row0 + i * 16 + kb * 4 + rr;
                            if (m < M) atomicAdd(&y[m * L.N + (int64_t)(nt0 + j) * 16 + col], v);
                        }
                    }
                }
            }
        }
    }
}

__global__ void zero_f4_kernel(float4* p, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) p[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}

template <int BM, int BN, int KS, bool ACC, bool MINF, int W8 = 0, int WNW = 2>
int launch_tiles_m(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                 const float* bias, float* y, int32_t* acc, int S, hipStream_t st)
{
    const int MT = (int)((M + BM - 1) / BM);
    const int NT = (int)((L.N + BN - 1) / BN);
    constexpr size_t smem = (size_t)KS * Lds<BM, BN, MINF, W8>::BYTES;
    auto kern = prefill_kernel<BM, BN, KS, ACC, MINF, W8, WNW>;
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
    if (S > 1) {
        const int64_t n4 = M * L.N / 4;      // N is a multiple of 16
        hipLaunchKernelGGL(zero_f4_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st,
                           reinterpret_cast<float4*>(y), n4);
        MNNQ_HIP_TRY(hipGetLastError());
    }
    const int64_t blocks = (int64_t)MT * S * ((NT + 7) / 8) * 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(128 * WNW * KS), smem, st, packed, L, M, xq, sx, bias, y, acc, MT,
                       NT, S);
    MNNQ_HIP_TRY(hipGetLastError());
    return MNNQ_OK;
}

template <int BM, int BN, int KS, bool ACC>
int launch_tiles(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                 const float* bias, float* y, int32_t* acc, int S, hipStream_t st)
{
    if (L.minf)
        return launch_tiles_m<BM, BN, KS, ACC, true>(packed, L, M, xq, sx, bias, y, acc, S, st);
    return launch_tiles_m<BM, BN, KS, ACC, false>(packed, L, M, xq, sx, bias, y, acc, S, st);
}

// Eight waves per K part (128 x 32 or 64 x 32 outputs per wave).
template <int BM, int KS>
int launch_wide(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                const float* bias, float* y, int S, hipStream_t st)
{
    if (L.minf) {
        if constexpr (BM == 256 && KS == 2) return MNNQ_ERR_UNSUPPORTED;   // not built: see launch_prefill
        else return launch_tiles_m<BM, 128, KS, false, true, false, 4>(packed, L, M, xq, sx, bias, y, nullptr, S, st);
    }
    return launch_tiles_m<BM, 128, KS, false, false, false, 4>(packed, L, M, xq, sx, bias, y, nullptr, S, st);
}

// Tile, K-part and split choice.  A SIMD is full with four waves of the forms that need at most
// 128 registers (eight waves per K part: 128 x 32 or 64 x 32 outputs per wave), with two otherwise.
//   * 256-row tiles share one B unpack between 8 MFMAs and are preferred when they
//     alone give every CU two workgroups (of eight waves each);
//   * with at most one 128-row tile per CU, the tile's K range is split inside the
//     workgroup (two K parts of eight waves), which fills the SIMDs without any traffic
//     through memory;
//   * in between (more 128-row tiles than CUs, fewer than two each) a second round of
//     workgroups would run on a few CUs only; 256-row tiles with the same K split inside the
//     workgroup use fewer CUs but use them fully;
//   * a split of K over two workgroups (S = 2, fp32 atomics onto a zeroed y) is left
//     for long rows with so few tiles that most CUs would idle.
struct TilePlan {
    bool big;
    int KS;
    int S;
    bool wide;   // 256-row tile worked on by eight waves (128 x 32 outputs each), two workgroups per CU
    bool tiny;   // 64-row tile (few tokens): the call is bound by the weight stream, not by the MFMAs
    bool narrow; // ... of 64 columns: twice the workgroups for layers with few output columns
};

TilePlan plan_tiles(const Layout& L, int64_t M)
{
    TilePlan p{true, 1, 1, false, false, false};
    const int64_t cus = num_cus();
    auto tiles = [&](int bm) { return ((M + bm - 1) / bm) * ((L.N + 127) / 128); };
    if (M <= 128 && L.mode != MNNQ_W8_MIN_FLOAT && !(M > 64 && tiles(128) >= 4 * cus)) {
        // Up to 128 tokens (batched decoding): 64-row tiles, a quarter of the MFMAs of a 128-row tile
        // per chunk.  Such a call is bound by stalls, not by the MFMAs, and runs the faster the more
        // waves a CU holds: 64-column tiles (twice the workgroups, of 21 KiB of LDS each) unless there
        // are very many tiles, the K range in 1, 2 or 4 parts of four waves, and long rows also cut in
        // two.  (Beyond 64 tokens and with that many tiles, 128-row tiles are faster: the plans below.)
        p.big = false;
        p.tiny = true;
        int64_t t = tiles(64);
        if (t < 4 * cus) {
            p.narrow = true;
            t *= 2;
        }
        p.KS = t >= 4 * cus ? 1 : (2 * t >= cus ? 2 : 4);
        if (4 * t <= cus && L.C >= 64) p.S = 2;
    } else if (M > 128 && tiles(256) >= 2 * cus) {
        p.big = true;
        p.wide = !L.minf;   // the float minimum form needs more registers than four waves per SIMD leave
    } else if (tiles(128) <= cus) {
        p.big = false;
        p.KS = 2;
        p.wide = true;      // sixteen waves: two K parts of eight
        if (tiles(128) * 2 <= cus && L.C >= 64) p.S = 2;
    } else if (tiles(128) < 2 * cus) {
        // (float minimum form: the sixteen-wave 256-row form would spill; eight waves on 128-row tiles
        // measured 5 - 9 % faster than two K parts of four waves on 256-row tiles)
        p.big = M > 128 && !L.minf;
        p.KS = p.big ? 2 : 1;
        p.wide = p.big || L.minf;
    } else {
        p.big = false;
    }
    if (const char* e = debug_option(kDbgPrefillTile)) {   // tuning and tests: "b"/"s", split digit, "k" = K parts
        if (e[0] == 'b' || e[0] == 'w') p.big = true;
        if (e[0] == 's' || e[0] == 'v' || e[0] == 't' || e[0] == 'n') p.big = false;
        p.wide = (e[0] == 'w' || e[0] == 'v');     // "w"/"v" = "b"/"s" worked on by twice the waves
        p.tiny = (e[0] == 't' || e[0] == 'n') && L.mode != MNNQ_W8_MIN_FLOAT;   // "t" = 64-row tile; "k" / "q" = 2 / 4 K parts
        p.narrow = p.tiny && e[0] == 'n';                                        // "n" = 64 x 64 tile
        if (e[0] && (e[1] == '1' || e[1] == '2' || e[1] == '4')) {
            p.S = e[1] - '0';
            p.KS = (e[2] == 'k') ? 2 : ((e[2] == 'q' && p.tiny) ? 4 : 1);
        }
    }
    return p;
}

}  // namespace

int num_cus()
{
    static thread_local int cached_dev = -1, cached = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev != cached_dev) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached = n;
        cached_dev = dev;
    }
    return cached;
}

namespace {

// What launch_prefill starts for a shape: tile rows, K parts inside the workgroup, K split over
// workgroups, waves along N per K part (2 x WNW waves each), merged nibble planes of int8 weights.
struct PrefillLaunch {
    int BM, KS, S, WNW;
    bool w8;
    int BN;
};

PrefillLaunch resolve_prefill(const Layout& L, int64_t M)
{
    TilePlan p = plan_tiles(L, M);
    if (L.out16) p.S = 1;   // the split over two workgroups adds fp32 partial sums in the output array
    const bool forced_plan = debug_option(kDbgPrefillTile) != nullptr;
    PrefillLaunch r{p.big ? 256 : (p.tiny ? 64 : 128), p.KS, p.S, 2, false, p.narrow ? 64 : 128};
    // 8-bit weights: both nibble planes of a chunk in one MFMA (128-row tiles: two B tiles need the LDS
    // of the larger A tile).  MNNQ_W8_PLANES=1 (tests, comparisons) keeps one MFMA per plane instead.
    const char* planes = debug_option(kDbgW8Planes);
    if (L.mode == MNNQ_W8_MIN_FLOAT && (L.native8 || !(planes && planes[0] == '1'))) {
        r.w8 = true;
        r.BM = 128;
        const int64_t tiles128 = ((M + 127) / 128) * ((L.N + 127) / 128), cus = num_cus();
        if (!forced_plan) {   // the plan above counted 256-row tiles too
            r.KS = tiles128 <= cus ? 2 : 1;
            r.WNW = tiles128 < 2 * cus ? 4 : 2;     // few tiles: twice the waves on each
        } else {
            r.WNW = p.wide ? 4 : 2;
        }
        if (r.S > 1 && L.Cx < 64) r.S = 1;
        return r;
    }
    // twice the waves per tile; the combinations not listed run in the four-wave form
    if (p.wide && ((r.BM == 256 && r.KS == 1) || (r.BM == 256 && r.KS == 2 && !L.minf) || r.BM == 128))
        r.WNW = 4;   // (256 rows, two K parts, float minimum form: would spill registers)
    return r;
}

static_assert(Lds<256, 128, false>::BYTES == 2 * 256 * 128 + 8 * 1024 + 8 * 128 + 8 * 32, "prefill_lds_bytes");
static_assert(Lds<128, 128, true, true>::BYTES == 2 * 128 * 128 + 16 * 1024 + 8 * 128 + 8 * 128, "prefill_lds_bytes");
static_assert(Lds<64, 64, false>::BYTES == 2 * 64 * 128 + 4 * 1024 + 4 * 128 + 8 * 32, "prefill_lds_bytes");

size_t prefill_lds_bytes(const PrefillLaunch& r, bool minf)
{
    const int nt16 = r.BN / 16;
    return (size_t)r.KS * (2 * r.BM * 128 + nt16 * 1024 * (r.w8 ? 2 : 1) + nt16 * 128 + (minf ? nt16 * 128 : 8 * 32));
}

}  // namespace

void describe_prefill(const Layout& L, int64_t M, int32_t out[8])
{
    const PrefillLaunch r = resolve_prefill(L, M);
    const int64_t MT = (M + r.BM - 1) / r.BM, NT = (L.N + r.BN - 1) / r.BN;
    out[0] = r.BM;
    out[1] = r.BN;
    out[2] = r.KS;
    out[3] = r.S;
    out[4] = 2 * r.WNW * r.KS;                                   // waves per workgroup
    out[5] = (int32_t)prefill_lds_bytes(r, L.minf);
    out[6] = (int32_t)(MT * r.S * ((NT + 7) / 8) * 8);           // workgroups
    out[7] = r.w8 ? (L.native8 ? 2 : 1) : 0;   // int8 weights: merged nibble planes / byte form
}

int launch_prefill(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                   const float* bias, float* y, int32_t* acc_debug, hipStream_t st)
{
    if (acc_debug) {
        if (M > 128) return launch_tiles<256, 128, 1, true>(packed, L, M, xq, sx, bias, y, acc_debug, 1, st);
        return launch_tiles<128, 128, 1, true>(packed, L, M, xq, sx, bias, y, acc_debug, 1, st);
    }
    const PrefillLaunch r = resolve_prefill(L, M);
#define MNNQ_ARGS packed, L, M, xq, sx, bias, y, nullptr, r.S, st
    if (r.w8 && L.native8) {   // byte form: the chunk's two kilobytes are the two groups' operands
        if (r.KS == 2 && r.WNW == 4) return launch_tiles_m<128, 128, 2, false, true, 2, 4>(MNNQ_ARGS);
        if (r.WNW == 4) return launch_tiles_m<128, 128, 1, false, true, 2, 4>(MNNQ_ARGS);
        if (r.KS == 2) return launch_tiles_m<128, 128, 2, false, true, 2>(MNNQ_ARGS);
        return launch_tiles_m<128, 128, 1, false, true, 2>(MNNQ_ARGS);
    }
    if (r.w8) {
        if (r.KS == 2 && r.WNW == 4) return launch_tiles_m<128, 128, 2, false, true, true, 4>(MNNQ_ARGS);
        if (r.WNW == 4) return launch_tiles_m<128, 128, 1, false, true, true, 4>(MNNQ_ARGS);
        if (r.KS == 2) return launch_tiles_m<128, 128, 2, false, true, true>(MNNQ_ARGS);
        return launch_tiles_m<128, 128, 1, false, true, true>(MNNQ_ARGS);
    }
    if (r.WNW == 4) {
        if (r.BM == 256 && r.KS == 1) return launch_wide<256, 1>(packed, L, M, xq, sx, bias, y, r.S, st);
        if (r.BM == 256) return launch_wide<256, 2>(packed, L, M, xq, sx, bias, y, r.S, st);
        if (r.KS == 2) return launch_wide<128, 2>(packed, L, M, xq, sx, bias, y, r.S, st);
        return launch_wide<128, 1>(packed, L, M, xq, sx, bias, y, r.S, st);
    }
    if (r.BM == 64 && r.BN == 64) {
        if (r.KS == 4) return launch_tiles<64, 64, 4, false>(MNNQ_ARGS);
        if (r.KS == 2) return launch_tiles<64, 64, 2, false>(MNNQ_ARGS);
        return launch_tiles<64, 64, 1, false>(MNNQ_ARGS);
    }
    if (r.BM == 64) {
        if (r.KS == 4) return launch_tiles<64, 128, 4, false>(MNNQ_ARGS);
        if (r.KS == 2) return launch_tiles<64, 128, 2, false>(MNNQ_ARGS);
        return launch_tiles<64, 128, 1, false>(MNNQ_ARGS);
    }
    if (r.BM == 256 && r.KS == 2) return launch_tiles<256, 128, 2, false>(MNNQ_ARGS);
    if (r.BM == 256) return launch_tiles<256, 128, 1, false>(MNNQ_ARGS);
    if (r.KS == 2) return launch_tiles<128, 128, 2, false>(MNNQ_ARGS);
    return launch_tiles<128, 128, 1, false>(MNNQ_ARGS);
#undef MNNQ_ARGS
}

}  // namespace mnnq
