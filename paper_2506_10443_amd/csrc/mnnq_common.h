// Shared definitions of the mnnq HIP library (gfx950 only).
//
// Packed weight layout ("chunk layout").  The paper rearranges weights once at
// load so that the inner loop reads exactly what one instruction consumes
// (Section 5.1); on CDNA4 the unit is one 128-bit load per lane of a 64-wide
// wavefront:
//
//   row tile  t = n / 16            (16 output rows)
//   chunk     c = g / 2             (two quantization groups = 128 values of K)
//   C = ceil(G / 2) chunks per row tile; an odd G gets one zero padding group.
//
//   codes  : [T][C][64 lanes][16 B]   at byte 0
//            lane l serves row 16 t + (l % 16), k-block kb = l / 16;
//            bytes 0..7  = its 16 codes of group 2c   (k = 64 (2c)   + 16 kb + j),
//            bytes 8..15 = its 16 codes of group 2c+1 (k = 64 (2c+1) + 16 kb + j).
//            Inside 8 bytes, dword d, byte b holds code j = 8 d + b in the low
//            nibble and code j = 8 d + 4 + b in the high nibble, so that
//            `w & 0x0f0f0f0f` and `(w >> 4) & 0x0f0f0f0f` give codes 8d..8d+3
//            and 8d+4..8d+7 in byte order.
//   scales : [T][C][16 rows][2] fp32  at byte T*C*1024
//   zeros  : [T][C][16 rows][2] u8    at byte T*C*1024 + T*C*128        (mode MNNQ_W4_ZP_INT)
//   mins   : [T][C][16 rows][2] fp32  at the same place                 (mode MNNQ_W4_MIN_FLOAT:
//            the group minimum of Eq. 1 as a float offset instead of an integer zero point)
//
// One chunk is exactly one wave-wide 128-bit load (1 KiB) for the decode GEMV,
// and lane l's 16 bytes are exactly its B operands of two 16x16x64 int8 MFMAs
// (one per group) for the prefill GEMM.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/mnnq.h"

namespace mnnq {

constexpr int kGroup = 64;
constexpr int kTileN = 16;
constexpr int kChunkBytes = 1024;

// int8 weights (mode MNNQ_W8_MIN_FLOAT) reuse this layout and the int4 kernels: a code
// q8 = 16 hi + lo is stored as two 4-bit planes along a doubled reduction axis - groups
// 0..G-1 hold the high nibbles with step 16 s and the group minimum, groups G..2G-1 the low
// nibbles with step s and minimum 0 - so that q8 s + min = hi (16 s) + min + lo s.  The
// activation row is not doubled: chunk c of the packed matrix meets chunk c % Cx of the row.
// Byte form of int8 weights (mode flag MNNQ_NATIVE_8BIT): the reduction axis is not doubled; chunk
// (t, c) is two kilobytes, one per group - lane l of kilobyte h holds the 16 codes k = 64 (2 c + h) +
// 16 (l / 16) + j of row 16 t + l % 16 as bytes q8 - 128, i.e. the B operand of v_mfma_i32_16x16x64_i8 and
// of four v_dot4_i32_i8 as it stands; scales (the step s) and minima [T][C][16][2] fp32 as in the float
// minimum form.  With D = sum xq (q8 - 128) and xs = sum xq a group's term is  s D + (min + 128 s) xs.
// Matrix-core plane (mode flag MNNQ_WITH_MATRIX_PLANE): a second copy of the int4 weights behind the
// chunk layout, as the B operand of the fp6 matrix instruction v_mfma_scale_f32_32x32x64_f8f6f4 -
// every q - zero (|q - zero| <= 15) is the e2m3 value (q - zero) / 8 exactly, and its code is the
// sign-magnitude form of q - zero.  Unit: column tile tn = n / 32 and group g (64 values of K):
//   codes  [G][T32p][1536 B]: lane l (0..63) holds column 32 tn + l % 32 and the 32 values
//          k = 64 g + 32 (l / 32) + j, j = 0..31, code j at bits [6 j, 6 j + 6) of its 192 bits;
//          dwords 0..3 of lane l at byte 16 l, dwords 4..5 at byte 1024 + 8 l of the block;
//   scales [G][T32p][32] fp32 behind the codes.
// T32p = column tiles rounded up to a multiple of 8 (zero codes and scales in the padding), so that a
// workgroup's tile of up to 256 columns is one contiguous, in-range piece per group.
constexpr int kPlaneBlockBytes = 1536;
constexpr int kPlaneTilePad = 8;

struct Layout {
    int64_t N, K;   // K: length of the packed reduction axis (2 x the row length for int8 weights)
    int64_t Kx;     // length of an activation row
    int64_t Cx;     // chunks of an activation row
    int mode;       // mnnq_mode
    bool minf;      // groups carry an fp32 minimum instead of a one-byte zero point
    bool out16;     // the output array holds IEEE binary16 values (set per call, not a property of the packing)
    int64_t T;  // row tiles
    int64_t G;  // groups per row
    int64_t C;  // chunks per row tile
    size_t codes_bytes, scales_bytes, zeros_bytes;
    bool native8;     // int8 weights as bytes: a chunk is two kilobytes, one per group (see below)
    bool plane;       // the packed buffer carries the matrix-core plane behind the chunk layout
    int64_t T32p;     // column tiles of 32 in the plane (padded to a multiple of 8)
    int64_t Gx;       // quantization groups of an activation row (= groups of the plane)
    __host__ __device__ size_t scales_off() const { return codes_bytes; }
    __host__ __device__ size_t zeros_off() const { return codes_bytes + scales_bytes; }
    // bytes of the chunk layout (what the decode kernels and the int8 GEMM read)
    __host__ __device__ size_t total() const { return codes_bytes + scales_bytes + zeros_bytes; }
    __host__ __device__ size_t plane_off() const { return (total() + 255) / 256 * 256; }
    __host__ __device__ size_t plane_codes_bytes() const { return (size_t)Gx * T32p * kPlaneBlockBytes; }
    __host__ __device__ size_t plane_scales_bytes() const { return (size_t)Gx * T32p * 32 * sizeof(float); }
    __host__ __device__ size_t plane_bytes() const { return plane_codes_bytes() + plane_scales_bytes(); }
    // bytes of the whole packed buffer
    __host__ __device__ size_t full_total() const { return plane ? plane_off() + plane_bytes() : total(); }
};

constexpr int kModeMask = 15;

inline __host__ __device__ Layout make_layout(int64_t N, int64_t K, int mode_and_flags = MNNQ_W4_ZP_INT)
{
    Layout L;
    const int mode = mode_and_flags & kModeMask;
    L.plane = (mode_and_flags & MNNQ_WITH_MATRIX_PLANE) != 0;
    L.T32p = ((N + 31) / 32 + kPlaneTilePad - 1) / kPlaneTilePad * kPlaneTilePad;
    L.Gx = K / kGroup;
    L.N = N;
    L.native8 = mode == MNNQ_W8_MIN_FLOAT && (mode_and_flags & MNNQ_NATIVE_8BIT) != 0;
    L.Kx = K;
    L.K = (mode == MNNQ_W8_MIN_FLOAT && !L.native8) ? 2 * K : K;
    L.mode = mode;
    L.minf = (mode != MNNQ_W4_ZP_INT);
    L.out16 = false;
    L.T = N / kTileN;
    L.G = L.K / kGroup;
    L.C = (L.G + 1) / 2;
    L.Cx = (K / kGroup + 1) / 2;
    L.codes_bytes = (size_t)L.T * L.C * kChunkBytes * (L.native8 ? 2 : 1);
    L.scales_bytes = (size_t)L.T * L.C * 32 * sizeof(float);
    L.zeros_bytes = (size_t)L.T * L.C * 32 * (L.minf ? sizeof(float) : 1);
    return L;
}

#if defined(__HIPCC__)
// One output value: fp32, or rounded once (nearest even) to binary16 when the call asked for it.
__device__ __forceinline__ void store_out(float* y, int64_t i, float v, bool out16)
{
    if (out16) reinterpret_cast<_Float16*>(y)[i] = (_Float16)v;
    else y[i] = v;
}

// Activation codes (Section 4.2, per-token symmetric int8): the definition is
// clamp(rint(fl(x / scale)), -127, 127) with IEEE binary32 operations, but
// a correctly rounded division per element is expensive (about ten vector
// instructions).  r = x * fl(1 / scale) differs from fl(x / scale) by
// less than 3 * 2^-24 * 127.5 < 2.3e-5, so both round to the same integer unless
// r is within that distance of a half-integer, i.e. unless |r - rint(r)| (exact:
// the two are within 0.5 of each other) exceeds 0.5 - 6e-5; only then (about one
// element in ten thousand) the division is done, for the four elements of a dword
// together.  |r| <= 127 (1 + 2^-22) in this path, so rint(r) needs no clamp.
// (lim is 0.5 - 6e-5 normally; negative - "always divide" - when 1 / scale is not
// a normal number; the division path clamps as the definition does.)
// rint(r) itself is taken from the sum r + 1.5 * 2^23 (round to nearest even happens in the
// addition), which costs an add and a subtract instead of a rounding and a convert instruction
// per element - converts run at a fraction of the rate of the other vector instructions.
// Callers are compiled with -ffp-contract=off: x * inv - rint(x * inv) must be a
// product rounded to binary32 and an exact subtraction.
__device__ __forceinline__ int quant4_fast(float4 v, float scale, float inv, float lim)
{
    // Round to nearest even by adding 1.5 * 2^23: for |r| < 2^22 the sum is exactly 12582912 + rint(r),
    // and its bit pattern is 0x4B400000 + rint(r), i.e. the low byte already is the int8 code.
    constexpr float kMagic = 12582912.0f;
    const float r0 = v.x * inv, r1 = v.y * inv, r2 = v.z * inv, r3 = v.w * inv;
    float m0 = r0 + kMagic, m1 = r1 + kMagic, m2 = r2 + kMagic, m3 = r3 + kMagic;
    const float d0 = fabsf(r0 - (m0 - kMagic)), d1 = fabsf(r1 - (m1 - kMagic));
    const float d2 = fabsf(r2 - (m2 - kMagic)), d3 = fabsf(r3 - (m3 - kMagic));
    if (!(fmaxf(fmaxf(d0, d1), fmaxf(d2, d3)) <= lim)) {
        m0 = fminf(fmaxf(rintf(v.x / scale), -127.0f), 127.0f) + kMagic;
        m1 = fminf(fmaxf(rintf(v.y / scale), -127.0f), 127.0f) + kMagic;
        m2 = fminf(fmaxf(rintf(v.z / scale), -127.0f), 127.0f) + kMagic;
        m3 = fminf(fmaxf(rintf(v.w / scale), -127.0f), 127.0f) + kMagic;
    }
    // low bytes of the four patterns into one dword
    const uint32_t lo = __builtin_amdgcn_perm(__float_as_uint(m1), __float_as_uint(m0), 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(__float_as_uint(m3), __float_as_uint(m2), 0x04000c0cu);
    return (int)(lo | hi);
}

// Lane exchange inside a row of 16 lanes as an operand modifier of the vector ALU (a general shuffle
// goes through the LDS pipe and costs a round trip each).  CTRL: 0xB1 / 0x4E = lanes xor 1 / xor 2
// of a quad, 0x141 / 0x140 = mirror of 8 / of 16 lanes.
template <int CTRL>
__device__ __forceinline__ int row_exchange(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}

// Maximum of a non-negative, non-NaN value over the wave (as integers: the order of such floats),
// the same in all lanes.
__device__ __forceinline__ float wave_max_nonneg(float a)
{
    int v = __float_as_int(a);
    v = max(v, row_exchange<0xB1>(v));
    v = max(v, row_exchange<0x4E>(v));
    v = max(v, row_exchange<0x141>(v));
    v = max(v, row_exchange<0x140>(v));     // every lane: maximum of its row of 16
    const int m = max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
                      max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
    return __int_as_float(m);
}

// Sum over each row of 16 lanes, the same in all of its lanes.
__device__ __forceinline__ int row_sum16(int v)
{
    v += row_exchange<0xB1>(v);
    v += row_exchange<0x4E>(v);
    v += row_exchange<0x141>(v);     // the quads hold equal values: the mirrored lane is in the other quad
    v += row_exchange<0x140>(v);
    return v;
}

__device__ __forceinline__ float quant_fast_limit(float scale, float inv)
{
    return (inv < 1.0e37f && scale > 1.0e-30f) ? 0.5f - 6.0e-5f : -1.0f;   // largest |r - rint(r)| of the fast path
}

#endif

// Test and tuning switches (mnnq_debug_set): nullptr unless set by that call.  The launch plans depend
// on the shapes alone otherwise; the environment is never read.
enum DebugKey {
    kDbgDecodeKsplit, kDbgDecodeWaves, kDbgDecodeEarly, kDbgPrefillTile, kDbgNoSkinny, kDbgSkinnyStaged,
    kDbgW8Planes, kDbgFusedTwoKernelMib, kDbgPrefill6Plan, kDbgPrefill6Stages, kDbgCount
};
const char* debug_option(DebugKey key);

// Records a failing HIP call for mnnq_last_hip_error() and maps it to a status.
int record_hip_error(hipError_t e);

#define MNNQ_HIP_TRY(expr)                                   \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return ::mnnq::record_hip_error(e_); \
    } while (0)

// Kernel launchers (one translation unit each).  All return a status.
int launch_pack(const float* W, const Layout& L, uint8_t* packed, hipStream_t st);
// zero: uint8 zero points (mode MNNQ_W4_ZP_INT) or fp32 group minima (mode MNNQ_W4_MIN_FLOAT), [N, G].
int launch_repack(const uint8_t* q, const float* scale, const void* zero, const Layout& L, uint8_t* packed,
                  hipStream_t st);
int launch_unpack(const uint8_t* packed, const Layout& L, uint8_t* q, float* scale, void* zero,
                  hipStream_t st);
int launch_quant_act(const float* x, int64_t M, int64_t K, int8_t* xq, float* sx, int32_t* xsum,
                     hipStream_t st);
int launch_decode(const uint8_t* packed, const Layout& L, const int8_t* xq, const float* sx,
                  const float* bias, float* y, hipStream_t st);
int launch_decode_fused(const uint8_t* packed, const Layout& L, const float* x, const float* bias, float* y,
                        hipStream_t st);
int launch_decode_acc(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq,
                      int32_t* acc, hipStream_t st);
int launch_prefill(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq,
                   const float* sx, const float* bias, float* y, int32_t* acc_debug, hipStream_t st);
// GEMM on the fp6 matrix instructions (mnnq_prefill6.hip): needs the matrix-core plane in the packed
// buffer and `planes_ws`, prefill6_ws_bytes(M, K) bytes of scratch for the activation planes.
int launch_plane_build(uint8_t* packed, const Layout& L, hipStream_t st);
// planes: the activation planes launch_act_planes wrote for the same M and K.
int launch_act_planes(const int8_t* xq, int64_t M, int64_t K, void* planes, hipStream_t st);
int launch_prefill6(const uint8_t* packed, const Layout& L, int64_t M, const void* planes, const float* sx,
                    const float* bias, float* y, int32_t* acc_debug, hipStream_t st);
size_t prefill6_ws_bytes(int64_t M, int64_t K);
// possible: the plane is there, more than 32 tokens, sizes within the kernels' 32-bit offsets;
// wanted: possible, and the shape has enough output tiles for this GEMM to beat the int8 one (or a plan is forced).
bool prefill6_possible(const Layout& L, int64_t M);
bool prefill6_wanted(const Layout& L, int64_t M);
void describe_prefill6(const Layout& L, int64_t M, int32_t out[8]);
// M <= 16 tokens sharing one pass over the weights.
int launch_skinny(const uint8_t* packed, const Layout& L, int64_t M, const int8_t* xq, const float* sx,
                  const float* bias, float* y, hipStream_t st);
int launch_decode_f16(const uint8_t* packed, const Layout& L, const uint16_t* x16, const float* bias,
                      float* y, hipStream_t st);
// rs: optional per-row factor applied to the fp32 sums before the bias (NULL = none).
int launch_prefill_f16(const uint8_t* packed, const Layout& L, int64_t M, const uint16_t* x16,
                       const float* rs, const float* bias, float* y, hipStream_t st);

// Compute units of the current device (cached per thread and device).
int num_cus();

// LDS of a workgroup on gfx950, and the amount a kernel may use without asking.
constexpr size_t kLdsPerWorkgroup = 160 * 1024;
constexpr size_t kLdsDefault = 64 * 1024;

// Allows `kern` more than 64 KiB of dynamic LDS (needed once per kernel and device; remembered per
// thread in `allowed_dev`, which starts at -1).  Returns a status.
template <typename Kernel>
int allow_large_lds(Kernel kern, size_t bytes, int& allowed_dev)
{
    if (bytes <= kLdsDefault) return MNNQ_OK;
    if (bytes > kLdsPerWorkgroup) return MNNQ_ERR_UNSUPPORTED;
    int dev = 0;
    MNNQ_HIP_TRY(hipGetDevice(&dev));
    if (allowed_dev != dev) {
        MNNQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)kLdsPerWorkgroup));
        allowed_dev = dev;
    }
    return MNNQ_OK;
}

// Launch configuration the launchers above would choose (host logic only, nothing is launched).
// prefill: {tile rows, tile columns, K parts in the workgroup, K split over workgroups, waves per
// workgroup, LDS bytes, workgroups, 1 if the nibble planes of int8 weights are merged};
// decode: {waves per workgroup, waves per row tile, chunks held in registers, 1 if the wave loops with
// a prefetch, LDS bytes, workgroups, row tiles per workgroup, 0}.
void describe_prefill(const Layout& L, int64_t M, int32_t out[8]);
void describe_decode(const Layout& L, bool fused, int32_t out[8]);

}  // namespace mnnq
