// C-ABI entry points of libmnnq.so: argument validation (all of it before the
// first HIP call), then the kernel launchers.
#include "mnnq_common.h"

#include <stdlib.h>
#include <string.h>

#include <mutex>

namespace mnnq {

static thread_local int t_last_hip_error = 0;

int record_hip_error(hipError_t e)
{
    t_last_hip_error = (int)e;
    return MNNQ_ERR_HIP;
}

namespace {
struct DebugSlot {
    const char* name;
    char value[16];
    bool set;
};
DebugSlot g_debug[kDbgCount] = {
    {"MNNQ_DECODE_KSPLIT", "", false},  {"MNNQ_DECODE_WAVES", "", false},   {"MNNQ_DECODE_EARLY", "", false},
    {"MNNQ_PREFILL_TILE", "", false},   {"MNNQ_NO_SKINNY", "", false},      {"MNNQ_SKINNY_STAGED", "", false},
    {"MNNQ_W8_PLANES", "", false},      {"MNNQ_FUSED_TWO_KERNEL_MIB", "", false}, {"MNNQ_PREFILL6_PLAN", "", false},
    {"MNNQ_PREFILL6_STAGES", "", false}};
}  // namespace

const char* debug_option(DebugKey key) { return g_debug[key].set ? g_debug[key].value : nullptr; }

namespace {

constexpr int64_t kMaxDecodeK = 126976;    // int8 row + block sums in LDS: 160 B per 128 k, under 160 KiB
// fp16 row in LDS: sixteen waves stage ceil(C / 16) chunks of 128 values each, 256 B per chunk, plus 1 KiB
// of partial sums, under 160 KiB: at most 39 chunks per wave, C <= 624
constexpr int64_t kMaxDecodeKF16 = 79872;
constexpr int64_t kMaxDecodeKF16Min = 71680;  // float minimum form: 32 B of block sums more per chunk (35 chunks per wave)
constexpr int64_t kMaxM = 65535;

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Shape / mode checks shared by every call.  Returns MNNQ_OK or the error.
int check_shape(int64_t N, int64_t K, int group, int mode_and_flags)
{
    if (N <= 0 || K <= 0) return MNNQ_ERR_SHAPE;
    const int mode = mode_and_flags & kModeMask;
    if (mode_and_flags < 0 || (mode_and_flags & ~(kModeMask | MNNQ_WITH_MATRIX_PLANE | MNNQ_NATIVE_8BIT)))
        return MNNQ_ERR_UNSUPPORTED;
    // the byte form is a form of the int8 weights
    if ((mode_and_flags & MNNQ_NATIVE_8BIT) && mode != MNNQ_W8_MIN_FLOAT) return MNNQ_ERR_UNSUPPORTED;
    // the matrix-core plane holds q - zero: integer zero point form only
    if ((mode_and_flags & MNNQ_WITH_MATRIX_PLANE) && mode != MNNQ_W4_ZP_INT) return MNNQ_ERR_UNSUPPORTED;
    if (group != kGroup || mode < MNNQ_W4_ZP_INT || mode > MNNQ_W8_MIN_FLOAT) return MNNQ_ERR_UNSUPPORTED;
    if (K % group != 0) return MNNQ_ERR_SHAPE;
    if (mode == MNNQ_W8_MIN_FLOAT && K % (2 * group) != 0) return MNNQ_ERR_UNSUPPORTED;   // whole chunks per plane
    if (N % kTileN != 0) return MNNQ_ERR_UNSUPPORTED;
    if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24) return MNNQ_ERR_UNSUPPORTED;
    return MNNQ_OK;
}

// The prefill kernel addresses the activations and the packed weights with
// 32-bit buffer offsets.
size_t fused_ws_bytes(int64_t K) { return (size_t)((K + 127) / 128 * 128 + 16); }

// Scratch of the fused prefill call: the int8 codes [M, K], then the fp32 scales [M], each part
// rounded up to 16 bytes.
size_t fused_prefill_codes_bytes(int64_t M, int64_t K) { return (size_t)((M * K + 15) / 16 * 16); }
size_t fused_prefill_ws_bytes(int64_t M, int64_t K)
{
    return fused_prefill_codes_bytes(M, K) + (size_t)((4 * M + 15) / 16 * 16);
}

// With the matrix-core plane in the packed buffer, a prefill call's workspace starts with the
// activation planes (a multiple of 256 bytes); the fused call's codes and scales follow.
size_t planes_ws_bytes(const Layout& L, int64_t M) { return prefill6_possible(L, M) ? prefill6_ws_bytes(M, L.Kx) : 0; }

// Above this many bytes of packed weights quantizing the row once, in a kernel of its own (about
// 4 us), beats quantizing it in every workgroup (measured: 75 MiB 16.4 us fused against 4.2 + 14.6 us,
// 300 MiB 58 us against 4.2 + 45.7 us).
constexpr size_t kFusedTwoKernelBytes = (size_t)96 << 20;

bool prefill_fits(int64_t M, int64_t N, int64_t K, int mode = MNNQ_W4_ZP_INT, int act_bytes = 1)
{
    const int64_t lim = ((int64_t)1 << 31) - 1;
    // 32-bit byte offsets: activation rows of a whole tile, the packed weights, the output.
    return M <= ((int64_t)1 << 24) && (M + 256) * K * act_bytes <= lim &&
           (int64_t)make_layout(N, K, mode).total() <= lim && (M + 256) * N * 4 <= lim;
}

// Batches beyond what prefill_fits allows are processed in slabs of this many rows (a multiple of
// 256, so every slab starts on a 16-byte boundary of x and y), one launch each; 0 if even the packed
// matrix or a single slab is out of reach of the 32-bit offsets.
int64_t prefill_slab_rows(int64_t N, int64_t K, int mode, int act_bytes = 1)
{
    const int64_t lim = ((int64_t)1 << 31) - 1;
    if ((int64_t)make_layout(N, K, mode).total() > lim) return 0;
    int64_t rows = lim / (K * act_bytes) < lim / (N * 4) ? lim / (K * act_bytes) : lim / (N * 4);
    rows = (rows - 256) / 256 * 256;
    if (rows > ((int64_t)1 << 24)) rows = (int64_t)1 << 24;
    return rows >= 256 ? rows : 0;
}

Layout layout_for(int64_t N, int64_t K, int mode, bool out16)
{
    Layout L = make_layout(N, K, mode);
    L.out16 = out16;
    return L;
}

// The four linear calls that exist with fp32 and with binary16 output; y points to the output array
// of the requested kind (the kernels store through it according to Layout::out16).
int decode_impl(const void* packed, int64_t N, int64_t K, int group, int mode, const int8_t* xq, const float* sx,
                const float* bias, void* y, bool out16, void* stream)
{
    if (!packed || !xq || !sx || !y) return MNNQ_ERR_NULL;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (make_layout(N, K, mode).K > kMaxDecodeK) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(xq) || misaligned(y) || misaligned(bias)) return MNNQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(sx) & 3u) return MNNQ_ERR_ALIGN;
    return launch_decode(static_cast<const uint8_t*>(packed), layout_for(N, K, mode, out16), xq, sx, bias,
                         static_cast<float*>(y), static_cast<hipStream_t>(stream));
}

int prefill_impl(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode, const int8_t* xq,
                 const float* sx, const float* bias, void* y, bool out16, void* workspace, size_t workspace_bytes,
                 void* stream)
{
    if (!packed || !xq || !sx || !y) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    const int64_t slab = prefill_fits(M, N, K, mode) ? M : prefill_slab_rows(N, K, mode);
    if (slab <= 0) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(xq) || misaligned(y) || misaligned(bias) || misaligned(workspace))
        return MNNQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(sx) & 3u) return MNNQ_ERR_ALIGN;
    const Layout L = layout_for(N, K, mode, out16);
    if (slab < M) {   // a batch too large for one launch: slab by slab
        for (int64_t m0 = 0; m0 < M; m0 += slab) {
            const int64_t rows = M - m0 < slab ? M - m0 : slab;
            void* ys = static_cast<uint8_t*>(y) + (size_t)m0 * N * (out16 ? 2 : 4);
            if (int s = prefill_impl(packed, rows, N, K, group, mode, xq + m0 * K, sx + m0, bias, ys, out16, workspace,
                                     workspace_bytes, stream))
                return s;
        }
        return MNNQ_OK;
    }
    // A few tokens (batched or speculative decoding) are still memory-bound: one pass over the
    // weights in the GEMV's streaming order, all tokens at once in the matrix cores.
    // With the matrix-core plane and room for the activations' planes: the GEMM on the fp6 matrix instructions.
    if (prefill6_wanted(L, M) && workspace && workspace_bytes >= prefill6_ws_bytes(M, K)) {
        if (int s = launch_act_planes(xq, M, K, workspace, static_cast<hipStream_t>(stream))) return s;
        return launch_prefill6(static_cast<const uint8_t*>(packed), L, M, workspace, sx, bias, static_cast<float*>(y),
                               nullptr, static_cast<hipStream_t>(stream));
    }
    if (M <= 16 && !debug_option(kDbgNoSkinny) && !L.native8)   // (the byte form: a few tokens through the tiled GEMM)
        return launch_skinny(static_cast<const uint8_t*>(packed), L, M, xq, sx, bias, static_cast<float*>(y),
                             static_cast<hipStream_t>(stream));
    return launch_prefill(static_cast<const uint8_t*>(packed), L, M, xq, sx, bias, static_cast<float*>(y), nullptr,
                          static_cast<hipStream_t>(stream));
}

int decode_f16_impl(const void* packed, int64_t N, int64_t K, int group, int mode, const uint16_t* x16,
                    const float* bias, void* y, bool out16, void* stream)
{
    if (!packed || !x16 || !y) return MNNQ_ERR_NULL;
    if (int s = check_shape(N, K, group, mode)) return s;
    const Layout L = layout_for(N, K, mode, out16);   // the packed reduction axis is what is staged
    if (L.native8) return MNNQ_ERR_UNSUPPORTED;      // the fp16-activation kernels read the plane form
    if (L.K > (L.minf ? kMaxDecodeKF16Min : kMaxDecodeKF16)) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(x16) || misaligned(y) || misaligned(bias)) return MNNQ_ERR_ALIGN;
    return launch_decode_f16(static_cast<const uint8_t*>(packed), L, x16, bias, static_cast<float*>(y),
                             static_cast<hipStream_t>(stream));
}

int prefill_f16_impl(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode, const uint16_t* x16,
                     const float* row_scale, const float* bias, void* y, bool out16, void* stream)
{
    if (!packed || !x16 || !y) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (mode & MNNQ_NATIVE_8BIT) return MNNQ_ERR_UNSUPPORTED;   // the fp16-activation kernels read the plane form
    const int64_t slab = prefill_fits(M, N, K, mode, 2) ? M : prefill_slab_rows(N, K, mode, 2);   // byte offsets of fp16 rows
    if (slab <= 0) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(x16) || misaligned(y) || misaligned(bias)) return MNNQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(row_scale) & 3u) return MNNQ_ERR_ALIGN;
    if (slab < M) {
        for (int64_t m0 = 0; m0 < M; m0 += slab) {
            const int64_t rows = M - m0 < slab ? M - m0 : slab;
            void* ys = static_cast<uint8_t*>(y) + (size_t)m0 * N * (out16 ? 2 : 4);
            if (int s = prefill_f16_impl(packed, rows, N, K, group, mode, x16 + m0 * K, row_scale ? row_scale + m0 : nullptr,
                                         bias, ys, out16, stream))
                return s;
        }
        return MNNQ_OK;
    }
    return launch_prefill_f16(static_cast<const uint8_t*>(packed), layout_for(N, K, mode, out16), M, x16, row_scale,
                              bias, static_cast<float*>(y), static_cast<hipStream_t>(stream));
}

// The fused calls: activation quantizer and linear layer in one call.
int decode_fused_impl(const void* packed, int64_t N, int64_t K, int group, int mode, const float* x,
                      const float* bias, void* y, bool out16, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!packed || !x || !y) return MNNQ_ERR_NULL;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (make_layout(N, K, mode).K > kMaxDecodeK) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(x) || misaligned(y) || misaligned(bias) || misaligned(workspace))
        return MNNQ_ERR_ALIGN;
    const Layout L = layout_for(N, K, mode, out16);
    hipStream_t st = static_cast<hipStream_t>(stream);
    size_t two_kernel_bytes = kFusedTwoKernelBytes;
    if (const char* e = debug_option(kDbgFusedTwoKernelMib)) two_kernel_bytes = (size_t)atoll(e) << 20;   // tuning only
    if (workspace && workspace_bytes >= fused_ws_bytes(K) && L.total() > two_kernel_bytes) {
        int8_t* xq = static_cast<int8_t*>(workspace);
        float* sx = reinterpret_cast<float*>(xq + (K + 127) / 128 * 128);
        if (int s = launch_quant_act(x, 1, K, xq, sx, nullptr, st)) return s;
        return launch_decode(static_cast<const uint8_t*>(packed), L, xq, sx, bias, static_cast<float*>(y), st);
    }
    return launch_decode_fused(static_cast<const uint8_t*>(packed), L, x, bias, static_cast<float*>(y), st);
}

int prefill_fused_impl(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode, const float* x,
                       const float* bias, void* y, bool out16, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    if (!packed || !x || !y || !workspace) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (!prefill_fits(M, N, K, mode) && prefill_slab_rows(N, K, mode) <= 0) return MNNQ_ERR_UNSUPPORTED;
    if (workspace_bytes < fused_prefill_ws_bytes(M, K)) return MNNQ_ERR_SIZE;
    if (misaligned(packed) || misaligned(x) || misaligned(workspace) || misaligned(y) || misaligned(bias))
        return MNNQ_ERR_ALIGN;
    // The activation planes of the fp6 GEMM lie in front when they fit as well (else: the int8 GEMM).
    size_t planes = planes_ws_bytes(make_layout(N, K, mode), M);
    if (workspace_bytes < planes + fused_prefill_ws_bytes(M, K)) planes = 0;
    int8_t* xq = static_cast<int8_t*>(workspace) + planes;
    float* sx = reinterpret_cast<float*>(xq + fused_prefill_codes_bytes(M, K));
    if (int s = launch_quant_act(x, M, K, xq, sx, nullptr, static_cast<hipStream_t>(stream))) return s;
    return prefill_impl(packed, M, N, K, group, mode, xq, sx, bias, y, out16, planes ? workspace : nullptr, planes, stream);
}

// Scratch of mnnq_linear_prefill_fused_static: the int8 codes [M, K] and the scales [M] pass through
// this array instead of a caller's workspace.  Every device the library runs on holds its own copy
// at its own address; in host code the array's name is only a handle for hipGetSymbolAddress.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch`, per device; NULL until first asked for
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up once per device).
int static_scratch(uint8_t** out)
{
    int dev = 0;
    MNNQ_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MNNQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        MNNQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return MNNQ_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<uint8_t*>(g_scratch_ptr[dev]);
    return MNNQ_OK;
}

}  // namespace
}  // namespace mnnq

using namespace mnnq;

extern "C" {

const char* mnnq_status_string(int status)
{
    switch (status) {
        case MNNQ_OK: return "ok";
        case MNNQ_ERR_NULL: return "null pointer";
        case MNNQ_ERR_SHAPE: return "bad shape";
        case MNNQ_ERR_UNSUPPORTED: return "unsupported group, mode or size";
        case MNNQ_ERR_SIZE: return "buffer too small";
        case MNNQ_ERR_ALIGN: return "pointer not 16-byte aligned";
        case MNNQ_ERR_HIP: return "HIP call failed";
        default: return "unknown status";
    }
}

int mnnq_last_hip_error(void) { return t_last_hip_error; }

int mnnq_version(void) { return 100; }

size_t mnnq_packed_size(int64_t N, int64_t K, int group, int mode)
{
    if (check_shape(N, K, group, mode) != MNNQ_OK) return 0;
    return make_layout(N, K, mode).full_total();
}

size_t mnnq_workspace_size(int64_t M, int64_t N, int64_t K, int group, int mode)
{
    if (check_shape(N, K, group, mode) != MNNQ_OK) return 0;
    // Split rows are combined inside a workgroup (decode) or directly in y (prefill): nothing
    // needs scratch.  The fused decode call can use room for the quantized row and its scale.
    if (M == 1) return fused_ws_bytes(K);
    return M > 1 ? planes_ws_bytes(make_layout(N, K, mode), M) + fused_prefill_ws_bytes(M, K) : 0;
}

int mnnq_pack_weights(const float* W, int64_t N, int64_t K, int group, int mode, void* packed,
                      size_t packed_bytes, void* stream)
{
    if (!W || !packed) return MNNQ_ERR_NULL;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (misaligned(W) || misaligned(packed)) return MNNQ_ERR_ALIGN;
    const Layout L = make_layout(N, K, mode);
    if (packed_bytes < L.full_total()) return MNNQ_ERR_SIZE;
    if (int s = launch_pack(W, L, static_cast<uint8_t*>(packed), static_cast<hipStream_t>(stream))) return s;
    return L.plane ? launch_plane_build(static_cast<uint8_t*>(packed), L, static_cast<hipStream_t>(stream)) : MNNQ_OK;
}

int mnnq_pack_from_quantized(const uint8_t* q, const float* scale, const void* zero, int64_t N, int64_t K,
                             int group, int mode, void* packed, size_t packed_bytes, void* stream)
{
    if (!q || !scale || !zero || !packed) return MNNQ_ERR_NULL;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (misaligned(q) || misaligned(packed)) return MNNQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(scale) & 3u) return MNNQ_ERR_ALIGN;
    if ((mode & kModeMask) != MNNQ_W4_ZP_INT && (reinterpret_cast<uintptr_t>(zero) & 3u)) return MNNQ_ERR_ALIGN;
    const Layout L = make_layout(N, K, mode);
    if (packed_bytes < L.full_total()) return MNNQ_ERR_SIZE;
    if (int s = launch_repack(q, scale, zero, L, static_cast<uint8_t*>(packed), static_cast<hipStream_t>(stream))) return s;
    return L.plane ? launch_plane_build(static_cast<uint8_t*>(packed), L, static_cast<hipStream_t>(stream)) : MNNQ_OK;
}

int mnnq_unpack_weights(const void* packed, int64_t N, int64_t K, int group, int mode, uint8_t* q,
                        float* scale, void* zero, void* stream)
{
    if (!packed) return MNNQ_ERR_NULL;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (misaligned(packed) || misaligned(q) || misaligned(scale) || misaligned(zero)) return MNNQ_ERR_ALIGN;
    if (!q && !scale && !zero) return MNNQ_OK;
    return launch_unpack(static_cast<const uint8_t*>(packed), make_layout(N, K, mode), q, scale, zero,
                         static_cast<hipStream_t>(stream));
}

int mnnq_quant_act(const float* x, int64_t M, int64_t K, int group, int8_t* xq, float* sx, int32_t* xsum,
                   void* stream)
{
    if (!x || !xq || !sx) return MNNQ_ERR_NULL;
    if (M <= 0 || K <= 0) return MNNQ_ERR_SHAPE;
    if (group != kGroup) return MNNQ_ERR_UNSUPPORTED;
    if (K % group != 0) return MNNQ_ERR_SHAPE;
    if (M > ((int64_t)1 << 31) - 1) return MNNQ_ERR_UNSUPPORTED;
    // sx and xsum are arrays of 4-byte items; only the vector-accessed buffers need 16 bytes.
    if (misaligned(x) || misaligned(xq)) return MNNQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(sx) & 3u) || (reinterpret_cast<uintptr_t>(xsum) & 3u)) return MNNQ_ERR_ALIGN;
    return launch_quant_act(x, M, K, xq, sx, xsum, static_cast<hipStream_t>(stream));
}

int mnnq_linear_decode(const void* packed, int64_t N, int64_t K, int group, int mode, const int8_t* xq,
                       const float* sx, const float* bias, float* y, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    (void)workspace; (void)workspace_bytes;
    return decode_impl(packed, N, K, group, mode, xq, sx, bias, y, false, stream);
}

int mnnq_linear_decode_fused(const void* packed, int64_t N, int64_t K, int group, int mode, const float* x,
                             const float* bias, float* y, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_fused_impl(packed, N, K, group, mode, x, bias, y, false, workspace, workspace_bytes, stream);
}

int mnnq_linear_decode_fused_o16(const void* packed, int64_t N, int64_t K, int group, int mode, const float* x,
                                 const float* bias, uint16_t* y16, void* workspace, size_t workspace_bytes,
                                 void* stream)
{
    return decode_fused_impl(packed, N, K, group, mode, x, bias, y16, true, workspace, workspace_bytes, stream);
}

int mnnq_linear_prefill(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                        const int8_t* xq, const float* sx, const float* bias, float* y, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return prefill_impl(packed, M, N, K, group, mode, xq, sx, bias, y, false, workspace, workspace_bytes, stream);
}

int mnnq_linear_prefill_fused(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                              const float* x, const float* bias, float* y, void* workspace, size_t workspace_bytes,
                              void* stream)
{
    return prefill_fused_impl(packed, M, N, K, group, mode, x, bias, y, false, workspace, workspace_bytes, stream);
}

int mnnq_linear_prefill_fused_static(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                     const float* x, const float* bias, float* y, void* stream)
{
    if (!packed || !x || !y) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (fused_prefill_ws_bytes(M, K) > kStaticScratchBytes) return MNNQ_ERR_SIZE;
    uint8_t* ws = nullptr;
    // (every other check is made by the call this one forwards to, before anything is launched)
    if (misaligned(packed) || misaligned(x) || misaligned(y) || misaligned(bias)) return MNNQ_ERR_ALIGN;
    if (!prefill_fits(M, N, K, mode) && prefill_slab_rows(N, K, mode) <= 0) return MNNQ_ERR_UNSUPPORTED;
    if (int s = static_scratch(&ws)) return s;
    // (with the matrix-core plane, the fp6 GEMM runs when the activations' planes fit in the array too)
    return prefill_fused_impl(packed, M, N, K, group, mode, x, bias, y, false, ws, kStaticScratchBytes, stream);
}

size_t mnnq_static_scratch_bytes(void) { return kStaticScratchBytes; }

int mnnq_linear_prefill_fused_o16(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                  const float* x, const float* bias, uint16_t* y16, void* workspace,
                                  size_t workspace_bytes, void* stream)
{
    return prefill_fused_impl(packed, M, N, K, group, mode, x, bias, y16, true, workspace, workspace_bytes, stream);
}

int mnnq_linear_decode_f16(const void* packed, int64_t N, int64_t K, int group, int mode, const uint16_t* x16,
                           const float* bias, float* y, void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    return decode_f16_impl(packed, N, K, group, mode, x16, bias, y, false, stream);
}

int mnnq_linear_prefill_f16(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                            const uint16_t* x16, const float* row_scale, const float* bias, float* y,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    return prefill_f16_impl(packed, M, N, K, group, mode, x16, row_scale, bias, y, false, stream);
}

int mnnq_linear_decode_o16(const void* packed, int64_t N, int64_t K, int group, int mode, const int8_t* xq,
                           const float* sx, const float* bias, uint16_t* y16, void* stream)
{
    return decode_impl(packed, N, K, group, mode, xq, sx, bias, y16, true, stream);
}

int mnnq_linear_prefill_o16(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                            const int8_t* xq, const float* sx, const float* bias, uint16_t* y16, void* stream)
{
    return prefill_impl(packed, M, N, K, group, mode, xq, sx, bias, y16, true, nullptr, 0, stream);
}

int mnnq_linear_decode_f16_o16(const void* packed, int64_t N, int64_t K, int group, int mode, const uint16_t* x16,
                               const float* bias, uint16_t* y16, void* stream)
{
    return decode_f16_impl(packed, N, K, group, mode, x16, bias, y16, true, stream);
}

int mnnq_linear_prefill_f16_o16(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                const uint16_t* x16, const float* row_scale, const float* bias, uint16_t* y16,
                                void* stream)
{
    return prefill_f16_impl(packed, M, N, K, group, mode, x16, row_scale, bias, y16, true, stream);
}

int mnnq_plan_debug(int what, int64_t M, int64_t N, int64_t K, int group, int mode, int32_t* out8)
{
    if (!out8) return MNNQ_ERR_NULL;
    if (what < 0 || what > 2) return MNNQ_ERR_UNSUPPORTED;
    if (what == 0 && M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    const Layout L = make_layout(N, K, mode);
    if (what == 0) {
        const int64_t slab = prefill_fits(M, N, K, mode) ? M : prefill_slab_rows(N, K, mode);
        if (slab <= 0) return MNNQ_ERR_UNSUPPORTED;
        const int64_t rows = slab < M ? slab : M;         // (of the first slab, for batches beyond one launch)
        if (prefill6_wanted(L, rows)) describe_prefill6(L, rows, out8);   // (when the call is given its workspace)
        else describe_prefill(L, rows, out8);
    } else {
        if (L.K > kMaxDecodeK) return MNNQ_ERR_UNSUPPORTED;
        describe_decode(L, what == 2, out8);
    }
    return MNNQ_OK;
}

int mnnq_linear_acc_debug_planes(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                 const int8_t* xq, int32_t* acc, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!packed || !xq || !acc || !workspace) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    const Layout L = make_layout(N, K, mode);
    if (M > kMaxM || !prefill_fits(M, N, K, mode) || !prefill6_possible(L, M)) return MNNQ_ERR_UNSUPPORTED;
    if (workspace_bytes < prefill6_ws_bytes(M, K)) return MNNQ_ERR_SIZE;
    if (misaligned(packed) || misaligned(xq) || misaligned(acc) || misaligned(workspace)) return MNNQ_ERR_ALIGN;
    if (int s = launch_act_planes(xq, M, K, workspace, static_cast<hipStream_t>(stream))) return s;
    return launch_prefill6(static_cast<const uint8_t*>(packed), L, M, workspace, nullptr, nullptr, nullptr, acc,
                           static_cast<hipStream_t>(stream));
}

size_t mnnq_act_planes_size(int64_t M, int64_t K, int group)
{
    if (M <= 0 || K <= 0 || group != kGroup || K % group != 0) return 0;
    return prefill6_ws_bytes(M, K);
}

int mnnq_act_planes(const int8_t* xq, int64_t M, int64_t K, int group, void* planes, size_t planes_bytes, void* stream)
{
    if (!xq || !planes) return MNNQ_ERR_NULL;
    if (M <= 0 || K <= 0) return MNNQ_ERR_SHAPE;
    if (group != kGroup) return MNNQ_ERR_UNSUPPORTED;
    if (K % group != 0) return MNNQ_ERR_SHAPE;
    if (M > ((int64_t)1 << 24) || (int64_t)prefill6_ws_bytes(M, K) > ((int64_t)1 << 31) - 1) return MNNQ_ERR_UNSUPPORTED;
    if (planes_bytes < prefill6_ws_bytes(M, K)) return MNNQ_ERR_SIZE;
    if (misaligned(xq) || misaligned(planes)) return MNNQ_ERR_ALIGN;
    return launch_act_planes(xq, M, K, planes, static_cast<hipStream_t>(stream));
}

int mnnq_linear_prefill_planes(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                               const void* planes, const float* sx, const float* bias, float* y, void* stream)
{
    if (!packed || !planes || !sx || !y) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    const Layout L = make_layout(N, K, mode);
    if (!prefill_fits(M, N, K, mode) || !prefill6_possible(L, M)) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(planes) || misaligned(y) || misaligned(bias)) return MNNQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(sx) & 3u) return MNNQ_ERR_ALIGN;
    return launch_prefill6(static_cast<const uint8_t*>(packed), L, M, planes, sx, bias, y, nullptr,
                           static_cast<hipStream_t>(stream));
}

int mnnq_debug_set(const char* key, const char* value)
{
    if (!key) return MNNQ_ERR_NULL;
    for (int i = 0; i < kDbgCount; ++i) {
        if (strcmp(key, g_debug[i].name) != 0) continue;
        if (value && strlen(value) >= sizeof(g_debug[i].value)) return MNNQ_ERR_SIZE;
        g_debug[i].set = value != nullptr;
        if (value) strcpy(g_debug[i].value, value);
        return MNNQ_OK;
    }
    return MNNQ_ERR_UNSUPPORTED;
}

int mnnq_linear_acc_debug(const void* packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                          const int8_t* xq, int32_t* acc, int use_prefill_kernel, void* stream)
{
    if (!packed || !xq || !acc) return MNNQ_ERR_NULL;
    if (M <= 0) return MNNQ_ERR_SHAPE;
    if (int s = check_shape(N, K, group, mode)) return s;
    if (M > kMaxM || (mode & MNNQ_NATIVE_8BIT)) return MNNQ_ERR_UNSUPPORTED;   // (no dump in the byte form)
    if (!use_prefill_kernel && make_layout(N, K, mode).K > kMaxDecodeK) return MNNQ_ERR_UNSUPPORTED;
    if (use_prefill_kernel && !prefill_fits(M, N, K, mode)) return MNNQ_ERR_UNSUPPORTED;
    if (misaligned(packed) || misaligned(xq) || misaligned(acc)) return MNNQ_ERR_ALIGN;
    const Layout L = make_layout(N, K, mode);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (use_prefill_kernel)
        return launch_prefill(static_cast<const uint8_t*>(packed), L, M, xq, nullptr, nullptr, nullptr, acc, st);
    return launch_decode_acc(static_cast<const uint8_t*>(packed), L, M, xq, acc, st);
}

}  // extern "C"
