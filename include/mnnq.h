/*
 * mnnq - W4A8 / W4A16 quantized linear layer for AMD MI355X (gfx950).
 *
 * C-ABI boundary of the library.  The operation is the quantized Linear layer
 * of the MNN-LLM paper (arXiv 2506.10443): weights [h, l] are quantized once,
 * at load time, to asymmetric int4 (Section 4.2, Eq. 1); activations [e, l]
 * arrive at run time and are quantized to int8 (Section 4.2); the result is
 * [e, h] (Section 5.1).  Below: M = e (tokens), K = l (reduction), N = h
 * (output features), G = K / 64 quantization groups along K.
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer, 16-byte aligned, owned by the caller.
 *     The library never allocates, frees or synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; buffers must stay valid until the stream has
 *     passed that work.
 *   - Stream capture: the calls enqueue kernels only (no memset or copy nodes) and can be recorded
 *     into a HIP graph.  The first call of a kernel variant on a device may also set a function
 *     attribute (more than 64 KiB of LDS), so run a call once outside the capture before recording it.
 *   - Return value: MNNQ_OK (0) or a negative mnnq_status.  All argument
 *     checks run before the first HIP call, so they also work on a machine
 *     without a GPU.  NaN / Inf in W or x: undefined result, no error.
 *   - Limits (MNNQ_ERR_UNSUPPORTED beyond them): N and K up to 2^24.  Decode calls: K up to
 *     126976 (with fp16 activations 79872, or 71680 in the float-minimum modes; for int8
 *     weights half of these), the row is staged in LDS.  Prefill calls address with 32-bit byte offsets: the packed matrix
 *     must stay below 2 GiB; batches for which (M + 256) * K (twice that with fp16 activations) or
 *     (M + 256) * N * 4 reaches 2 GiB are processed in slabs of rows, one launch per slab.
 *     mnnq_linear_acc_debug: M up to 65535 and within one such slab.
 *   - Only group == 64 is implemented.  K must be a multiple of 64 and N a
 *     multiple of 16.  `mode` selects the weight quantizer (mnnq_mode); a packed
 *     buffer must be used with the mode it was written with.
 */
#ifndef MNNQ_H
#define MNNQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MNNQ_OK = 0,
    MNNQ_ERR_NULL = -1,        /* a required pointer is NULL */
    MNNQ_ERR_SHAPE = -2,       /* M, N or K <= 0, or K not a multiple of the group */
    MNNQ_ERR_UNSUPPORTED = -3, /* group != 64, unknown mode, N not a multiple of 16, or a size limit (see Limits) */
    MNNQ_ERR_SIZE = -4,        /* packed / workspace buffer too small */
    MNNQ_ERR_ALIGN = -5,       /* a pointer is not 16-byte aligned */
    MNNQ_ERR_HIP = -6          /* a HIP call failed; see mnnq_last_hip_error() */
} mnnq_status;

typedef enum {
    /* int4 codes 0..15, fp32 scale and integer zero point per (row, group):
     * scale = (max - min) / 15, zero = round(-min / scale),
     * q = clamp(round(w / scale) + zero, 0, 15), w^ = (q - zero) * scale.
     * This is Eq. 1 of Section 4.2 with the offset rounded to the code grid. */
    MNNQ_W4_ZP_INT = 0,
    /* Eq. 1 of Section 4.2 exactly as printed: the group minimum stays a float
     * offset.  step = (max - min) / 15, q = clamp(round((w - min) / step), 0, 15),
     * w^ = q * step + min (a constant group: step 1, codes 0).  Stored per
     * (row, group): fp32 step and fp32 min (3 bytes more than a zero point).
     *   y[m,n] = sx[m] * sum_g (step[n,g] * A[m,n,g] + min[n,g] * xs[m,g]) (+ bias[n]),
     *   A = sum_{k in g} xq[m,k] * q[n,k],  xs[m,g] = sum_{k in g} xq[m,k].
     * Supported by the pack / unpack / import calls and the W4A8 linear calls;
     * the fp16-activation calls return MNNQ_ERR_UNSUPPORTED for it. */
    MNNQ_W4_MIN_FLOAT = 1,
    /* int8 weights (Section 4.2: parameters are quantized to int4 or int8, the LM
     * head preferably to int8): Eq. 1 with clip range 0..255 and a float minimum,
     * step = (max - min) / 255, q = clamp(round((w - min) / step), 0, 255),
     * w^ = q * step + min.  Needs K to be a multiple of 128.  The packed form holds
     * a code as two 4-bit planes and runs on the int4 kernels (1.25 bytes per
     * weight).  Supported by the same calls as MNNQ_W4_MIN_FLOAT; q of the
     * unpack / import calls holds the 8-bit codes; mnnq_linear_acc_debug returns
     * 2 K/64 sums per (m, n): first the high-nibble planes, then the low ones. */
    MNNQ_W8_MIN_FLOAT = 2,
    /* Flag, to be OR-ed to MNNQ_W4_ZP_INT in every call that takes a mode: the packed buffer also
     * holds the weights a second time, rearranged at load (Section 5.1) for the fp6 matrix
     * instructions of gfx950 (the "matrix-core plane": 0.81 bytes per weight more).  The prefill calls
     * then run on those instructions when they are also given a workspace for the activations'
     * counterpart (mnnq_workspace_size); every other call reads the chunk layout in front as before.
     * Results are those of the unflagged mode: the plane holds the same integers q - zero. */
    MNNQ_WITH_MATRIX_PLANE = 16,
    /* Flag, to be OR-ed to MNNQ_W8_MIN_FLOAT in every call that takes a mode: the 8-bit codes are stored
     * as bytes (q - 128, the operand of the int8 dot and matrix instructions as it stands; 1.125 bytes
     * per weight: Section 5.1's rearrangement for the instruction that consumes the data) instead of two
     * 4-bit planes.  Same quantizer, same results up to the order of the fp32 sums.  Supported by the
     * pack / unpack / import calls and the W8A8 linear calls (decode, prefill, their fused and binary16
     * forms; a few tokens at once run through the tiled GEMM); the fp16-activation calls and the
     * accumulator dumps return MNNQ_ERR_UNSUPPORTED for it - they read the plane form. */
    MNNQ_NATIVE_8BIT = 32
} mnnq_mode;

/* Text for a status code (static storage). */
const char *mnnq_status_string(int status);

/* Raw hipError_t of the last MNNQ_ERR_HIP returned on the calling thread. */
int mnnq_last_hip_error(void);

/* Library version, major * 10000 + minor * 100 + patch. */
int mnnq_version(void);

/* Bytes of the packed form of an [N, K] weight matrix; 0 if the arguments are
 * not supported.  For K a multiple of 128 this is exactly N*K/2 + 5*N*K/64
 * (codes + fp32 scale + one-byte zero point); for K = 64 * odd, one padding
 * group per row tile is added. */
size_t mnnq_packed_size(int64_t N, int64_t K, int group, int mode);

/* Bytes of device scratch the linear calls can make use of for these shapes.
 * No call needs a workspace: NULL / 0 is always accepted.  For M = 1 the value
 * is what mnnq_linear_decode_fused uses, when given, to hold the int8 row and
 * its scale (K rounded up to 128, plus 16): for layers above 96 MiB of packed
 * weights it then runs the quantizer as a kernel of its own in front of the
 * GEMV, which is faster there than quantizing inside every workgroup.  The
 * result does not depend on the route.  For M > 1 the value is what
 * mnnq_linear_prefill_fused requires: room for the int8 codes [M, K] and the scales [M]. */
size_t mnnq_workspace_size(int64_t M, int64_t N, int64_t K, int group, int mode);

/* Load-time step (Section 4.2 Eq. 1, Section 5.1 "rearranged at model loading
 * phase"): quantize W and store it in the layout the decode and prefill kernels
 * read.  W: device fp32 [N, K] row-major.  packed: device buffer of at least
 * mnnq_packed_size() bytes, opaque; position independent, may be copied. */
int mnnq_pack_weights(const float *W, int64_t N, int64_t K, int group, int mode,
                      void *packed, size_t packed_bytes, void *stream);

/* Canonical view of a packed matrix (for tests and export): q [N, K] one code
 * per byte, scale [N, G] fp32, zero [N, G]: uint8 zero points in mode
 * MNNQ_W4_ZP_INT, fp32 group minima in mode MNNQ_W4_MIN_FLOAT.  Any output may
 * be NULL. */
int mnnq_unpack_weights(const void *packed, int64_t N, int64_t K, int group, int mode,
                        uint8_t *q, float *scale, void *zero, void *stream);

/* Run-time activation quantizer (Section 4.2: activations are quantized to
 * int8 during calculation), per token, symmetric: sx[m] = max_k |x[m,k]| / 127,
 * xq = clamp(round(x / sx), -127, 127); a zero row gives sx = 0, xq = 0.
 * x: fp32 [M, K]; xq: int8 [M, K]; sx: fp32 [M]; xsum: int32 [M, G] sums of xq
 * per group, or NULL. */
int mnnq_quant_act(const float *x, int64_t M, int64_t K, int group,
                   int8_t *xq, float *sx, int32_t *xsum, void *stream);

/* Decode step, one token (Section 2.1: memory-bound phase):
 *   y[n] = sx * sum_g scale[n,g] * sum_{k in g} xq[k] * (q[n,k] - zero[n,g]) (+ bias[n]).
 * xq: int8 [K]; sx: fp32 [1]; bias: fp32 [N] or NULL; y: fp32 [N]. */
int mnnq_linear_decode(const void *packed, int64_t N, int64_t K, int group, int mode,
                       const int8_t *xq, const float *sx, const float *bias, float *y,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Decode step with the activation quantizer fused in: takes the fp32 activation
 * row x [K] and quantizes it inside the kernel exactly as mnnq_quant_act does
 * (Section 4.2: activations are quantized to int8 during calculation), then
 * computes the same y as mnnq_linear_decode.  Saves one launch and the round
 * trip of xq through memory on the latency-critical decode path.
 * workspace: optional, see mnnq_workspace_size; 16-byte aligned; its contents
 * are scratch and calls sharing one workspace must not overlap in time. */
int mnnq_linear_decode_fused(const void *packed, int64_t N, int64_t K, int group, int mode,
                             const float *x, const float *bias, float *y,
                             void *workspace, size_t workspace_bytes, void *stream);

/* Prefill, M tokens (Section 2.1: compute-bound phase): the same formula for
 * every row m with its own sx[m].  xq: int8 [M, K]; sx: fp32 [M];
 * y: fp32 [M, N] row-major. */
int mnnq_linear_prefill(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                        const int8_t *xq, const float *sx, const float *bias, float *y,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Same as mnnq_quant_act followed by mnnq_linear_prefill (Section 4.2: the activations are
 * quantized to int8 during calculation): x fp32 [M, K] in, y fp32 [M, N] out, bit for bit the
 * result of the two calls.  The codes and scales pass through `workspace`, which this call
 * requires: at least mnnq_workspace_size(M, N, K, group, mode) bytes, 16-byte aligned, scratch
 * (MNNQ_ERR_NULL without it, MNNQ_ERR_SIZE if too small); calls sharing one workspace must not
 * overlap in time.  M = 1 is accepted too (the value mnnq_workspace_size gives for M = 1 is
 * large enough), though mnnq_linear_decode_fused is the call made for single tokens. */
int mnnq_linear_prefill_fused(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                              const float *x, const float *bias, float *y,
                              void *workspace, size_t workspace_bytes, void *stream);

/* The two steps of mnnq_linear_prefill on a packed buffer with the matrix-core plane, as calls of their
 * own - for callers that feed several projections with the same activations (q, k, v; gate, up) and
 * want the activations rearranged once (Section 5.1 rearranges operands for the instruction that
 * consumes them; for activations that has to happen per call):
 *   mnnq_act_planes: int8 codes xq [M, K] -> the activation operand of the fp6 matrix instructions
 *     (every code as sign * (16 hi + lo), both parts exact e2m3 numbers), mnnq_act_planes_size(M, K, group) bytes;
 *   mnnq_linear_prefill_planes: y [M, N] from those planes, the scales sx [M] and the packed weights;
 *     mode must carry MNNQ_WITH_MATRIX_PLANE and M must exceed 32 (MNNQ_ERR_UNSUPPORTED otherwise).
 * The result is that of mnnq_linear_prefill with a workspace, bit for bit, whenever that call takes
 * the fp6 GEMM as well (it leaves shapes with very few output tiles and a long K to the int8 GEMM;
 * mnnq_plan_debug tells). */
size_t mnnq_act_planes_size(int64_t M, int64_t K, int group);
int mnnq_act_planes(const int8_t *xq, int64_t M, int64_t K, int group, void *planes, size_t planes_bytes,
                    void *stream);
int mnnq_linear_prefill_planes(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                               const void *planes, const float *sx, const float *bias, float *y, void *stream);

/* mnnq_linear_prefill_fused for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the int8
 * codes and scales pass through an array inside the library instead, of
 * mnnq_static_scratch_bytes() = 32 MiB per device, which every device the library runs on holds
 * until the process ends.  The call allocates and frees nothing.  Same arguments, checks and result
 * (bit for bit) as mnnq_linear_prefill_fused without the workspace; additionally MNNQ_ERR_SIZE when
 * M * K rounded up to 16, plus 4 * M rounded up to 16, exceeds mnnq_static_scratch_bytes().
 * All calls on one device share that device's array: calls that overlap in time on one device
 * (different streams or threads) race and give undefined results; calls ordered on one stream are
 * safe.  Nothing in the array has to survive between calls. */
int mnnq_linear_prefill_fused_static(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                     const float *x, const float *bias, float *y, void *stream);
size_t mnnq_static_scratch_bytes(void);

/* fp16-activation variants (Section 4.2: quantized weights with fp16 activations on GPUs;
 * W4A16, and W8A16 with mode MNNQ_W8_MIN_FLOAT):
 *   y[m,n] = sum_k float(x16[m,k]) * w^[n,k] (+ bias[n]),  w^ the weight the stored code
 * stands for in the packed buffer's mode ((q - zero) * scale, or q * step + min),
 * fp32 accumulation.  x16: IEEE binary16 bits, [K] resp. [M, K]. */
int mnnq_linear_decode_f16(const void *packed, int64_t N, int64_t K, int group, int mode,
                           const uint16_t *x16, const float *bias, float *y,
                           void *workspace, size_t workspace_bytes, void *stream);
/* row_scale: fp32 [M] or NULL; when given, row m of the sums is multiplied by
 * row_scale[m] before the bias is added.  With x16 holding the int8 activation
 * codes as fp16 (exact) and row_scale = sx this is the W4A8 result of
 * mnnq_linear_prefill, computed on the fp16 matrix cores: every group sum is an
 * integer below 2^24 and so exact in fp32. */
int mnnq_linear_prefill_f16(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                            const uint16_t *x16, const float *row_scale, const float *bias, float *y,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Output in IEEE binary16 (Section 4.2 runs the GPU path in fp16): the same sums as the calls
 * above, accumulated in fp32 and rounded once, to nearest even, when stored.  y16: binary16 bits,
 * [N] resp. [M, N] row-major, 16-byte aligned; every other argument as in the call of the same
 * name without the suffix.  Results beyond the binary16 range become infinities. */
int mnnq_linear_decode_o16(const void *packed, int64_t N, int64_t K, int group, int mode,
                           const int8_t *xq, const float *sx, const float *bias, uint16_t *y16, void *stream);
int mnnq_linear_prefill_o16(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                            const int8_t *xq, const float *sx, const float *bias, uint16_t *y16, void *stream);
int mnnq_linear_decode_f16_o16(const void *packed, int64_t N, int64_t K, int group, int mode,
                               const uint16_t *x16, const float *bias, uint16_t *y16, void *stream);
int mnnq_linear_prefill_f16_o16(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                const uint16_t *x16, const float *row_scale, const float *bias, uint16_t *y16,
                                void *stream);
/* The two fused calls keep their workspace arguments (optional for decode, required for prefill). */
int mnnq_linear_decode_fused_o16(const void *packed, int64_t N, int64_t K, int group, int mode,
                                 const float *x, const float *bias, uint16_t *y16,
                                 void *workspace, size_t workspace_bytes, void *stream);
int mnnq_linear_prefill_fused_o16(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                  const float *x, const float *bias, uint16_t *y16,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* Import of weights that were quantized elsewhere (Section 4.2: quantized
 * weights, e.g. from GPTQ, can be imported): canonical arrays in, packed form
 * out - the inverse of mnnq_unpack_weights.
 * q: uint8 [N, K], one code per byte (taken modulo 16); scale: fp32 [N, K/group];
 * zero: [N, K/group], uint8 zero points (values above 15 are stored as 15) in
 * mode MNNQ_W4_ZP_INT, fp32 group minima in mode MNNQ_W4_MIN_FLOAT; all
 * row-major device pointers, q and packed 16-byte aligned.  The packed buffer then behaves
 * exactly like one written by mnnq_pack_weights. */
int mnnq_pack_from_quantized(const uint8_t *q, const float *scale, const void *zero,
                             int64_t N, int64_t K, int group, int mode,
                             void *packed, size_t packed_bytes, void *stream);

/* Integer group accumulators of the W4A8 kernels, for bit-exact checks:
 *   acc[m, n, g] = sum_{k in g} xq[m,k] * (q[n,k] - zero[n,g])      (int32 [M, N, G]);
 * in mode MNNQ_W4_MIN_FLOAT there is no zero point: acc = sum_{k in g} xq[m,k] * q[n,k]
 * (MNNQ_W8_MIN_FLOAT: per nibble plane, see there; MNNQ_ERR_UNSUPPORTED with MNNQ_NATIVE_8BIT).
 * use_prefill_kernel = 0 runs the decode kernel's inner loop row by row (any M),
 * 1 runs the prefill kernel's MFMA loop. */
int mnnq_linear_acc_debug(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                          const int8_t *xq, int32_t *acc, int use_prefill_kernel, void *stream);

/* The same integers from the GEMM on the fp6 matrix instructions (mode with MNNQ_WITH_MATRIX_PLANE,
 * M > 32): acc[m, n, g] as above.  workspace: at least mnnq_workspace_size(M, N, K, group, mode) bytes. */
int mnnq_linear_acc_debug_planes(const void *packed, int64_t M, int64_t N, int64_t K, int group, int mode,
                                 const int8_t *xq, int32_t *acc, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* Tests and tuning: overrides of the launch plans, which otherwise follow from the shapes alone (the
 * library never reads the environment).  key: one of MNNQ_DECODE_KSPLIT (waves per row tile of the GEMV:
 * 1, 2, 4, 8, 16), MNNQ_DECODE_WAVES (4, 8, 16), MNNQ_DECODE_EARLY (0/1), MNNQ_PREFILL_TILE (tile letter,
 * K split digit, k/q), MNNQ_NO_SKINNY, MNNQ_SKINNY_STAGED (0/1), MNNQ_W8_PLANES (1), MNNQ_FUSED_TWO_KERNEL_MIB,
 * MNNQ_PREFILL6_PLAN (0..5: tile plan of the fp6 GEMM), MNNQ_PREFILL6_STAGES (2..4: depth of its LDS rings);
 * value: a string of at most 15 characters, or NULL to clear the override.  Applies to all later calls of the process; not thread safe.  MNNQ_ERR_UNSUPPORTED
 * for an unknown key. */
int mnnq_debug_set(const char *key, const char *value);

/* Test view of the host logic (Section 5.1 chooses loop tiling from the problem's dimensions; here:
 * which kernel configuration a call would launch).  Nothing is launched and no device is needed.
 * what = 0: mnnq_linear_prefill with M > 16 tokens (the tiled GEMM); out8 = {tile rows, tile columns,
 *           K parts inside a workgroup, K split over workgroups, waves per workgroup, LDS bytes per
 *           workgroup, workgroups, form: 0 int4 on the int8 matrix instruction, 1 int8 weights with the two
 *           nibble planes merged in registers, 2 int8 weights in the byte form, 6 the GEMM on the fp6 matrix
 *           instructions (what a call with a workspace runs for a buffer with the matrix-core plane)};
 * what = 1: mnnq_linear_decode; what = 2: mnnq_linear_decode_fused without workspace; out8 = {waves per
 *           workgroup, waves per row tile, weight chunks a wave holds in registers, 1 if it loops with a
 *           prefetch, LDS bytes per workgroup, workgroups, row tiles per workgroup, 1 if the activation
 *           row is requested ahead of the weights and handled while they arrive}.
 * out8: HOST pointer to 8 int32.  Same shape / mode errors as the calls themselves. */
int mnnq_plan_debug(int what, int64_t M, int64_t N, int64_t K, int group, int mode, int32_t *out8);

#ifdef __cplusplus
}
#endif
#endif /* MNNQ_H */
