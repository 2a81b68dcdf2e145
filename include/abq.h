/*
 * abq.h — C ABI of the MI355X (gfx950) arbitrary-precision quantized matmul
 *
 *      Y = dequant( A_q · W_pᵀ ),   p = weight bits, q = activation bits, both in 1..8
 *
 * after ABQ-LLM (arXiv 2408.08554), Sec. 3.4 "Custom Software Engine" and Appendix B
 * "Arbitrary Bit Matrix Calculation".  The integer accumulator is the paper's
 * Y = sum_{s<p} sum_{t<q} 2^(s+t) · BMMA(W^s, X^t)  with  w^s = (w >> s) & 1  (Appendix B),
 * i.e. exactly sum_k A[m,k]·W[n,k] over the unsigned codes; the epilogue applies the affine
 * quantizer of Eq. 3 backwards (value = Delta·(code − z); per output channel for weights,
 * per token for activations, Sec. 4.1).
 *
 * Conventions
 *  - Plain C, every call returns an int status (ABQ_OK or a negative ABQ_ERR_*), nothing is
 *    printed, no exception crosses the boundary.
 *  - Every data pointer is a DEVICE pointer (caller-owned; the library never allocates or
 *    frees device memory) and must be 16-byte aligned.  Sizes come from the *_bytes queries.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *    enqueued asynchronously on it; no call synchronises unless its comment says so.
 *  - Argument validation happens before the first HIP call, so the error paths can be
 *    exercised on a host without a GPU.
 *  - Shapes: A is [M,K] row-major, W is [N,K] row-major (K contiguous on both), Y is [M,N]
 *    row-major.  Any M,N >= 1; 1 <= K <= ABQ_MAX_K and K·(2^p−1)·(2^q−1) <= INT32_MAX
 *    (the paper's "32-bit output"); K need not be a multiple of anything (packers pad with
 *    zero bits, which add nothing to any popcount).
 *  - Same inputs give bit-identical outputs from run to run.
 *
 * Packed operands are opaque blobs whose internal order is private to the kernels.  `layout`
 * says which representations a blob carries and must be the same value at pack time and at
 * every later call that reads the blob:
 *    ABQ_LAYOUT_PLANES  the paper's BitPacking (Sec. 3.4 step 1): [bits][rows][K] 1-bit planes;
 *                       consumed by the AND+popcount bit-serial kernels.
 *    ABQ_LAYOUT_FIELDS  bit-planes kept interleaved in groups of 1/2/4/8 planes (weights) or
 *                       as whole int8 codes (activations), tiled for the int8 MFMA kernels.
 *    ABQ_LAYOUT_BOTH    both of the above.
 *    ABQ_LAYOUT_AUTO    the library's default (currently FIELDS).
 */
#ifndef ABQ_H
#define ABQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ABQ_OK            0
#define ABQ_ERR_NULL     (-1)  /* a required pointer is NULL */
#define ABQ_ERR_BITS     (-2)  /* p or q outside 1..8 */
#define ABQ_ERR_SHAPE    (-3)  /* M,N,K <= 0, K > ABQ_MAX_K, or K·(2^p−1)(2^q−1) > INT32_MAX */
#define ABQ_ERR_ALIGN    (-4)  /* a device pointer is not 16-byte aligned */
#define ABQ_ERR_SIZE     (-5)  /* a caller buffer is smaller than its size query */
#define ABQ_ERR_LAYOUT   (-6)  /* unknown layout value, or the blob lacks what the call needs */
#define ABQ_ERR_HIP      (-7)  /* a HIP call failed; see abq_last_hip_error() */

#define ABQ_LAYOUT_AUTO    0
#define ABQ_LAYOUT_PLANES  1
#define ABQ_LAYOUT_FIELDS  2
#define ABQ_LAYOUT_BOTH    3
#define ABQ_LAYOUT_FIELDS_G128 4   /* field-packed weights with a scale and zero-point per 128 values of K (abq_pack_weights_g128) */
/* abq_gemm only: OR one of these onto a BOTH layout to force a kernel family (A/B timing). */
#define ABQ_USE_PLANES     0x10
#define ABQ_USE_FIELDS     0x20

#define ABQ_MAX_K          131072

int         abq_version(void);                 /* major*10000 + minor*100 + patch */
const char* abq_status_string(int status);     /* static string, never NULL */
int         abq_last_hip_error(void);          /* hipError_t of the last failing HIP call on this thread */
/* Test hook: which decode kernel (Sec. 3.4, GEMV case) the last abq_gemm / abq_gemm_act_codes* call of this thread with
 * M <= 16 on field-packed operands launched; 0 before the first such call. */
#define ABQ_DECODE_DIRECT          1   /* A operand loaded into registers, one workgroup per tile */
#define ABQ_DECODE_STREAMING       2   /* A staged in LDS, ring of weight loads, workgroups walking tiles */
#define ABQ_DECODE_SHARED_OPERAND  3   /* one copy of A in LDS per workgroup of several tiles, every load up front */
int         abq_last_decode_kernel(void);

/* ------------------------------------------------------------------------------------------
 * Weights, offline (Sec. 3.4 step 1 "BitPacking"; "weight BitPacking is implemented offline").
 * ------------------------------------------------------------------------------------------ */

/* Bytes of the packed-weight blob; 0 on invalid arguments. */
size_t abq_packed_weight_bytes(int p, int N, int K, int layout);

/* Packs p-bit weight codes.  Also stores per-channel sum_k W[n,k] (needed by the zero-point
 * correction), w_scale and w_zero inside the blob.
 *   w_codes  [N,K] uint8, values < 2^p (higher bits are ignored)
 *   w_scale  [N] float, Delta_w per output channel
 *   w_zero   [N] int32, integer zero-point in 0..2^p−1
 *   packed_out / packed_bytes: caller buffer of at least abq_packed_weight_bytes(...) bytes;
 *   fully overwritten.  Inputs are not modified. */
int abq_pack_weights(int p, int N, int K,
                     const uint8_t* w_codes, const float* w_scale, const int32_t* w_zero,
                     int layout, void* packed_out, size_t packed_bytes, void* stream);

/* Per-group weight quantization (Appendix C: the method is orthogonal to group-wise weight scales; the
 * group runs along K and holds 128 values, "g128").  The blob is field-packed like ABQ_LAYOUT_FIELDS and
 * carries, per output channel and group, a binary16 scale and an integer zero-point:
 *   Y[m,n] = half_rne( a_scale[m] · sum_g w_scale[n,g] · sum_{k in group g} (A[m,k] − az[m])·(W[n,k] − wz[n,g]) )
 * with G = ceil(K/128) groups per channel, the last one short when 128 does not divide K.  The inner
 * sums are exact integers; the sum over groups is accumulated in binary32 (one rounding per group), so
 * the result carries a relative error of about G·2^-24 of the summed terms' size before the final
 * rounding to binary16.
 *   w_codes      [N,K] uint8, values < 2^p
 *   w_scale_fp16 [N,G] binary16 bit patterns (the precision deployed group formats store)
 *   w_zero       [N,G] int32 in 0..2^p−1
 *   packed_out / packed_bytes: at least abq_packed_weight_bytes(p, N, K, ABQ_LAYOUT_FIELDS_G128) bytes.
 * The order of that binary32 sum follows the launch plan (how K is split over waves), so the same problem
 * through different entry points agrees to this bound, not to the bit.
 * abq_gemm, abq_gemm_act_codes and abq_gemm_grouped take such a blob with w_layout =
 * ABQ_LAYOUT_FIELDS_G128.  Up to 16 rows of A run on the streaming (decode) kernel, more rows on a tiled kernel
 * that flushes its integer accumulators through the group's scale every 128 k.  They cannot return the raw integer
 * accumulator: acc_i32 must be NULL (ABQ_ERR_LAYOUT otherwise).  abq_pack_weights rejects this layout value
 * (ABQ_ERR_LAYOUT). */
int abq_pack_weights_g128(int p, int N, int K,
                          const uint8_t* w_codes, const uint16_t* w_scale_fp16, const int32_t* w_zero,
                          void* packed_out, size_t packed_bytes, void* stream);

/* Test hook: recovers the codes from a blob.  `which` is ABQ_LAYOUT_PLANES or ABQ_LAYOUT_FIELDS
 * and selects the representation to decode (it must be present in the blob).
 *   w_codes_out [N,K] uint8. */
int abq_unpack_weights(int p, int N, int K, int layout, const void* packed, int which,
                       uint8_t* w_codes_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Activations, online (Fig. 3b "ReQuant" + "BitPacking": [M,K,q] -> [q,M,K]).
 * ------------------------------------------------------------------------------------------ */

size_t abq_packed_act_bytes(int q, int M, int K, int layout);

/* Per-token quantize + pack.  For each row m (all float steps in IEEE binary32):
 *   lo = min(min_k x, 0), hi = max(max_k x, 0), Delta = (hi−lo)/(2^q−1)  (Delta=1, z=0 if hi==lo)
 *   z = clamp(rint(−lo/Delta), 0, 2^q−1),  code = clamp(rint(x/Delta) + z, 0, 2^q−1)
 * (the clamp(round(x/Delta)+z) form of Eq. 3; the paper fixes only "per-token").  Stores the
 * codes, Delta, z and sum_k code inside the blob.  NaN/Inf inputs: undefined.
 *   x_fp16 [M,K] IEEE binary16 bit patterns. */
int abq_quant_pack_act(int q, int M, int K, const uint16_t* x_fp16,
                       int layout, void* packed_out, size_t packed_bytes, void* stream);

/* Packs activation codes that are already quantized.
 *   a_codes [M,K] uint8 (< 2^q; higher bits ignored), a_scale [M] float, a_zero [M] int32. */
int abq_pack_act_codes(int q, int M, int K,
                       const uint8_t* a_codes, const float* a_scale, const int32_t* a_zero,
                       int layout, void* packed_out, size_t packed_bytes, void* stream);

/* RMSNorm with the quantizer fused in (Sec. 3.4 / Fig. 3b: the online quantization of a linear layer's input
 * is folded into the operator in front of it; for the LLaMA models of the paper that operator is RMSNorm,
 * y = x / sqrt(mean(x^2) + eps) * gamma, whose formula the paper does not print).  Per token m:
 *   y[m,:] in binary16 (sum of squares exact, 1/sqrt in double rounded once to float, two float products,
 *   one rounding to binary16), then the quantizer of abq_quant_pack_act on y[m,:].
 *   x_fp16 [M,K], gamma_fp16 [K]: binary16 bit patterns;  eps >= 0
 *   a_codes_out [M,K] uint8, a_scale_out [M] float, a_zero_out [M] int32: the inputs of abq_gemm_act_codes
 *   y_fp16_out  [M,K] binary16, optional (NULL to skip): the normalized row before quantization
 * NaN/Inf inputs are undefined. */
int abq_rmsnorm_quant_act(int q, int M, int K, const uint16_t* x_fp16, const uint16_t* gamma_fp16, float eps,
                          uint8_t* a_codes_out, float* a_scale_out, int32_t* a_zero_out,
                          uint16_t* y_fp16_out, void* stream);

/* The same with the residual add in front (Sec. 3.4 / Fig. 3b again: the quantizer rides on the operator that
 * produces the linear layer's input; in the LLaMA block that operator adds a sub-layer's output to the hidden
 * state and normalizes the sum): h = half_rne(float(x) + float(residual)) — one binary32 addition, one rounding to binary16 —
 * then abq_rmsnorm_quant_act on h, all in one kernel.
 *   x_fp16, residual_fp16 [M,K] binary16;  sum_fp16_out [M,K] binary16, required: h, the next residual (it may be the
 *   buffer residual_fp16 itself, not x_fp16);  the other arguments as above. */
int abq_add_rmsnorm_quant_act(int q, int M, int K, const uint16_t* x_fp16, const uint16_t* residual_fp16,
                              const uint16_t* gamma_fp16, float eps,
                              uint8_t* a_codes_out, float* a_scale_out, int32_t* a_zero_out,
                              uint16_t* sum_fp16_out, uint16_t* y_fp16_out, void* stream);

/* SiLU(gate) * up with the quantizer fused in: the producer in front of down_proj in the LLaMA MLP (same passage).
 * Per element h = half_rne((g / (1 + exp(-g))) * up), exp taken as a fixed sequence of binary32 operations
 * (t = clamp(-g * log2 e, -126, 126), n = rint(t), 2^(t-n) by a degree-6 polynomial, scaled by 2^n: within
 * 2e-7 of exp, the same bits on every machine), then the quantizer of abq_quant_pack_act on h[m,:].
 *   gate_fp16, up_fp16 [M,K] binary16;  outputs as for abq_rmsnorm_quant_act (h_fp16_out optional). */
int abq_silu_mul_quant_act(int q, int M, int K, const uint16_t* gate_fp16, const uint16_t* up_fp16,
                           uint8_t* a_codes_out, float* a_scale_out, int32_t* a_zero_out,
                           uint16_t* h_fp16_out, void* stream);

/* Test hook: decodes an activation blob.  Any output pointer may be NULL.
 *   a_codes_out [M,K] uint8, a_scale_out [M] float, a_zero_out [M] int32, a_sum_out [M] int32. */
int abq_unpack_act(int q, int M, int K, int layout, const void* packed, int which,
                   uint8_t* a_codes_out, float* a_scale_out, int32_t* a_zero_out,
                   int32_t* a_sum_out, void* stream);

/* Load-time validation of a packed blob.  The matmul calls take a blob's geometry from their own arguments and
 * never read its header (that would cost a synchronising copy per call), so a p/q, N/M, K or layout value that
 * differs from pack time makes them read outside the blob.  This call is the check: it copies the blob's header
 * to the host — it SYNCHRONISES with `stream` — and compares magic, format version, bit width, rows, K and
 * layout with the arguments, and packed_bytes with the size query.
 *   kind: 0 = packed weights (bits = p, rows = N), 1 = packed activations (bits = q, rows = M)
 * ABQ_OK on a match; ABQ_ERR_LAYOUT on any mismatch (also for an unknown kind or layout value); ABQ_ERR_SIZE
 * when packed_bytes is smaller than the size query (checked before the first HIP call). */
int abq_check_packed(int kind, int bits, int rows, int K, int layout, const void* packed, size_t packed_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Matmul + bit reduction + fused dequant (Sec. 3.4 steps 2–6, Appendix B, Fig. 3b "DeQuant").
 * ------------------------------------------------------------------------------------------ */

/* Scratch bytes abq_gemm needs for this problem (may be 0). */
size_t abq_gemm_workspace_bytes(int p, int q, int M, int N, int K);

/* acc[m,n]  = sum_k A[m,k]·W[n,k]                                  (exact, int32)
 * acc'[m,n] = acc − wz[n]·sum_k A[m,k] − az[m]·sum_k W[n,k] + K·az[m]·wz[n]   (exact, int32)
 * Y[m,n]    = half_rne( float(acc') · a_scale[m] · w_scale[n] )
 *   packed_act, packed_w: blobs written by the pack calls above with the same q,M,K / p,N,K
 *   a_layout, w_layout: the layout value each blob was packed with; w_layout may carry an
 *                 ABQ_USE_* flag.  The kernel family is chosen from what both blobs carry.
 *   y_fp16    [M,N] binary16 bit patterns, required, fully overwritten
 *   acc_i32   [M,N] raw acc, optional (NULL to skip)
 *   workspace at least abq_gemm_workspace_bytes(...) bytes (may be NULL when that is 0);
 *             contents on entry are irrelevant, contents on return are unspecified. */
int abq_gemm(int p, int q, int M, int N, int K,
             const void* packed_act, int a_layout, const void* packed_w, int w_layout,
             uint16_t* y_fp16, int32_t* acc_i32,
             void* workspace, size_t workspace_bytes, void* stream);

/* Activation BitPacking fused into the matmul (Fig. 3b packs activations online on the way into
 * the kernel; Sec. 3.4 keeps that overhead down by fusing it into an existing operator).  Same
 * result, bit for bit, as abq_pack_act_codes followed by abq_gemm on the same arguments.
 *   a_codes [M,K] uint8 row-major, values < 2^q;  a_scale [M] float;  a_zero [M] int32  (device)
 *   packed_w, w_layout, y_fp16, acc_i32, stream: as for abq_gemm
 *   workspace at least abq_gemm_act_codes_workspace_bytes(...) bytes.  That query returns 0 when
 *             the call runs as ONE kernel: the decode shapes (M <= 16, or M <= 64 with few output
 *             tiles) on field-packed weights with K a multiple of 16 — the codes are offset to
 *             signed bytes and their row sums taken while the kernel stages them.  For every
 *             other problem the packed activations are written to the workspace and the two
 *             steps run back to back on the stream.
 * Errors as abq_gemm (ABQ_ERR_NULL / ABQ_ERR_SIZE when a needed workspace is missing / too small). */
size_t abq_gemm_act_codes_workspace_bytes(int p, int q, int M, int N, int K, int w_layout);
int abq_gemm_act_codes(int p, int q, int M, int N, int K,
                       const uint8_t* a_codes, const float* a_scale, const int32_t* a_zero,
                       const void* packed_w, int w_layout,
                       uint16_t* y_fp16, int32_t* acc_i32,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ReQuant fused into the matmul epilogue (Fig. 3b: the kernel's output is quantized again for the next layer; the last
 * paragraph of Sec. 3.4 folds quantization into neighbouring operators — this is the consumer side, the producers
 * above are the other).  abq_gemm_act_codes that also (or only) writes the next layer's activation codes.  A token's
 * own range is unknown before its whole output row exists, so Delta and z per token are the caller's (a calibrated or
 * previous-step range):
 *   code[m,n] = clamp( clamp(rint(Y[m,n] / out_scale[m]), -2^24, 2^24) + out_zero[m], 0, 2^q_out − 1 )
 * on the binary16 value Y[m,n] of abq_gemm, division and rint in IEEE binary32 (Eq. 3's clamp(round(x/Delta)+z)).
 *   q_out      1..8;  out_scale [M] float > 0;  out_zero [M] int32  (device)
 *   codes_out  [M,N] uint8, required: feeds the next abq_gemm_act_codes together with out_scale / out_zero
 *   y_fp16     [M,N] binary16, optional here (NULL to skip)
 *   the other arguments, the workspace and the errors as for abq_gemm_act_codes (same workspace query); ABQ_ERR_BITS
 *   also for q_out; ABQ_ERR_LAYOUT for ABQ_LAYOUT_FIELDS_G128 blobs (not built for them).  NaN/Inf outputs and
 *   out_scale <= 0 are undefined. */
int abq_gemm_act_codes_requant(int p, int q, int M, int N, int K,
                               const uint8_t* a_codes, const float* a_scale, const int32_t* a_zero,
                               const void* packed_w, int w_layout,
                               int q_out, const float* out_scale, const int32_t* out_zero, uint8_t* codes_out,
                               uint16_t* y_fp16, void* workspace, size_t workspace_bytes, void* stream);

/* abq_gemm_act_codes for callers that cannot allocate device memory or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same call with no workspace argument.
 * Where abq_gemm_act_codes needs a workspace (the packed activations of its two-kernel path) this variant keeps
 * it in a buffer of ABQ_STATIC_SCRATCH_BYTES bytes that is part of the library's device image (every GPU the
 * library runs on holds it until the process ends).  It allocates nothing and frees nothing.
 * Same arguments, results (bit for bit) and errors as abq_gemm_act_codes; in addition ABQ_ERR_SIZE when
 * abq_gemm_act_codes_workspace_bytes(...) for the problem exceeds ABQ_STATIC_SCRATCH_BYTES (checked before
 * the first HIP call).  All calls on one GPU share that GPU's buffer: calls that may overlap on one GPU
 * (different streams, different host threads) race on it and must be serialized by the caller; calls on one
 * stream are safe.  The buffer needs no clearing between calls (each call writes what it reads). */
#define ABQ_STATIC_SCRATCH_BYTES (32u << 20)
int abq_gemm_act_codes_static(int p, int q, int M, int N, int K,
                              const uint8_t* a_codes, const float* a_scale, const int32_t* a_zero,
                              const void* packed_w, int w_layout,
                              uint16_t* y_fp16, int32_t* acc_i32, void* stream);

/* Very low bit widths on gfx950's 4-bit floating-point MFMA (Sec. 3.4 / Table 4: narrower operands should run faster;
 * Appendix B's sum over 1-bit planes is what makes that true on tensor cores that multiply bits).  For weights AND
 * activations of one or two bits the codes 0..3 are E2M1 values and the sums of their products are exact in the
 * instruction's binary32 accumulator for every K <= ABQ_MAX_K, so abq_f4_gemm returns the same int32 accumulator and
 * binary16 output as abq_gemm, at twice the matrix rate of the int8 path.  Both operands use one packed layout:
 *   abq_f4_packed_bytes(bits, rows, K)  size of the blob for a [rows][K] operand (0 for arguments out of range)
 *   abq_f4_pack_codes   codes u8 [rows][K] (device, row-major; bits above `bits` are dropped), scale f32 [rows] and
 *                       zero i32 [rows] (device; the zero-point of a `bits`-bit code, 0..2^bits-1: the matmul's
 *                       epilogue relies on it) -> blob `packed_out` (device, caller-owned, >= the size above);
 *                       for the weights rows = N, for the activations rows = M
 *   abq_f4_gemm         Y[M,N] = dequant(A . W^T) from two such blobs (p: bits of W, q: bits of A, both 1 or 2);
 *                       y_fp16 [M][N] device, acc_i32 [M][N] device or NULL
 * Device pointers 16-byte aligned; work is enqueued on `stream`; nothing is allocated.  ABQ_ERR_NULL, ABQ_ERR_BITS
 * (bits outside 1..2), ABQ_ERR_SHAPE, ABQ_ERR_ALIGN, ABQ_ERR_SIZE, ABQ_ERR_HIP as elsewhere.  The blobs are not
 * interchangeable with those of abq_pack_weights / abq_pack_act_codes. */
size_t abq_f4_packed_bytes(int bits, int rows, int K);
int abq_f4_pack_codes(int bits, int rows, int K, const uint8_t* codes, const float* scale, const int32_t* zero,
                      void* packed_out, size_t packed_bytes, void* stream);
int abq_f4_gemm(int p, int q, int M, int N, int K, const void* packed_act, const void* packed_w,
                uint16_t* y_fp16, int32_t* acc_i32, void* stream);

/* Launch-plan table (Appendix D, "auto kernel search": the engine picks, per problem size, the fastest of a
 * set of kernel configurations found by timing them).  The library chooses every launch plan from closed-form
 * rules; this table lets a tuner (paper_2408_08554_amd/tune.py times the candidates on the device) replace the
 * rule for exact problem sizes.  A field left 0 keeps the rule for that knob; a plan that does not fit the
 * problem (say, more waves than K has 512-blocks) is ignored and the rule applies.  Results never depend on
 * the plan (per-group weight scales: to their stated bound).  Process-wide, thread-safe; entries hold no
 * device state.
 *   skinny_waves    waves per workgroup of the decode kernel = K split of a tile: 1, 2, 4..8
 *   skinny_kgroups  K groups of the decode kernel: 1..4
 *   tiled_mt        rows of A per workgroup tile of the prefill kernel / 16: 4 or 8
 *   tiled_ntw       16-channel tiles of W per wave: 1, 2 or 4
 *   tiled_wd        operand steps in flight: 2 or 4 (4 exists for tiled_mt = 4 with tiled_ntw <= 2)
 *   tiled_band      row blocks of A per band of the tile order: >= 1
 *   direct_r        decode kernel for M <= 16: -1 the streaming kernel (A staged in LDS, load ring); 1, 2 or 4 the
 *                   direct kernel (A operand loaded into registers) with that many 512-k blocks per wave; -2 the
 *                   shared-operand kernel (one copy of A in LDS per workgroup of several tiles) where it fits, else the
 *                   streaming kernel
 * abq_plan_set: plan == NULL removes the entry.  ABQ_ERR_BITS / ABQ_ERR_SHAPE as abq_gemm; ABQ_ERR_LAYOUT for a
 * value outside the lists above.  abq_plan_get fills *out (all zero when there is no entry). */
typedef struct abq_plan {
    int skinny_waves, skinny_kgroups;
    int tiled_mt, tiled_ntw, tiled_wd, tiled_band;
    int direct_r;
} abq_plan;
int  abq_plan_set(int p, int q, int M, int N, int K, const abq_plan* plan);
int  abq_plan_get(int p, int q, int M, int N, int K, abq_plan* out);
void abq_plan_clear(void);

/* Grouped decode launch (Sec. 3.4: the engine replaces every linear layer of a decoder block; Table 4's
 * matmuls take microseconds each, so launching them one by one leaves the memory system idle between
 * them).  `count` independent problems that share p, q, M and the layouts, each with its own N, K,
 * weights, activations and outputs, are served by ONE kernel launch per eight problems when every
 * problem is decode-shaped: M <= 16, K >= 2048 (K a multiple of 16 for unpacked codes), up to 16 rows of
 * A fitting LDS ((M * (K + 528) below ~120 KB), field-packed weights.  Otherwise the problems run one
 * after the other exactly as abq_gemm / abq_gemm_act_codes would run them.  Results are bit-identical
 * to the single calls either way.
 *   host_problems: HOST array of `count` descriptors holding DEVICE pointers.  Each gives its activations
 *                  either packed (packed_act, a_codes = NULL) or as unpacked codes (a_codes, a_scale, a_zero,
 *                  packed_act = NULL); all problems of a call use the same form.  The array is read before the
 *                  call returns.
 *   workspace:     at least abq_gemm_grouped_workspace_bytes(...) bytes (0 whenever one launch serves the group
 *                  or the activations are packed).
 * Errors as abq_gemm; ABQ_ERR_SHAPE also for count < 1, ABQ_ERR_LAYOUT for mixed activation forms. */
typedef struct abq_problem {
    int N, K;
    const void* packed_w;       /* abq_pack_weights(p, N, K, ..., w_layout) */
    const void* packed_act;     /* abq_pack_act_codes / abq_quant_pack_act (q, M, K, ..., a_layout), or NULL */
    const uint8_t* a_codes;     /* [M,K] uint8 codes < 2^q, or NULL */
    const float* a_scale;       /* [M], with a_codes */
    const int32_t* a_zero;      /* [M], with a_codes */
    uint16_t* y_fp16;           /* [M,N], required */
    int32_t* acc_i32;           /* [M,N] raw accumulator, may be NULL */
} abq_problem;
size_t abq_gemm_grouped_workspace_bytes(int p, int q, int M, int count, const abq_problem* host_problems,
                                        int a_layout, int w_layout);
int abq_gemm_grouped(int p, int q, int M, int count, const abq_problem* host_problems,
                     int a_layout, int w_layout, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ABQ_H */
