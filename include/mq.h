/*
 * mq.h -- C boundary of the MI355X (gfx950) low-precision matrix-product library.
 *
 * The library implements the integer matrix-product path of arxiv 1805.12096:
 *   quant_int  (Section 4.2, "Quantization and integer products"): a float
 *              tensor is multiplied by a quantization multiplier and rounded to
 *              8- or 16-bit signed integers;
 *   dot'_int   (Section 4.3, "Memoization"): the product of two quantized
 *              tensors, A times the transpose of B, both contiguous along the
 *              contracted index, accumulated in 32 bits (Section 4.2);
 *   memoized   quant_int(B^T) of a parameter is a constant of the graph and is
 *              computed once (Section 4.3) -- here: mq_prepare_weight;
 *   epilogue   the integer product replaces the float product (Sections 4.3,
 *              4.4): sums are scaled back to float, the bias is added, outputs
 *              are not clipped or quantized (Section 4.2);
 *   arg-max    with beam size 1 no softmax is evaluated, the highest activation
 *              wins (Section 2.3, "Decoding with small beams").
 *
 * General rules
 *   - Every pointer named "dev" or documented as device memory is a HIP device
 *     pointer on the current device.  The CALLER owns every buffer; the library
 *     never allocates, frees, or keeps a pointer after the call returns.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and returns without synchronizing.  Results
 *     are valid once the stream has reached that point.
 *   - Matrices are dense and row-major.  A is [M x K]; the parameter is used
 *     as Wt = B^T, [N x K]; outputs are [M x N].
 *   - Quantization multipliers ("scales") live in device memory as one float
 *     each, so that chains of calls never wait for the host.
 *   - bits is 8 (values in [-127, 127], int8_t) or 16 ([-32767, 32767], int16_t).
 *   - Every function returning int returns an mq_status.  Arguments are checked
 *     before anything is enqueued; a failed check enqueues nothing.  Pointers
 *     to float / int32 data must be 4-byte aligned, `x`, `q`, `qA`, `packed`
 *     16-byte aligned (MQ_ERR_ALIGN otherwise).  Sizes must be non-zero and the
 *     element counts M*K, N*K, M*N must fit in 2^40 (MQ_ERR_SHAPE otherwise).
 *   - Inputs are expected to be finite.  A NaN never faults: it is ignored by
 *     the abs-max and quantizes to 0.
 *   - Integer sums are exact modulo 2^32 (two's complement wrap), independent of
 *     tiling.  With 8-bit operands no sum can wrap for K <= 133 144.
 *
 * Single-pass kernels (grid-wide agreement inside one launch)
 *   A per-tensor multiplier Qmax / max|x| needs the maximum over the whole tensor
 *   before the first element can be converted.  Where the tensor fits the registers
 *   of one resident grid, some calls do both in ONE launch: every workgroup
 *   publishes its maximum in a slot of the workspace, waits until all slots are
 *   filled and converts from registers.  These are mq_gemm_requant_single_packed,
 *   mq_ffn_i8_f32 / mq_ffn_i8_f32_prepared (first product and input quantizer),
 *   mq_quantize_absmax_pack_f32 (from 2^20 elements) and its _prepared form.
 *   What they need and what they do when they do not get it:
 *   - The agreement area is 2112 words of the workspace: eight copies of 256 slots
 *     (one per workgroup; eight so that pollers spread over cache lines), one sticky
 *     failure word, one count of workgroups that are done.  It must be all zero when
 *     the kernel starts; the plain entry points clear it with a small launch, the
 *     _prepared ones keep it zero from call to call.
 *   - The launcher only takes this path if the grid fits the device when the device
 *     is EMPTY (occupancy x compute units >= workgroups, and at most 256 workgroups;
 *     mq_single_pass_fits is that test).  It cannot know what else is running.  These
 *     calls therefore need the GPU to themselves while they run: no kernel of another
 *     stream or process resident at the same time, and never two single-pass calls
 *     in flight at once (not even on separate workspaces).  Otherwise some workgroups
 *     may not become resident while the others wait for them.
 *   - The wait is bounded (mq_set_barrier_timeout_us, default 0.5 s).  A workgroup
 *     that gives up raises the sticky word; the multiplier the call publishes
 *     (scale_out, or the internal one of the FFN block) is then NaN and so is every
 *     float computed from it; the status of the call is still MQ_OK, because nothing
 *     is known on the host.  Check the multiplier (or the output) for NaN where
 *     co-residency cannot be excluded, or switch the single-pass kernels off
 *     (mq_set_ffn_single_pass(0), mq_set_quantize_single_pass(0)): the two-pass forms
 *     give the same bits and wait for nothing.
 */
#ifndef MQ_H_
#define MQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mq_status {
  MQ_OK = 0,
  MQ_ERR_NULL = 1,        /* a required pointer is NULL */
  MQ_ERR_SHAPE = 2,       /* a size is zero or too large */
  MQ_ERR_DTYPE = 3,       /* bits is not 8 or 16 (or the call supports 8 only) */
  MQ_ERR_ALIGN = 4,       /* a pointer is not aligned as required */
  MQ_ERR_WORKSPACE = 5,   /* workspace smaller than the *_ws_bytes query says */
  MQ_ERR_UNSUPPORTED = 6, /* valid arguments the library cannot serve */
  MQ_ERR_HIP = 7,         /* the HIP runtime refused a launch; see mq_last_hip_error */
  MQ_ERR_LIMIT = 8        /* a size is beyond what the library's static scratch array serves */
} mq_status;

/* Library version: major * 10000 + minor * 100 + patch. */
int mq_version(void);

/* Static, NUL-terminated description of a status code (never NULL). */
const char* mq_status_string(int status);

/* hipError_t value of the last failed HIP call made by this thread inside the
 * library (0 if none). */
int mq_last_hip_error(void);

/* Tuning knob for measurements in the spirit of the paper's auto-tuner (Section
 * 4.4: alternative implementations are timed per shape and the fastest is
 * kept).  variant 0 (default) lets the library choose the tile configuration of
 * the product kernels from the problem shape; 1..14 (8 bit) or 1..8 (16 bit)
 * force one configuration for every following product of this process (results
 * are identical, only speed changes; a variant that does not exist for the
 * operand width makes the product calls return MQ_ERR_UNSUPPORTED; the fused
 * epilogues of the FFN block keep to the tile shapes they support).  Not thread
 * safe. */
int mq_set_gemm_variant(int variant);

/* ---- quant_int (Section 4.2) -------------------------------------------- */

/* amax[0] = max_i |x[i]| over n floats (NaNs skipped).  The paper uses fixed
 * multipliers; a per-tensor multiplier Qmax / max|x| needs this reduction.
 * x: device, 16-byte aligned.  amax: device float[1], overwritten. */
int mq_absmax_f32(const float* x, size_t n, float* amax, void* stream);

/* scale[0] = Qmax(bits) / amax[0] as one correctly rounded binary32 division;
 * 1.0f if amax[0] is 0.  amax, scale: device float[1] (may be the same address). */
int mq_scale_from_amax(const float* amax, int bits, float* scale, void* stream);

/* quant_int: q[i] = clamp(round_half_even(x[i] * scale[0]), -Qmax, +Qmax), the
 * product taken in binary32.  x: device float [rows x cols]; q: device
 * int8_t / int16_t [rows x cols]; scale: device float[1].
 * rowsum (device int32 [rows], may be NULL): receives sum_c q[r][c]; the 16-bit
 * product needs it (see mq_gemm_i32). */
int mq_quantize_f32(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                    void* q, int32_t* rowsum, void* stream);

/* quant_int straight into the packed layout of mq_prepare_weight (the packed
 * layout is the same for both operands of dot'_int): packed receives
 * mq_packed_bytes(bits, rows, cols) bytes, padding included; for bits == 16 the
 * row sums the product needs are stored inside the buffer.  This is the fast
 * path for activations: the packed product kernels stream such a buffer into
 * LDS with linear copies.  x: device float [rows x cols]; scale: device float[1];
 * packed: device, 16-byte aligned.  mq_unpack_weight(packed, bits, rows, cols, q)
 * recovers the plain row-major integers. */
int mq_quantize_pack_f32(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                         void* packed, void* stream);

/* Abs-max and quant_int into the packed layout in two launches with no
 * shared-address atomics.  Same results as mq_absmax_f32 + mq_scale_from_amax +
 * mq_quantize_pack_f32; Qmax / max (one correctly rounded division) is stored in
 * scale_out[0].  Tensors of at most 2048 groups of 8 rows x 1024 columns
 * (16 bit: at most 16384 rows of at most 1024 columns) are read ONCE: after a
 * tiny launch that clears a few words of ws, one kernel holds the whole tensor
 * in registers while its workgroups agree on the maximum (bounded wait, NaN
 * multiplier on failure, as described at mq_gemm_requant_single_packed).  Larger
 * tensors take two passes: per-block partial maxima to ws, then the quantizing
 * kernel; so do tensors below 2^20 elements, for which two tiny kernels are
 * quicker than one with a grid-wide wait.  mq_set_quantize_single_pass(0) forces
 * the two-pass form, (2) the single-pass form whenever the tensor fits, (1) is
 * the default choice by size.
 * ws: device, 16-byte aligned, mq_quantize_absmax_ws_bytes(), contents
 * irrelevant on entry.  Layout: the agreement area first, the partial maxima of
 * the two-pass form behind it; the call leaves the agreement area as the
 * _prepared form below wants it (all zero) whenever it touched it, so the two
 * entry points may share a workspace. */
int mq_set_quantize_single_pass(int enable);
size_t mq_quantize_absmax_ws_bytes(void);
int mq_quantize_absmax_pack_f32(const float* x, size_t rows, size_t cols, int bits, void* packed,
                                float* scale_out, void* ws, size_t ws_bytes, void* stream);

/* The same for callers that keep the workspace to themselves (a decode loop, a captured graph): the agreement
 * words of the kernel that reads x once are zeroed ONCE by mq_quantize_absmax_ws_prepare and left zero by every
 * mq_quantize_absmax_pack_f32_prepared call (the last workgroup done with them zeroes them), so no call spends
 * a launch on clearing them and the one-kernel form is used for every tensor that fits it, small ones included.
 * Results are identical to mq_quantize_absmax_pack_f32.  Nobody else may write to the workspace between the
 * calls, and calls sharing a workspace must not overlap.  A call whose agreement timed out (multiplier NaN)
 * still leaves the words zero.  Arguments as above. */
int mq_quantize_absmax_ws_prepare(void* ws, size_t ws_bytes, void* stream);
int mq_quantize_absmax_pack_f32_prepared(const float* x, size_t rows, size_t cols, int bits, void* packed,
                                         float* scale_out, void* ws, size_t ws_bytes, void* stream);

/* ---- memoized quant_int(B^T) (Section 4.3) ------------------------------ */

/* Bytes of the packed parameter for an [N x K] Wt; 0 if bits is invalid or a
 * size is zero. */
size_t mq_packed_bytes(int bits, size_t N, size_t K);

/* Quantize a float parameter, transpose it to [N x K] if needed and store it in
 * the tile order the product kernels read.  Done once per parameter; the packed
 * buffer is then a constant that any number of products reuse.
 *   B: device float; b_is_transposed == 0: B is [K x N]; != 0: B is Wt, [N x K].
 *   scale_or_null: device float[1] multiplier to use, or NULL to use
 *     Qmax / max|B| (computed here).
 *   scale_out: device float[1], receives the multiplier used (required).
 *   packed: device, 16-byte aligned, mq_packed_bytes(bits, N, K) bytes, fully
 *     overwritten (padding included), opaque but position independent: it may
 *     be copied or saved as plain bytes. */
int mq_prepare_weight(const float* B, int b_is_transposed, size_t N, size_t K, int bits,
                      const float* scale_or_null, float* scale_out, void* packed, void* stream);

/* Inverse of the packing, for inspection and tests: q_out receives the
 * quantized Wt as plain row-major int8_t / int16_t [N x K] (device). */
int mq_unpack_weight(const void* packed, int bits, size_t N, size_t K, void* q_out, void* stream);

/* ---- dot'_int (Sections 4.2, 4.3) --------------------------------------- */

/* C[m][n] = sum_k qA[m][k] * Wt[n][k] modulo 2^32, raw 32-bit sums.
 *   qA: device int8_t / int16_t [M x K], row-major.
 *   rowsumA: device int32 [M] with sum_k qA[m][k]; required for bits == 16
 *     (the 16-bit product runs as four 8-bit products on offset byte planes and
 *     the row sums undo the offset), ignored for bits == 8 (may be NULL).
 *   packedW: from mq_prepare_weight with the same bits, N, K.
 *   C: device int32 [M x N]. */
int mq_gemm_i32(const void* qA, const int32_t* rowsumA, const void* packedW, int bits,
                size_t M, size_t N, size_t K, int32_t* C, void* stream);

/* Product with the float epilogue fused:
 *   Y[m][n] = fma((float)acc[m][n], 1 / (sA[0] * sW[0]), bias ? bias[n] : 0),
 *   then max(Y, 0) if relu != 0.
 * sA, sW: device float[1] multipliers of the two operands.  bias: device float
 * [N] or NULL.  Y: device float [M x N].
 * out_amax: NULL, or device float[1] that the CALLER has set to 0 (or to a
 * running maximum): on return it holds max(previous, max |Y|), so the next
 * quant_int of Y needs no separate reduction pass. */
int mq_gemm_dequant(const void* qA, const int32_t* rowsumA, const void* packedW, int bits,
                    size_t M, size_t N, size_t K, const float* sA, const float* sW,
                    const float* bias, int relu, float* Y, float* out_amax, void* stream);

/* The same two products with the activations packed by mq_quantize_pack_f32
 * (packedA: [M x K], same bits as packedW).  Results are identical to the
 * row-major calls; these are the fast kernels (direct-to-LDS loads of both
 * operands, several K steps in flight). */
int mq_gemm_i32_packed(const void* packedA, const void* packedW, int bits, size_t M, size_t N, size_t K,
                       int32_t* C, void* stream);
int mq_gemm_dequant_packed(const void* packedA, const void* packedW, int bits, size_t M, size_t N, size_t K,
                           const float* sA, const float* sW, const float* bias, int relu, float* Y,
                           float* out_amax, void* stream);

/* Two-pass re-quantizing product (8 bit), the building block of mq_ffn_i8_f32:
 * pass 1 computes y = fma((float)acc, 1/(sA sW), bias) (+ReLU) exactly like
 * mq_gemm_dequant_packed but only writes one partial max|y| per tile to ws;
 * pass 2 computes the same y again, forms s = 127 / max|y| from the partials
 * (1 if the maximum is 0), stores it in scale_out[0] and writes
 * quant_int(y, s) as packed 8-bit activations [M x N] (mq_packed_bytes(8, M, N)
 * bytes) ready to be the A operand of the next product.  The float tensor y is
 * never stored.  Both passes must see the same arguments (and the same
 * mq_set_gemm_variant setting).  ws: device, 16-byte aligned,
 * mq_gemm_amax_ws_bytes(M, N) bytes. */
size_t mq_gemm_amax_ws_bytes(size_t M, size_t N);
int mq_gemm_amax_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                        const float* sA, const float* sW, const float* bias, int relu,
                        void* ws, size_t ws_bytes, void* stream);
int mq_gemm_requant_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                           const float* sA, const float* sW, const float* bias, int relu,
                           const void* ws, size_t ws_bytes, float* scale_out, void* packed_out, void* stream);

/* The same result in ONE pass over the operands, for results small enough that
 * every 256 x 256 tile is resident on the chip at once (at most one tile per
 * compute unit; MQ_ERR_UNSUPPORTED beyond that, nothing computed): each tile
 * keeps its sums in registers while all workgroups agree on max|y| through the
 * agreement area at the start of ws (2112 words, see "Single-pass kernels" at
 * the top), then quantizes and stores.  Two launches (clearing the area, the
 * product).  The wait for the other workgroups is bounded (0.5 s);
 * should it ever expire, scale_out[0] is set to NaN so that nothing computed
 * from it can pass for a result.  Needs the GPU to itself (see the top).
 * Arguments and results as mq_gemm_requant_packed; ws is written here.
 * mq_single_pass_fits(M, N, resident) is the launcher's size test on its own
 * (no device needed): 1 if an [M x N] result has at most min(resident, 256)
 * tiles of 256 x 256, where `resident` is the number of workgroups of the kernel
 * the device holds at once (occupancy x compute units; 256 on MI355X).
 * mq_set_barrier_timeout_us changes the bound on the wait (default 500000, at
 * most 10^7; 0 makes every waiter give up at once, which is how the tests
 * reach the failure path without a kernel that hangs). */
int mq_set_barrier_timeout_us(unsigned us);
int mq_single_pass_fits(size_t M, size_t N, size_t resident);
int mq_gemm_requant_single_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                  const float* sA, const float* sW, const float* bias, int relu,
                                  void* ws, size_t ws_bytes, float* scale_out, void* packed_out,
                                  void* stream);

/* Single-pass variant for multipliers fixed in advance, the paper's own scheme
 * (Section 4.2: 2^10 for 16 bit, 127/2 after clipping to [-2, 2] for 8 bit):
 * quant_int of the next product's input is done in the epilogue of the product
 * that creates it, with the given multiplier s_out[0] (device float[1], read
 * only); values beyond +-127 / s_out saturate, which is the clipping of Section
 * 4.2.  No abs-max pass, no workspace. */
int mq_gemm_requant_fixed_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                 const float* sA, const float* sW, const float* bias, int relu,
                                 const float* s_out, void* packed_out, void* stream);

/* The same for 16-bit operands (Section 4.2: 16-bit values with the fixed
 * multiplier 2^10): both operands packed 16 bit, the result
 * quant_int(relu?(A Bt / (sA sW) + bias), s_out[0]) saturated to +-32767 and
 * written as packed 16-bit activations [M x N] (mq_packed_bytes(16, M, N)
 * bytes: both byte planes and the row sums the next product needs; the row
 * sums are cleared and accumulated here).  Two launches, no workspace. */
int mq_gemm_requant_fixed_packed_i16(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                     const float* sA, const float* sW, const float* bias, int relu,
                                     const float* s_out, void* packed_out, void* stream);

/* ---- auto-tuning (Section 4.4) ------------------------------------------
 * The paper times alternative implementations per tensor shape over a fixed
 * number of runs and then uses the fastest for all following calls.  Here the
 * alternatives are the tile configurations of the packed product kernels.
 * mq_autotune_gemm times every configuration valid for `bits` on an [M x K] x
 * [N x K] problem (`runs` launches each, in two rounds of which the faster counts,
 * after about 30 ms of untimed launches that bring an idle device to its working
 * clock; on dummy operands inside ws), records
 * the fastest in a process-wide table keyed by (bits, M, N, K) -- which all
 * packed products of that shape consult from then on, unless
 * mq_set_gemm_variant forces a configuration -- and reports it.  Results of the
 * products never depend on the configuration.  UNLIKE every other call this one
 * synchronizes with the stream (it reads timers) and is meant for set-up time.
 * ws: device, 256-byte aligned, mq_autotune_ws_bytes(bits, M, N, K) bytes.
 * best_variant / best_us (host pointers, may be NULL) receive the choice and its
 * average microseconds.  Not thread safe; the table holds 256 shapes. */
size_t mq_autotune_ws_bytes(int bits, size_t M, size_t N, size_t K);
/* The times of the most recent mq_autotune_gemm run: us_by_variant (HOST float[n]) receives the microseconds per
 * launch of variant v at index v (index 0 and variants that do not exist for the operand width: -1), winners and
 * losers alike.  For 16 bit the candidates are six tile configurations of the decomposition onto four 8-bit matrix
 * products (1..6) and the vector-ALU kernel built on the 16-bit dot instruction (7), the chip's counterpart of the
 * instruction the paper's 16-bit kernel uses (Section 4.2). */
int mq_autotune_report(float* us_by_variant, int n);
int mq_autotune_gemm(int bits, size_t M, size_t N, size_t K, int runs, void* ws, size_t ws_bytes,
                     void* stream, int* best_variant, float* best_us);

/* ---- greedy output layer (Section 2.3) ---------------------------------- */

/* Workspace bytes mq_gemm_argmax needs for an M-row problem. */
size_t mq_argmax_ws_bytes(size_t M, size_t N);

/* 8-bit product against the (tied embedding) output matrix with the beam-1
 * arg-max fused; the M x N logits are never written:
 *   tok[m]      = smallest n with acc[m][n] == max_n acc[m][n]
 *   maxlogit[m] = (float)max_n acc[m][n] * (1 / (sA[0] * sW[0]))
 * qA: device int8_t [M x K]; packedW: 8-bit packed [N x K]; tok: device int32
 * [M]; maxlogit: device float [M]; ws: device, 16-byte aligned, at least
 * mq_argmax_ws_bytes(M, N) bytes, contents irrelevant on entry and undefined
 * on return.  N must be below 2^31. */
int mq_gemm_argmax(const void* qA, const void* packedW, size_t M, size_t N, size_t K,
                   const float* sA, const float* sW, int32_t* tok, float* maxlogit,
                   void* ws, size_t ws_bytes, void* stream);

/* The same with the hidden states packed by mq_quantize_pack_f32 (8 bit): the
 * decode-step kernel.  The hidden states sit in registers, the embedding
 * streams through LDS exactly once, each block reports one candidate per
 * sentence and a second small kernel picks the winners.  Rows are processed
 * 384 at a time (the embedding streams once per pass).  Serves K <= 512
 * (MQ_ERR_UNSUPPORTED beyond; use mq_gemm_argmax there).  Same results, same
 * workspace query. */
int mq_gemm_argmax_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                          const float* sA, const float* sW, int32_t* tok, float* maxlogit,
                          void* ws, size_t ws_bytes, void* stream);

/* mq_gemm_argmax_packed for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The per-workgroup candidates
 * (the `ws` of mq_gemm_argmax_packed) live in a static device array of the library instead: 768 KiB (384 rows x
 * 256 workgroups x 8 bytes) per GPU the library runs on, held until the process ends.  The call allocates
 * nothing and frees nothing, here or inside the runtime's allocator; inputs and outputs are still the caller's.
 * Same arguments otherwise, same results bit for bit.
 * Limits: K <= 512 and N <= 1044480 as for mq_gemm_argmax_packed (MQ_ERR_UNSUPPORTED beyond), M <= 24576 rows
 * (MQ_ERR_LIMIT beyond: "a size is beyond what the library's static scratch array serves").
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams or
 * threads) race and give undefined tokens; calls on one stream are ordered and safe.  Nothing in the array has
 * to be zero on entry (every word that is read was written by the same call before). */
int mq_gemm_argmax_packed_static(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                 const float* sA, const float* sW, int32_t* tok, float* maxlogit, void* stream);

/* Short-listed output layer (Section 4.1 "Shortlist": the output product is
 * restricted to a subset of translation candidates).  shortlist: device int32
 * [shortlist_len], vocabulary row ids in [0, N), strictly ascending.  Only these
 * rows of the packed [N x K] embedding are read (gathered by the loads
 * themselves, no compacted copy is made):
 *   tok[m] = the listed row with the largest sum (the smallest id on ties),
 *   maxlogit[m] as in mq_gemm_argmax.
 * The list is the caller's contract; it is not validated on the host (it lives in device memory).  An id outside
 * [0, N) never reads outside the embedding: the kernel scores row 0 (for a negative id) or row N - 1 in its
 * place, and if that candidate wins, tok[m] is the id as listed.  A list that is not ascending only changes
 * which of several equal sums wins.  Same limits and workspace as mq_gemm_argmax_packed. */
int mq_gemm_argmax_shortlist(const void* packedA, const void* packedW, const int32_t* shortlist,
                             size_t shortlist_len, size_t M, size_t N, size_t K,
                             const float* sA, const float* sW, int32_t* tok, float* maxlogit,
                             void* ws, size_t ws_bytes, void* stream);

/* ---- composition -------------------------------------------------------- */

/* Workspace bytes mq_linear_f32 needs. */
size_t mq_linear_ws_bytes(int bits, size_t M, size_t K);

/* Float-in, float-out replacement for Y = A * B + bias with a prepared
 * parameter (Section 4.3: the integer product as a drop-in for the float one):
 * abs-max and quant_int of A (or quant_int with the given multiplier if
 * sA_or_null is not NULL), dot'_int, dequantize + bias (+ReLU), with the results
 * of mq_quantize_f32 + mq_gemm_dequant bit for bit.  Two or three launches on
 * `stream`; for 8-bit products with at most 512 rows and K a multiple of 32 up
 * to 1024 (a decode step) quant_int runs inside the product kernel: one launch
 * with a given multiplier, two with abs-max.
 * A: device float [M x K], 16-byte aligned.  out_amax: optional device float
 * that is raised to max|Y| (the caller zeroes it).  ws: device workspace of
 * mq_linear_ws_bytes bytes, 16-byte aligned, contents irrelevant. */
int mq_linear_f32(const float* A, size_t M, size_t K, const float* sA_or_null,
                  const void* packedW, const float* sW, int bits, size_t N,
                  const float* bias, int relu, float* Y, float* out_amax,
                  void* ws, size_t ws_bytes, void* stream);

/* Workspace bytes mq_ffn_i8_f32 needs (0 for invalid sizes). */
size_t mq_ffn_ws_bytes(size_t M, size_t d, size_t f);

/* Transformer feed-forward block (Table 1: d -> f -> d) in 8 bit with per-tensor
 * abs-max multipliers, the hot path in one call:
 *   H = relu(dequant(dot'_int(quant_int(A), W1)) + b1),  Y = dequant(dot'_int(quant_int(H), W2)) + b2.
 * Every step is the one defined above (same quant_int, same sums, same fma), so Y
 * is bit-identical to the chain mq_absmax_f32 / mq_scale_from_amax /
 * mq_quantize_pack_f32 / mq_gemm_dequant_packed(out_amax) / ... -- but the float
 * intermediate H never goes to memory: the first product runs twice, once
 * reduced to max|H| and once re-quantized with the multiplier that maximum
 * gives, which is cheaper on this machine than writing and re-reading 4 M f bytes.
 * Five launches, no atomics, no host synchronisation.  When the intermediate
 * result is small enough for one tile per resident workgroup (M f <= 256 x 256 x
 * the number of compute units), the two passes become ONE launch:
 * the sums wait in registers while the grid agrees on max|H| (four launches).
 * mq_set_ffn_single_pass(0) switches that off (two passes always); results are
 * identical either way.
 *   A: device float [M x d], 16-byte aligned.  packedW1: 8-bit packed [f x d];
 *   packedW2: 8-bit packed [d x f]; sW1, sW2: their multipliers (device float[1]);
 *   b1: device float [f] or NULL; b2: device float [d] or NULL; Y: device float [M x d];
 *   ws: device, 256-byte aligned, mq_ffn_ws_bytes(M, d, f) bytes, contents
 *   irrelevant on entry, undefined on return. */
int mq_set_ffn_single_pass(int enable);
int mq_ffn_i8_f32(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
                  const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
                  void* ws, size_t ws_bytes, void* stream);

/* The same block for callers that run it again and again on one workspace (a decode loop, a captured graph).
 * The grid-wide agreements of the single-pass kernels need a few words of the workspace to be zero when a
 * kernel starts; mq_ffn_i8_f32 zeroes them with a small launch of its own on every call.  Here the caller
 * zeroes them ONCE with mq_ffn_ws_prepare and every mq_ffn_i8_f32_prepared call leaves them zero again (the
 * quantizing kernel and the first product clear each other's words on their way), which takes that launch out
 * of the block: three launches instead of four where the single-pass kernels apply.  Results are bit-identical
 * to mq_ffn_i8_f32.  Between prepare and the calls, and from call to call, the caller must not write to the
 * workspace or use it for anything else; sizes (M, d, f) must be those the workspace was prepared for; calls
 * sharing a workspace must not overlap (same rule as for mq_ffn_i8_f32).  After a call that failed, or whose
 * result carries the NaN of a timed-out agreement, prepare again.  mq_ffn_i8_f32 may be mixed in freely: it
 * also leaves the words zero.  Arguments as for mq_ffn_i8_f32; mq_ffn_ws_prepare: ws of at least
 * mq_ffn_ws_bytes(M, d, f) bytes, 256-byte aligned. */
int mq_ffn_ws_prepare(void* ws, size_t ws_bytes, size_t M, size_t d, size_t f, void* stream);
int mq_ffn_i8_f32_prepared(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
                           const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
                           void* ws, size_t ws_bytes, void* stream);

/* The same block in 16 bit (Transformer-big style): quant_int(A), product +
 * b1 + ReLU into a binary32 H kept in ws with max|H| as a by-product of the
 * epilogue, quant_int(H) straight into the packed layout with the multiplier
 * formed in that kernel, second product + b2.  (The input is read once where
 * it fits the one-kernel quantizer, see "Single-pass kernels" at the top.)  Five launches, no host
 * synchronisation; packedW1 / packedW2 from mq_prepare_weight(bits = 16).
 * Results are identical to the call-by-call chain.  Arguments as
 * mq_ffn_i8_f32; ws: mq_ffn_i16_ws_bytes(M, d, f) bytes (it holds H). */
size_t mq_ffn_i16_ws_bytes(size_t M, size_t d, size_t f);
int mq_ffn_i16_f32(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
                   const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
                   void* ws, size_t ws_bytes, void* stream);

/* The 16-bit block with multipliers fixed in advance, the paper's own 16-bit scheme (Section 4.2: every tensor
 * times 2^10, sums in 32 bits, so that no sum can wrap for the model's value range): quant_int(A, sA[0]), product +
 * b1 + ReLU re-quantized with sH[0] in the producing epilogue (saturating at +-32767; the intermediate goes to
 * memory once, as packed 16-bit values, never as floats), product + b2.  No abs-max pass anywhere.  Four launches.
 * sA, sH: device float[1] multipliers of the input and of the intermediate; packedW1 / packedW2 prepared with
 * bits = 16 and whatever multipliers sW1 / sW2 say (2^10 in the paper).  Results are those of
 * mq_quantize_pack_f32 + mq_gemm_requant_fixed_packed_i16 + mq_gemm_dequant_packed bit for bit.
 * ws: device, 256-byte aligned, mq_ffn_i16_fixed_ws_bytes(M, d, f) bytes, contents irrelevant. */
size_t mq_ffn_i16_fixed_ws_bytes(size_t M, size_t d, size_t f);
int mq_ffn_i16_fixed_f32(const float* A, size_t M, size_t d, size_t f, const float* sA, const void* packedW1,
                         const float* sW1, const float* b1, const float* sH, const void* packedW2, const float* sW2,
                         const float* b2, float* Y, void* ws, size_t ws_bytes, void* stream);

/* Output layer for beam search with beam size > 1 (Table 2, the b = 2 and b = 4
 * rows): for every row of the packed hidden states the k <= 4 most probable
 * words, best first (ties towards the lower vocabulary id), with
 * log p = y - log sum_n exp(y[n]),  y = (float) acc / (sA sW), the sum running
 * over all N words (or over the short list when one is given: ascending ids,
 * shortlist_len >= k; NULL = whole vocabulary).  The embedding streams through
 * the chip once per 256 rows; logits are never stored.  tok: int32 [M x k],
 * logprob: float [M x k].  Limits: K <= 512, N <= 1044480; MQ_ERR_UNSUPPORTED
 * beyond.  The words are exact (chosen on the integer sums); the log-
 * probabilities are binary32 (within 1e-4 of the binary64 value for logits of
 * magnitude up to ~100).  ws: device, 16-byte aligned, mq_topk_ws_bytes(M, N, k). */
size_t mq_topk_ws_bytes(size_t M, size_t N, int k);
int mq_gemm_topk_packed(const void* packedA, const void* packedW, const int32_t* shortlist_or_null,
                        size_t shortlist_len, size_t M, size_t N, size_t K, const float* sA, const float* sW,
                        int k, int32_t* tok, float* logprob, void* ws, size_t ws_bytes, void* stream);

/* ---- float glue of the averaging-attention decode step (Sections 3.1, 3.2) ----
 * Everything here is binary32 on device, row-major, caller-owned; each call is
 * one launch.  These are the operations between the integer products of a
 * decoder layer at one decode position. */

/* g = ((t - 1) g_prev + x) / t over n elements, t >= 1: the cumulative uniform
 * average over the decoder positions seen so far, from the last step only
 * (Section 3.2).  g may alias g_prev. */
int mq_running_average_f32(const float* g_prev, const float* x, size_t n, int t, float* g, void* stream);

/* out[m] = [a[m] ; b[m]] for M rows: a [M x da], b [M x db] -> out [M x (da + db)]
 * (the gate's input is the layer input next to the averaged path). */
int mq_concat2_f32(const float* a, size_t da, const float* b, size_t db, size_t M, float* out, void* stream);

/* y = LN(a + r) gamma + beta per row of width d <= 8192 with the biased
 * variance: residual connection + layer normalisation.  gamma, beta: [d]. */
int mq_add_layer_norm_f32(const float* a, const float* r, const float* gamma, const float* beta,
                          size_t M, size_t d, float eps, float* y, void* stream);

/* Gate of the averaging block and the normalisation after it, fused:
 * h = sigmoid(z[:, :d]) x + sigmoid(z[:, d:]) f,  y = LN(h + x) gamma + beta.
 * x, f: [M x d]; z: [M x 2d], the gate product's output on [x ; f]. */
int mq_gate_mix_layer_norm_f32(const float* x, const float* f, const float* z, const float* gamma,
                               const float* beta, size_t M, size_t d, float eps, float* y, void* stream);

/* Source attention of one query per sentence over that sentence's S source
 * positions: q [M x d], K, V [M x S x d] (precomputed), `heads` heads of width
 * d / heads: p = softmax_s(q_h . K_h[s] / sqrt(d / heads)), ctx_h = sum_s p[s] V_h[s].
 * heads * S <= 4096, d divisible by heads. */
int mq_cross_attention_f32(const float* q, const float* K, const float* V, size_t M, size_t S, size_t d,
                           int heads, float* ctx, void* stream);

/* One prepared 8-bit parameter product y = A . Wt^T + bias and one layer
 * normalisation, as plain device pointers. */
typedef struct mq_product {
  const void* packed;   /* mq_prepare_weight(bits = 8) of Wt [N x K] */
  const float* scale;   /* its multiplier, device float[1] */
  const float* bias;    /* device float[N], or NULL */
} mq_product;
typedef struct mq_norm {
  const float* gamma;   /* device float[d] */
  const float* beta;    /* device float[d] */
} mq_norm;
/* Parameters of one decoder layer (host struct, device pointers inside). */
typedef struct mq_aan_layer {
  mq_product aan_ffn1;  /* [aan_ffn x d], ReLU after it */
  mq_product aan_ffn2;  /* [d x aan_ffn] */
  mq_product aan_gate;  /* [2d x 2d] on [x ; f] */
  mq_norm ln1;
  mq_product ctx_q;     /* [d x d] query projection of the source attention */
  mq_product ctx_o;     /* [d x d] output projection */
  mq_norm ln2;
  mq_product ffn1;      /* [ffn x d], ReLU after it */
  mq_product ffn2;      /* [d x ffn] */
  mq_norm ln3;
  size_t d, ffn, aan_ffn;
} mq_aan_layer;

/* One decoder layer at decode position t for M sentences (all int8 products
 * with per-tensor abs-max multipliers, float glue in between):
 *   g   = running average of x                         -> g_out [M x d]
 *   f   = aan_ffn2(relu(aan_ffn1(g)))                  (use_ffn = 0: f = g)
 *   y1  = LN(gate(x, f, aan_gate([x ; f])) + x)        (use_gate = 0: LN(f + x))
 *   y2  = LN(ctx_o(attention(ctx_q(y1), K, V)) + y1)
 *   y   = LN(ffn2(relu(ffn1(y2))) + y2)                -> y [M x d]
 * use_ffn / use_gate = 0 give the "-ffn" / "-gate" variants of Table 2.
 * ws: device, 256-byte aligned, mq_aan_layer_ws_bytes bytes, contents irrelevant.
 * Only enqueues; y and g_out must not alias x or g_prev. */
size_t mq_aan_layer_ws_bytes(size_t M, size_t d, size_t ffn, size_t aan_ffn);
int mq_aan_layer_f32(const mq_aan_layer* P, const float* x, const float* g_prev, int t, const float* K,
                     const float* V, size_t M, size_t S, int heads, int use_ffn, int use_gate, float eps,
                     float* y, float* g_out, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MQ_H_ */
