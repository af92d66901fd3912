// Internal declarations shared by the library's translation units (not part of
// the C boundary, not used by the CPU oracle).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mq.h"

namespace mq {

constexpr int kWave = 64;          // wavefront width on gfx950
constexpr int kFragRows = 32;      // rows of Wt (or of A) per MFMA operand fragment
constexpr int kFragK = 32;         // contracted elements per v_mfma_i32_32x32x32_i8
constexpr int kFragBytes = 1024;   // 64 lanes x 16 bytes
constexpr int kKPad = 64;          // packed K is padded to this (two MFMA steps)

__host__ __device__ inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// Packed parameter geometry.  The quantized Wt [N x K] is cut into fragments of
// 32 rows x 32 contracted elements; fragment (nb, kb) holds, for lane l, the 16
// bytes Wt[32 nb + l % 32][32 kb + 16 (l / 32) + 0..15] at byte offset 16 l.
// Fragments of one row block follow each other along K, row blocks follow each
// other.  16-bit parameters store two byte planes per fragment (high byte, then
// low byte with its top bit flipped) and append sum_k Wt[n][k] as int32 [Np].
// Rows n >= N and elements k >= K are zero bytes in every plane.
struct PackedDims {
  size_t Np, Kp, nblocks, kfrags;
  int planes;
  __host__ __device__ PackedDims(int bits, size_t N, size_t K)
      : Np(round_up(N, kFragRows)), Kp(round_up(K, kKPad)), nblocks(Np / kFragRows),
        kfrags(Kp / kFragK), planes(bits == 16 ? 2 : 1) {}
  __host__ __device__ size_t frag_offset(size_t nb, size_t kb) const {
    return (nb * kfrags + kb) * (size_t)kFragBytes * planes;
  }
  __host__ __device__ size_t plane_bytes() const { return Np * Kp * planes; }
  __host__ __device__ size_t total_bytes() const {
    return plane_bytes() + (planes == 2 ? Np * sizeof(int32_t) : 0);
  }
};

// Records a HIP error for mq_last_hip_error and maps it to a status.
int check_hip(hipError_t e);

inline int qmax_of(int bits) { return bits == 8 ? 127 : (bits == 16 ? 32767 : 0); }

// Kernel launchers (each enqueues on `s` and returns an mq_status).
int launch_absmax(const float* x, size_t n, float* amax, hipStream_t s);
int launch_scale(const float* amax, int bits, float* scale, hipStream_t s);
int launch_quantize(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                    void* q, int32_t* rowsum, hipStream_t s);
int launch_prepare(const float* B, int transposed, size_t N, size_t K, int bits,
                   const float* scale, void* packed, hipStream_t s);
int launch_unpack(const void* packed, int bits, size_t N, size_t K, void* q, hipStream_t s);

enum Epilogue { kEpiRaw = 0, kEpiDequant = 1, kEpiArgmax = 2 };

struct GemmArgs {
  const void* qA;
  const int32_t* rowsumA;
  const void* packedW;
  int bits;
  size_t M, N, K;
  // raw
  int32_t* C;
  // dequant
  const float* sA;
  const float* sW;
  const float* bias;
  int relu;
  float* Y;
  float* out_amax;
  // argmax
  unsigned long long* keys;  // [M] packed (sum, ~index) maxima
  // fused FFN passes
  float* partial;
  unsigned npartial;
  float* s_out;
  void* packed_out;
  unsigned* barrier;
  // single-pass product only: words (of some OTHER kernel's grid-wide agreement) that workgroup 0 zeroes at its start
  unsigned* clear_words;
  unsigned nclear;
  // dequantizing epilogue of the packed tiled products: out_amax points to this many words (cleared by the caller),
  // workgroups spread their atomic maxima over them; the consumer takes the maximum of all.  0 = one word.
  unsigned amax_slots;
};
int launch_gemm(const GemmArgs& a, Epilogue epi, hipStream_t s);
void set_forced_variant(int v);
int forced_variant();
// Both operands packed (activations from launch_quantize_pack); a.qA is the packed activation buffer.
int launch_gemm_packed(const GemmArgs& a, Epilogue epi, hipStream_t s);
// Split-K form for few rows (8 bit, raw or dequantizing epilogue); launch_gemm_packed's variant 10.
int launch_gemm_small(const GemmArgs& a, Epilogue epi, hipStream_t s);
// With the dequantizing epilogue both small-product launchers also write max|y| of every workgroup to
// a.partial (if not NULL): gemm_small_partials / gemm_small_f32_partials values.
size_t gemm_small_partials(size_t M, size_t N, size_t K);
size_t gemm_small_f32_partials(size_t M, size_t N, size_t K);
// The same with quant_int of fp32 activations done in the operand fetch (8 bit, dequantizing epilogue):
// `scale` is the multiplier (npartial == 0) or npartial partial maxima of |A|; a.qA, a.sA are not used.
bool gemm_small_f32_supported(size_t M, size_t N, size_t K);
int launch_gemm_small_f32(const float* A, const float* scale, unsigned npartial, float* scale_out, const GemmArgs& a,
                          hipStream_t s);
// The same for an input given as two row-major pieces side by side, [A1 (K1 columns) | A2 (a.K - K1 columns)], each with
// partial maxima of its own (n1, n2 >= 1): the concatenation is never stored.  K1 must be a multiple of 4.
int launch_gemm_small_f32_pair(const float* A1, size_t K1, const float* part1, unsigned n1, const float* A2,
                               const float* part2, unsigned n2, float* scale_out, const GemmArgs& a, hipStream_t s);
int launch_quantize_pack(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                         void* packed, hipStream_t s);
int launch_argmax_init(unsigned long long* keys, size_t M, hipStream_t s);
int launch_argmax_finish(const unsigned long long* keys, size_t M, const float* sA, const float* sW,
                         int32_t* tok, float* maxlogit, hipStream_t s);

constexpr unsigned kAbsmaxPartials = 1024;   // floats of scratch launch_absmax_quantize_pack needs
int launch_absmax_quantize_pack(const float* x, size_t rows, size_t cols, int bits, float* partials,
                                float* scale_out, void* packed, hipStream_t s, unsigned* clear = nullptr,
                                unsigned nclear = 0);
int launch_absmax_partials(const float* x, size_t n, float* partials, unsigned* count, hipStream_t s);
// clear_words / nclear (optional): words of another kernel's agreement that workgroup 0 zeroes at its start.
// self_clean: the kernel leaves its own kBarrierWords words at `barrier` all zero (the last workgroup done zeroes them).
int launch_absmax_quantize_pack_fused(const float* x, size_t rows, size_t cols, int bits, unsigned* barrier,
                                      float* scale_out, void* packed, hipStream_t s, unsigned* clear_words = nullptr,
                                      unsigned nclear = 0, int self_clean = 0);
int launch_quantize_pack_partials(const float* x, size_t rows, size_t cols, int bits, const float* partials,
                                  unsigned npartials, float* scale_out, void* packed, hipStream_t s);
// Fused FFN pieces (8 bit): product + bias + ReLU reduced to per-tile abs-max partials, and the same
// product re-quantized with the multiplier formed from those partials, written as packed activations.
size_t gemm_amax_partials(size_t M, size_t N);
int launch_gemm_amax_partial(const GemmArgs& a, float* partials, hipStream_t s);
int launch_gemm_requant(const GemmArgs& a, const float* partials, float* s_out, void* packed_out, hipStream_t s);
// Words of the grid-wide barrier of the single-pass kernels: eight copies of one slot per workgroup
// (at most 256) and a sticky failure word, rounded up.
constexpr unsigned kBarrierWords = 8 * 256 + 64;
// Size test of the single-pass re-quantizing product: one 256 x 256 tile per workgroup, every workgroup resident
// on an otherwise empty device (`resident` = occupancy x compute units) and holding one of the 256 slots.
inline bool single_pass_fits(size_t M, size_t N, size_t resident) {
  if (M == 0 || N == 0) return false;
  const size_t tiles = ((M + 255) / 256) * ((N + 255) / 256);
  return tiles <= resident && tiles <= 256;
}
unsigned long long barrier_timeout_ticks();
void set_barrier_timeout_ticks(unsigned long long ticks);
size_t topk_stream_ws_bytes(size_t M, int k);
bool topk_stream_supported(size_t M, size_t N, size_t K, int k);
int launch_topk_stream(const void* packedA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                       const float* sW, int k, int32_t* tok, float* logprob, void* ws, const int32_t* shortlist,
                       size_t shortlist_len, hipStream_t s);
// float glue of the averaging-attention decode step (mq_glue.hip).  `partial` (optional) receives one
// max|output| per workgroup: running_average_partials(n) of them for the running average, M for the others.
size_t running_average_partials(size_t n);
int launch_running_average(const float* g_prev, const float* x, size_t n, int t, float* g, hipStream_t s,
                           float* partial = nullptr, unsigned* clear = nullptr, unsigned nclear = 0,
                           float* partial_x = nullptr);     // partial_x: the same number of maxima of |x|
int launch_concat2(const float* a, size_t da, const float* b, size_t db, size_t M, float* out, hipStream_t s,
                   float* partial = nullptr);
int launch_add_layer_norm(const float* a, const float* r, const float* gamma, const float* beta, size_t M, size_t d,
                          float eps, float* y, hipStream_t s, float* partial = nullptr);
int launch_gate_mix_layer_norm(const float* x, const float* f, const float* z, const float* gamma, const float* beta,
                               size_t M, size_t d, float eps, float* y, hipStream_t s, float* partial = nullptr);
int launch_cross_attention(const float* q, const float* K, const float* V, size_t M, size_t S, size_t d, int heads,
                           float* ctx, hipStream_t s, float* partial = nullptr);
int launch_clear_words(unsigned* p, unsigned n, hipStream_t s);
int launch_fill_pattern(void* p, size_t bytes, unsigned seed, hipStream_t s);     // pseudo-random bytes (timing runs)
int launch_gemm_requant_coop(const GemmArgs& a, float* s_out, void* packed_out, unsigned* barrier,
                             hipStream_t s);
int launch_gemm_requant_fixed(const GemmArgs& a, const float* s_fixed, void* packed_out, hipStream_t s);
int launch_gemm_requant_fixed_i16(const GemmArgs& a, const float* s_fixed, void* packed_out, hipStream_t s);
// Tiled 8-bit product with two extra waves per workgroup that only load (mq_gemm_prod.hip); variants 11 .. 13.
int launch_gemm_prod(const GemmArgs& a, Epilogue epi, int which, hipStream_t s);
// Variant 14 of the packed 8-bit products (mq_gemm_ks.hip): 128 x 128 tile, K split over two groups of four waves.
int launch_gemm_ks(const GemmArgs& a, Epilogue epi, hipStream_t s);
// 16-bit product on the vector ALU (v_dot2c_i32_i16), both operands packed; variant 7 of the packed 16-bit products.
int launch_gemm_dot2(const GemmArgs& a, Epilogue epi, hipStream_t s);
// 16-bit product with one workgroup per compute unit that walks through its tiles, loading across tile boundaries
// (mq_gemm_pers.hip); variant 8 of the packed 16-bit products.  MQ_ERR_UNSUPPORTED for K up to 64 (a single K step).
int launch_gemm_pers16(const GemmArgs& a, Epilogue epi, hipStream_t s);
// Auto-tuner table (shape + operand width -> tile variant of the packed kernels); 0 = not tuned.
int tuned_variant(int bits, size_t M, size_t N, size_t K);
void set_tuned_variant(int bits, size_t M, size_t N, size_t K, int variant);
int packed_variant_count(int bits);

// Streaming arg-max product for decode-sized batches (both operands packed, 8 bit).
size_t argmax_stream_ws_bytes(size_t M);
bool argmax_stream_supported(size_t M, size_t N, size_t K);
// max_grid: columns of the partials array at ws (0 = as many as argmax_stream_ws_bytes provides).
int launch_argmax_stream(const void* packedA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                         const float* sW, int32_t* tok, float* maxlogit, void* ws, const int32_t* shortlist,
                         size_t shortlist_len, hipStream_t s, unsigned max_grid = 0);
// The same with the partial winners in a static device array of the library (no workspace, no allocation).
size_t argmax_static_max_rows();
int launch_argmax_stream_static(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                const float* sA, const float* sW, int32_t* tok, float* maxlogit, hipStream_t s);

}  // namespace mq
