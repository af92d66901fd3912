// C boundary: argument checks, then launches.  Nothing here computes.
#include "mq_internal.h"

namespace mq {

static thread_local int g_last_hip_error = 0;

int check_hip(hipError_t e) {
  if (e == hipSuccess) return MQ_OK;
  g_last_hip_error = (int)e;
  return MQ_ERR_HIP;
}

// ---- auto-tuner table (arxiv 1805.12096, Section 4.4: hash shapes and algorithm ids, time the
// alternatives, keep the fastest for all following calls) ---------------------------------------
namespace {
struct TunedEntry { int bits; size_t M, N, K; int variant; };
constexpr int kTunedSlots = 256;
TunedEntry g_tuned[kTunedSlots];
int g_tuned_count = 0;
}  // namespace

int tuned_variant(int bits, size_t M, size_t N, size_t K) {
  for (int i = 0; i < g_tuned_count; ++i)
    if (g_tuned[i].bits == bits && g_tuned[i].M == M && g_tuned[i].N == N && g_tuned[i].K == K) return g_tuned[i].variant;
  return 0;
}

void set_tuned_variant(int bits, size_t M, size_t N, size_t K, int variant) {
  for (int i = 0; i < g_tuned_count; ++i)
    if (g_tuned[i].bits == bits && g_tuned[i].M == M && g_tuned[i].N == N && g_tuned[i].K == K) {
      g_tuned[i].variant = variant;
      return;
    }
  if (g_tuned_count < kTunedSlots) g_tuned[g_tuned_count++] = TunedEntry{bits, M, N, K, variant};
}

namespace {

constexpr size_t kMaxElems = (size_t)1 << 40;
constexpr size_t kMaxDim = (size_t)1 << 31;

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
bool bits_ok(int bits) { return bits == 8 || bits == 16; }
bool dims_ok(size_t M, size_t N, size_t K) {
  if (M == 0 || N == 0 || K == 0) return false;
  if (M >= kMaxDim || N >= kMaxDim || K >= kMaxDim) return false;
  if (M > kMaxElems / K || N > kMaxElems / K || M > kMaxElems / N) return false;
  return true;
}
hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// Layout of the scratch area used by mq_linear_f32 / mq_gemm_argmax.
struct LinearWs {
  size_t off_scale, off_q, off_part, total;
  LinearWs(int bits, size_t M, size_t K) {
    off_scale = 0;                       // float multiplier
    off_q = 256;                         // packed quantized activations
    off_part = off_q + round_up(PackedDims(bits, M, K).total_bytes(), 256);     // partial maxima
    total = off_part + kAbsmaxPartials * sizeof(float);
  }
};

int gemm_common_checks(const void* qA, const int32_t* rowsumA, const void* packedW, int bits,
                       size_t M, size_t N, size_t K) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (qA == nullptr || packedW == nullptr) return MQ_ERR_NULL;
  if (bits == 16 && rowsumA == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(qA, 16) || !aligned(packedW, 16)) return MQ_ERR_ALIGN;
  if (rowsumA != nullptr && !aligned(rowsumA, 4)) return MQ_ERR_ALIGN;
  return MQ_OK;
}

}  // namespace
}  // namespace mq

using namespace mq;

extern "C" {

int mq_version(void) { return 100; }

const char* mq_status_string(int status) {
  switch (status) {
    case MQ_OK: return "ok";
    case MQ_ERR_NULL: return "a required pointer is NULL";
    case MQ_ERR_SHAPE: return "a size is zero or too large";
    case MQ_ERR_DTYPE: return "bits must be 8 or 16 (8 only for the arg-max product)";
    case MQ_ERR_ALIGN: return "a pointer is not aligned as required";
    case MQ_ERR_WORKSPACE: return "workspace too small";
    case MQ_ERR_UNSUPPORTED: return "unsupported arguments";
    case MQ_ERR_HIP: return "HIP runtime error (see mq_last_hip_error)";
    case MQ_ERR_LIMIT: return "a size is beyond what the library's static scratch array serves";
    default: return "unknown status";
  }
}

int mq_last_hip_error(void) { return g_last_hip_error; }

int mq_set_gemm_variant(int variant) {
  if (variant < 0 || variant > 16) return MQ_ERR_UNSUPPORTED;
  set_forced_variant(variant);
  return MQ_OK;
}

int mq_absmax_f32(const float* x, size_t n, float* amax, void* stream) {
  if (x == nullptr || amax == nullptr) return MQ_ERR_NULL;
  if (n == 0 || n > kMaxElems) return MQ_ERR_SHAPE;
  if (!aligned(x, 16) || !aligned(amax, 4)) return MQ_ERR_ALIGN;
  return launch_absmax(x, n, amax, as_stream(stream));
}

int mq_scale_from_amax(const float* amax, int bits, float* scale, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (amax == nullptr || scale == nullptr) return MQ_ERR_NULL;
  if (!aligned(amax, 4) || !aligned(scale, 4)) return MQ_ERR_ALIGN;
  return launch_scale(amax, bits, scale, as_stream(stream));
}

int mq_quantize_f32(const float* x, size_t rows, size_t cols, int bits, const float* scale, void* q,
                    int32_t* rowsum, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (x == nullptr || scale == nullptr || q == nullptr) return MQ_ERR_NULL;
  if (rows == 0 || cols == 0 || rows >= kMaxDim || cols >= kMaxDim || rows > kMaxElems / cols)
    return MQ_ERR_SHAPE;
  if (!aligned(x, 16) || !aligned(q, 16) || !aligned(scale, 4)) return MQ_ERR_ALIGN;
  if (rowsum != nullptr && !aligned(rowsum, 4)) return MQ_ERR_ALIGN;
  return launch_quantize(x, rows, cols, bits, scale, q, rowsum, as_stream(stream));
}

int mq_quantize_pack_f32(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                         void* packed, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (x == nullptr || scale == nullptr || packed == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(1, rows, cols)) return MQ_ERR_SHAPE;
  if (!aligned(x, 16) || !aligned(packed, 16) || !aligned(scale, 4)) return MQ_ERR_ALIGN;
  return launch_quantize_pack(x, rows, cols, bits, scale, packed, as_stream(stream));
}

static int g_quantize_single_pass = 1;

int mq_set_quantize_single_pass(int enable) {
  g_quantize_single_pass = enable < 0 ? 0 : (enable > 2 ? 2 : enable);
  return MQ_OK;
}

size_t mq_quantize_absmax_ws_bytes(void) {      // agreement words, then partial maxima: one workspace serves every form
  return round_up(kBarrierWords * sizeof(unsigned), 256) + kAbsmaxPartials * sizeof(float);
}

int mq_quantize_absmax_ws_prepare(void* ws, size_t ws_bytes, void* stream) {
  if (ws == nullptr) return MQ_ERR_NULL;
  if (!aligned(ws, 16)) return MQ_ERR_ALIGN;
  if (ws_bytes < mq_quantize_absmax_ws_bytes()) return MQ_ERR_WORKSPACE;
  return launch_clear_words(static_cast<unsigned*>(ws), kBarrierWords, as_stream(stream));
}

int mq_quantize_absmax_pack_f32_prepared(const float* x, size_t rows, size_t cols, int bits, void* packed,
                                         float* scale_out, void* ws, size_t ws_bytes, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (x == nullptr || scale_out == nullptr || packed == nullptr || ws == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(1, rows, cols)) return MQ_ERR_SHAPE;
  if (!aligned(x, 16) || !aligned(packed, 16) || !aligned(scale_out, 4) || !aligned(ws, 16)) return MQ_ERR_ALIGN;
  if (ws_bytes < mq_quantize_absmax_ws_bytes()) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  // Whatever fits the registers of one resident grid takes the kernel that reads x once; it finds its agreement
  // words zero and leaves them zero.  Without a clearing launch in front of it that kernel also wins for small
  // tensors, where the plain entry point prefers two tiny kernels.
  if (g_quantize_single_pass != 0) {
    const int rc = launch_absmax_quantize_pack_fused(x, rows, cols, bits, static_cast<unsigned*>(ws), scale_out, packed,
                                                     s, nullptr, 0, 1);
    if (rc != MQ_ERR_UNSUPPORTED) return rc;
  }
  float* partials = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + round_up(kBarrierWords * sizeof(unsigned), 256));
  return launch_absmax_quantize_pack(x, rows, cols, bits, partials, scale_out, packed, s);
}

int mq_quantize_absmax_pack_f32(const float* x, size_t rows, size_t cols, int bits, void* packed,
                                float* scale_out, void* ws, size_t ws_bytes, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (x == nullptr || scale_out == nullptr || packed == nullptr || ws == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(1, rows, cols)) return MQ_ERR_SHAPE;
  if (!aligned(x, 16) || !aligned(packed, 16) || !aligned(scale_out, 4) || !aligned(ws, 16)) return MQ_ERR_ALIGN;
  if (ws_bytes < mq_quantize_absmax_ws_bytes()) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  // (below a million elements two tiny kernels are quicker than one with a grid-wide wait)
  if (g_quantize_single_pass != 0 && (g_quantize_single_pass > 1 || rows * cols >= ((size_t)1 << 20))) {
    // small enough for the registers of one resident grid: clear the agreement words, then one kernel
    // that reads x once; larger tensors take the two-pass form below
    int rc = launch_clear_words(static_cast<unsigned*>(ws), kBarrierWords, s);
    if (rc != MQ_OK) return rc;
    // (self-cleaning like the prepared form: a prepared workspace handed to this entry point stays prepared)
    rc = launch_absmax_quantize_pack_fused(x, rows, cols, bits, static_cast<unsigned*>(ws), scale_out, packed, s, nullptr,
                                           0, 1);
    if (rc != MQ_ERR_UNSUPPORTED) return rc;
  }
  // the partial maxima live behind the agreement words, as in the prepared form: this path never touches those
  float* partials = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + round_up(kBarrierWords * sizeof(unsigned), 256));
  return launch_absmax_quantize_pack(x, rows, cols, bits, partials, scale_out, packed, s);
}

size_t mq_packed_bytes(int bits, size_t N, size_t K) {
  if (!bits_ok(bits) || N == 0 || K == 0 || N >= kMaxDim || K >= kMaxDim) return 0;
  return PackedDims(bits, N, K).total_bytes();
}

int mq_prepare_weight(const float* B, int b_is_transposed, size_t N, size_t K, int bits,
                      const float* scale_or_null, float* scale_out, void* packed, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (B == nullptr || scale_out == nullptr || packed == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(1, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(B, 16) || !aligned(packed, 16) || !aligned(scale_out, 4)) return MQ_ERR_ALIGN;
  if (scale_or_null != nullptr && !aligned(scale_or_null, 4)) return MQ_ERR_ALIGN;
  hipStream_t s = as_stream(stream);
  if (scale_or_null == nullptr) {
    int rc = launch_absmax(B, N * K, scale_out, s);
    if (rc != MQ_OK) return rc;
    rc = launch_scale(scale_out, bits, scale_out, s);
    if (rc != MQ_OK) return rc;
  } else if (scale_or_null != scale_out) {
    int rc = check_hip(hipMemcpyAsync(scale_out, scale_or_null, sizeof(float), hipMemcpyDeviceToDevice, s));
    if (rc != MQ_OK) return rc;
  }
  return launch_prepare(B, b_is_transposed != 0, N, K, bits, scale_out, packed, s);
}

int mq_unpack_weight(const void* packed, int bits, size_t N, size_t K, void* q_out, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (packed == nullptr || q_out == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(1, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packed, 16) || !aligned(q_out, 2)) return MQ_ERR_ALIGN;
  return launch_unpack(packed, bits, N, K, q_out, as_stream(stream));
}

int mq_gemm_i32(const void* qA, const int32_t* rowsumA, const void* packedW, int bits, size_t M,
                size_t N, size_t K, int32_t* C, void* stream) {
  int rc = gemm_common_checks(qA, rowsumA, packedW, bits, M, N, K);
  if (rc != MQ_OK) return rc;
  if (C == nullptr) return MQ_ERR_NULL;
  if (!aligned(C, 4)) return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = qA; a.rowsumA = rowsumA; a.packedW = packedW; a.bits = bits; a.M = M; a.N = N; a.K = K; a.C = C;
  return launch_gemm(a, kEpiRaw, as_stream(stream));
}

int mq_gemm_dequant(const void* qA, const int32_t* rowsumA, const void* packedW, int bits, size_t M,
                    size_t N, size_t K, const float* sA, const float* sW, const float* bias, int relu,
                    float* Y, float* out_amax, void* stream) {
  int rc = gemm_common_checks(qA, rowsumA, packedW, bits, M, N, K);
  if (rc != MQ_OK) return rc;
  if (sA == nullptr || sW == nullptr || Y == nullptr) return MQ_ERR_NULL;
  if (!aligned(sA, 4) || !aligned(sW, 4) || !aligned(Y, 4)) return MQ_ERR_ALIGN;
  if ((bias != nullptr && !aligned(bias, 4)) || (out_amax != nullptr && !aligned(out_amax, 4)))
    return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = qA; a.rowsumA = rowsumA; a.packedW = packedW; a.bits = bits; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0; a.Y = Y; a.out_amax = out_amax;
  return launch_gemm(a, kEpiDequant, as_stream(stream));
}

int mq_gemm_i32_packed(const void* packedA, const void* packedW, int bits, size_t M, size_t N, size_t K,
                       int32_t* C, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (packedA == nullptr || packedW == nullptr || C == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(C, 4)) return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = bits; a.M = M; a.N = N; a.K = K; a.C = C;
  return launch_gemm_packed(a, kEpiRaw, as_stream(stream));
}

int mq_gemm_dequant_packed(const void* packedA, const void* packedW, int bits, size_t M, size_t N, size_t K,
                           const float* sA, const float* sW, const float* bias, int relu, float* Y,
                           float* out_amax, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || Y == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(Y, 4))
    return MQ_ERR_ALIGN;
  if ((bias != nullptr && !aligned(bias, 4)) || (out_amax != nullptr && !aligned(out_amax, 4)))
    return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = bits; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0; a.Y = Y; a.out_amax = out_amax;
  return launch_gemm_packed(a, kEpiDequant, as_stream(stream));
}

size_t mq_gemm_amax_ws_bytes(size_t M, size_t N) {
  if (M == 0 || N == 0 || M >= kMaxDim || N >= kMaxDim) return 0;
  // room for the two-pass partial maxima or for the single-pass barrier words, whichever is larger
  const size_t partials = round_up(gemm_amax_partials(M, N) * sizeof(float), 256);
  const size_t barrier = round_up(kBarrierWords * sizeof(unsigned), 256);
  return partials > barrier ? partials : barrier;
}

namespace {
int fused_pass_checks(const void* packedA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                      const float* sW, const float* bias, const void* ws, size_t ws_bytes) {
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || ws == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(ws, 16))
    return MQ_ERR_ALIGN;
  if (bias != nullptr && !aligned(bias, 4)) return MQ_ERR_ALIGN;
  if (ws_bytes < mq_gemm_amax_ws_bytes(M, N)) return MQ_ERR_WORKSPACE;
  return MQ_OK;
}
}  // namespace

int mq_gemm_amax_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                        const float* sW, const float* bias, int relu, void* ws, size_t ws_bytes, void* stream) {
  int rc = fused_pass_checks(packedA, packedW, M, N, K, sA, sW, bias, ws, ws_bytes);
  if (rc != MQ_OK) return rc;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = 8; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0;
  return launch_gemm_amax_partial(a, static_cast<float*>(ws), as_stream(stream));
}

int mq_gemm_requant_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                           const float* sA, const float* sW, const float* bias, int relu, const void* ws,
                           size_t ws_bytes, float* scale_out, void* packed_out, void* stream) {
  int rc = fused_pass_checks(packedA, packedW, M, N, K, sA, sW, bias, ws, ws_bytes);
  if (rc != MQ_OK) return rc;
  if (scale_out == nullptr || packed_out == nullptr) return MQ_ERR_NULL;
  if (!aligned(scale_out, 4) || !aligned(packed_out, 16)) return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = 8; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0;
  return launch_gemm_requant(a, static_cast<const float*>(ws), scale_out, packed_out, as_stream(stream));
}

int mq_single_pass_fits(size_t M, size_t N, size_t resident) {
  return single_pass_fits(M, N, resident) ? 1 : 0;
}

int mq_gemm_requant_single_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                  const float* sA, const float* sW, const float* bias, int relu, void* ws,
                                  size_t ws_bytes, float* scale_out, void* packed_out, void* stream) {
  int rc = fused_pass_checks(packedA, packedW, M, N, K, sA, sW, bias, ws, ws_bytes);
  if (rc != MQ_OK) return rc;
  if (scale_out == nullptr || packed_out == nullptr) return MQ_ERR_NULL;
  if (!aligned(scale_out, 4) || !aligned(packed_out, 16)) return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = 8; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0;
  unsigned* barrier = static_cast<unsigned*>(ws);
  rc = launch_clear_words(barrier, kBarrierWords, as_stream(stream));
  if (rc != MQ_OK) return rc;
  return launch_gemm_requant_coop(a, scale_out, packed_out, barrier, as_stream(stream));
}

int mq_gemm_requant_fixed_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                 const float* sA, const float* sW, const float* bias, int relu,
                                 const float* s_out, void* packed_out, void* stream) {
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || s_out == nullptr ||
      packed_out == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(s_out, 4) ||
      !aligned(packed_out, 16))
    return MQ_ERR_ALIGN;
  if (bias != nullptr && !aligned(bias, 4)) return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = 8; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0;
  return launch_gemm_requant_fixed(a, s_out, packed_out, as_stream(stream));
}

int mq_gemm_requant_fixed_packed_i16(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                     const float* sA, const float* sW, const float* bias, int relu,
                                     const float* s_out, void* packed_out, void* stream) {
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || s_out == nullptr ||
      packed_out == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(s_out, 4) ||
      !aligned(packed_out, 16))
    return MQ_ERR_ALIGN;
  if (bias != nullptr && !aligned(bias, 4)) return MQ_ERR_ALIGN;
  GemmArgs a{};
  a.qA = packedA; a.packedW = packedW; a.bits = 16; a.M = M; a.N = N; a.K = K;
  a.sA = sA; a.sW = sW; a.bias = bias; a.relu = relu != 0;
  return launch_gemm_requant_fixed_i16(a, s_out, packed_out, as_stream(stream));
}

// times of the last mq_autotune_gemm run, microseconds per launch by variant (index 0 unused; < 0: not available)
static float g_autotune_us[32];
static int g_autotune_count = 0;

int mq_autotune_report(float* us_by_variant, int n) {
  if (us_by_variant == nullptr) return MQ_ERR_NULL;
  if (n <= 0) return MQ_ERR_SHAPE;
  for (int v = 0; v < n; ++v) us_by_variant[v] = (v < g_autotune_count && v < 32) ? g_autotune_us[v] : -1.0f;
  return MQ_OK;
}

size_t mq_autotune_ws_bytes(int bits, size_t M, size_t N, size_t K) {
  if (!bits_ok(bits) || !dims_ok(M, N, K)) return 0;
  return round_up(PackedDims(bits, M, K).total_bytes(), 256) + round_up(PackedDims(bits, N, K).total_bytes(), 256) +
         round_up(M * N * sizeof(float), 256) + 256;
}

int mq_autotune_gemm(int bits, size_t M, size_t N, size_t K, int runs, void* ws, size_t ws_bytes, void* stream,
                     int* best_variant, float* best_us) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (ws == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, N, K) || runs <= 0) return MQ_ERR_SHAPE;
  if (!aligned(ws, 256)) return MQ_ERR_ALIGN;
  if (ws_bytes < mq_autotune_ws_bytes(bits, M, N, K)) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  uint8_t* base = static_cast<uint8_t*>(ws);
  const size_t a_bytes = round_up(PackedDims(bits, M, K).total_bytes(), 256);
  const size_t w_bytes = round_up(PackedDims(bits, N, K).total_bytes(), 256);
  void* pa = base;
  void* pw = base + a_bytes;
  float* Y = reinterpret_cast<float*>(base + a_bytes + w_bytes);
  float* scal = reinterpret_cast<float*>(base + a_bytes + w_bytes + round_up(M * N * sizeof(float), 256));
  // operand bytes only need to be valid memory; pseudo-random ones make the matrix units draw the power (and
  // hold the clock) they do on real data, which constant bytes do not; unit multipliers
  int rc = launch_fill_pattern(pa, a_bytes, 0x35u, s);
  if (rc == MQ_OK) rc = launch_fill_pattern(pw, w_bytes, 0xC7u, s);
  const float ones[2] = {1.0f, 1.0f};
  if (rc == MQ_OK) rc = check_hip(hipMemcpyAsync(scal, ones, sizeof ones, hipMemcpyHostToDevice, s));
  if (rc != MQ_OK) return rc;
  hipEvent_t e0, e1;
  if (check_hip(hipEventCreate(&e0)) != MQ_OK) return MQ_ERR_HIP;
  if (check_hip(hipEventCreate(&e1)) != MQ_OK) {
    (void)hipEventDestroy(e0);
    return MQ_ERR_HIP;
  }
  GemmArgs a{};
  a.qA = pa; a.packedW = pw; a.bits = bits; a.M = M; a.N = N; a.K = K;
  a.sA = scal; a.sW = scal + 1; a.relu = 0; a.Y = Y;
  const int saved = forced_variant();
  // `runs` timed launches of variant v (after one untimed: code upload, attribute set-up)
  auto time_variant = [&](int v, float* ms) -> int {
    set_forced_variant(v);
    int r = launch_gemm_packed(a, kEpiDequant, s);
    if (r != MQ_OK) return r;
    r = check_hip(hipEventRecord(e0, s));
    for (int i = 0; i < runs && r == MQ_OK; ++i) r = launch_gemm_packed(a, kEpiDequant, s);
    if (r == MQ_OK) r = check_hip(hipEventRecord(e1, s));
    if (r != MQ_OK) return r;
    if (check_hip(hipEventSynchronize(e1)) != MQ_OK) return MQ_ERR_HIP;
    return check_hip(hipEventElapsedTime(ms, e0, e1));
  };
  const int nv = packed_variant_count(bits);
  float best_of[32];
  for (int v = 0; v < 32; ++v) best_of[v] = -1.0f;
  // A device that has been idle runs its first tens of milliseconds below its working clock, which would favour
  // whatever is timed last: the first variant that exists runs untimed for about 30 ms first, and every variant is
  // timed in two rounds, of which the faster counts.
  for (int v = 1; v <= nv && rc == MQ_OK; ++v) {
    float ms = 0.f, spun = 0.f;
    int r = time_variant(v, &ms);
    if (r == MQ_ERR_UNSUPPORTED) continue;
    rc = r;
    for (int guard = 0; rc == MQ_OK && spun < 30.0f && guard < 4096; ++guard) {
      rc = time_variant(v, &ms);
      spun += ms > 0.f ? ms : 0.01f;
    }
    break;
  }
  for (int round = 0; round < 2 && rc == MQ_OK; ++round) {
    for (int v = 1; v <= nv && v < 32; ++v) {
      float ms = 0.f;
      const int r = time_variant(v, &ms);
      if (r == MQ_ERR_UNSUPPORTED) continue;
      if (r != MQ_OK) { rc = r; break; }
      if (best_of[v] < 0.f || ms < best_of[v]) best_of[v] = ms;
    }
  }
  int best = 0;
  float best_ms = 0.f;
  for (int v = 1; v <= nv && v < 32; ++v)
    if (best_of[v] >= 0.f && (best == 0 || best_of[v] < best_ms)) { best = v; best_ms = best_of[v]; }
  g_autotune_count = nv + 1 < 32 ? nv + 1 : 32;
  for (int v = 0; v < 32; ++v) g_autotune_us[v] = best_of[v] >= 0.f ? best_of[v] * 1000.0f / (float)runs : -1.0f;
  set_forced_variant(saved);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != MQ_OK && rc != MQ_ERR_UNSUPPORTED) return rc;
  if (best == 0) return MQ_ERR_UNSUPPORTED;
  set_tuned_variant(bits, M, N, K, best);
  if (best_variant != nullptr) *best_variant = best;
  if (best_us != nullptr) *best_us = best_ms * 1000.0f / (float)runs;
  return MQ_OK;
}

size_t mq_argmax_ws_bytes(size_t M, size_t N) {
  if (M == 0 || N == 0 || M >= kMaxDim || N >= kMaxDim) return 0;
  const size_t general = round_up(M * sizeof(unsigned long long), 256);
  const size_t stream = argmax_stream_ws_bytes(M);
  return general > stream ? general : stream;
}

int mq_gemm_argmax_packed(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                          const float* sA, const float* sW, int32_t* tok, float* maxlogit, void* ws,
                          size_t ws_bytes, void* stream) {
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || tok == nullptr ||
      maxlogit == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(tok, 4) ||
      !aligned(maxlogit, 4) || !aligned(ws, 16))
    return MQ_ERR_ALIGN;
  if (ws_bytes < mq_argmax_ws_bytes(M, N)) return MQ_ERR_WORKSPACE;
  if (!argmax_stream_supported(M, N, K)) return MQ_ERR_UNSUPPORTED;
  return launch_argmax_stream(packedA, packedW, M, N, K, sA, sW, tok, maxlogit, ws, nullptr, 0, as_stream(stream));
}

int mq_gemm_argmax_packed_static(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                 const float* sA, const float* sW, int32_t* tok, float* maxlogit, void* stream) {
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || tok == nullptr ||
      maxlogit == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(tok, 4) ||
      !aligned(maxlogit, 4))
    return MQ_ERR_ALIGN;
  if (!argmax_stream_supported(M, N, K)) return MQ_ERR_UNSUPPORTED;
  if (M > argmax_static_max_rows()) return MQ_ERR_LIMIT;
  return launch_argmax_stream_static(packedA, packedW, M, N, K, sA, sW, tok, maxlogit, as_stream(stream));
}

int mq_gemm_argmax_shortlist(const void* packedA, const void* packedW, const int32_t* shortlist,
                             size_t shortlist_len, size_t M, size_t N, size_t K, const float* sA, const float* sW,
                             int32_t* tok, float* maxlogit, void* ws, size_t ws_bytes, void* stream) {
  if (packedA == nullptr || packedW == nullptr || shortlist == nullptr || sA == nullptr || sW == nullptr ||
      tok == nullptr || maxlogit == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, N, K) || shortlist_len == 0 || shortlist_len > N) return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(shortlist, 4) || !aligned(sA, 4) ||
      !aligned(sW, 4) || !aligned(tok, 4) || !aligned(maxlogit, 4) || !aligned(ws, 16))
    return MQ_ERR_ALIGN;
  if (ws_bytes < mq_argmax_ws_bytes(M, N)) return MQ_ERR_WORKSPACE;
  if (!argmax_stream_supported(M, N, K)) return MQ_ERR_UNSUPPORTED;
  return launch_argmax_stream(packedA, packedW, M, N, K, sA, sW, tok, maxlogit, ws, shortlist, shortlist_len,
                              as_stream(stream));
}

size_t mq_topk_ws_bytes(size_t M, size_t N, int k) {
  if (M == 0 || N == 0 || M >= kMaxDim || N >= kMaxDim || k < 1 || k > 4) return 0;
  return topk_stream_ws_bytes(M, k);
}

int mq_gemm_topk_packed(const void* packedA, const void* packedW, const int32_t* shortlist_or_null,
                        size_t shortlist_len, size_t M, size_t N, size_t K, const float* sA, const float* sW, int k,
                        int32_t* tok, float* logprob, void* ws, size_t ws_bytes, void* stream) {
  if (packedA == nullptr || packedW == nullptr || sA == nullptr || sW == nullptr || tok == nullptr ||
      logprob == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, N, K) || k < 1 || k > 4 || (size_t)k > N) return MQ_ERR_SHAPE;
  if (shortlist_or_null != nullptr && (shortlist_len == 0 || shortlist_len > N || (size_t)k > shortlist_len))
    return MQ_ERR_SHAPE;
  if (!aligned(packedA, 16) || !aligned(packedW, 16) || !aligned(sA, 4) || !aligned(sW, 4) || !aligned(tok, 4) ||
      !aligned(logprob, 4) || !aligned(ws, 16) || (shortlist_or_null != nullptr && !aligned(shortlist_or_null, 4)))
    return MQ_ERR_ALIGN;
  if (ws_bytes < mq_topk_ws_bytes(M, N, k)) return MQ_ERR_WORKSPACE;
  if (!topk_stream_supported(M, N, K, k)) return MQ_ERR_UNSUPPORTED;
  return launch_topk_stream(packedA, packedW, M, N, K, sA, sW, k, tok, logprob, ws, shortlist_or_null, shortlist_len,
                            as_stream(stream));
}

int mq_gemm_argmax(const void* qA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                   const float* sW, int32_t* tok, float* maxlogit, void* ws, size_t ws_bytes,
                   void* stream) {
  int rc = gemm_common_checks(qA, nullptr, packedW, 8, M, N, K);
  if (rc != MQ_OK) return rc;
  if (sA == nullptr || sW == nullptr || tok == nullptr || maxlogit == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!aligned(sA, 4) || !aligned(sW, 4) || !aligned(tok, 4) || !aligned(maxlogit, 4) || !aligned(ws, 16))
    return MQ_ERR_ALIGN;
  if (ws_bytes < mq_argmax_ws_bytes(M, N)) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  unsigned long long* keys = static_cast<unsigned long long*>(ws);
  rc = launch_argmax_init(keys, M, s);
  if (rc != MQ_OK) return rc;
  GemmArgs a{};
  a.qA = qA; a.packedW = packedW; a.bits = 8; a.M = M; a.N = N; a.K = K; a.keys = keys;
  rc = launch_gemm(a, kEpiArgmax, s);
  if (rc != MQ_OK) return rc;
  return launch_argmax_finish(keys, M, sA, sW, tok, maxlogit, s);
}

namespace mq {
namespace {
// Scratch layout of mq_ffn_i8_f32.
struct FfnWs {
  size_t off_part1, off_part2, off_scal, off_bar, off_qA, off_qH, total;
  FfnWs(size_t M, size_t d, size_t f) {
    off_part1 = 0;
    off_part2 = round_up(off_part1 + kAbsmaxPartials * sizeof(float), 256);
    off_scal = round_up(off_part2 + gemm_amax_partials(M, f) * sizeof(float), 256);
    off_bar = off_scal + 256;
    off_qA = off_bar + round_up(2 * kBarrierWords * sizeof(unsigned), 256);     // two agreement areas
    off_qH = round_up(off_qA + PackedDims(8, M, d).total_bytes(), 256);
    total = round_up(off_qH + PackedDims(8, M, f).total_bytes(), 256);
  }
};
}  // namespace
}  // namespace mq

static int g_ffn_single_pass = 1;

int mq_set_barrier_timeout_us(unsigned us) {
  if (us > 10u * 1000 * 1000) return MQ_ERR_SHAPE;
  set_barrier_timeout_ticks(100ull * us);       // the wall clock runs at 100 MHz
  return MQ_OK;
}

int mq_set_ffn_single_pass(int enable) {
  g_ffn_single_pass = enable != 0;
  return MQ_OK;
}

size_t mq_ffn_ws_bytes(size_t M, size_t d, size_t f) {
  if (!dims_ok(M, f, d)) return 0;
  return FfnWs(M, d, f).total;
}

namespace {
// The int8 FFN block.  prepared: the caller guarantees that the agreement words of the workspace are zero (see
// mq_ffn_ws_prepare), so no launch clears them; either way a call that took the single-pass kernels leaves them zero.
int ffn_i8_run(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
               const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
               void* ws, size_t ws_bytes, void* stream, bool prepared) {
  if (A == nullptr || packedW1 == nullptr || sW1 == nullptr || packedW2 == nullptr || sW2 == nullptr ||
      Y == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, f, d)) return MQ_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(packedW1, 16) || !aligned(packedW2, 16) || !aligned(ws, 256) ||
      !aligned(sW1, 4) || !aligned(sW2, 4) || !aligned(Y, 4))
    return MQ_ERR_ALIGN;
  if ((b1 != nullptr && !aligned(b1, 4)) || (b2 != nullptr && !aligned(b2, 4))) return MQ_ERR_ALIGN;
  const FfnWs L(M, d, f);
  if (ws_bytes < L.total) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  uint8_t* base = static_cast<uint8_t*>(ws);
  float* part1 = reinterpret_cast<float*>(base + L.off_part1);
  float* part2 = reinterpret_cast<float*>(base + L.off_part2);
  float* sA = reinterpret_cast<float*>(base + L.off_scal);
  float* sH = sA + 1;
  void* qA = base + L.off_qA;
  void* qH = base + L.off_qH;
  // a1 + a2: abs-max and quant_int of the input: for a million elements or more the kernel that reads A once
  // (1.9 us less per block for config 2 than the two-launch form, measured on one device in alternation)
  // two agreement areas: the first product's (G) and the quantizer's (Q)
  unsigned* G = reinterpret_cast<unsigned*>(base + L.off_bar);
  unsigned* Q = G + kBarrierWords;
  int rc = MQ_ERR_UNSUPPORTED;
  bool q_used = false;
  // (with a clearing launch in front of it that kernel only pays from a million elements on; without, always)
  if (g_ffn_single_pass && (prepared || M * d >= ((size_t)1 << 20))) {
    // one kernel reads A once and agrees on max|A| across the grid.  Its agreement words and the first product's
    // are cleared by a tiny launch -- or, with a prepared workspace, its own are zero already and it zeroes the
    // first product's on its way (which in turn zeroes the quantizer's for the next call)
    if (!prepared) {
      rc = launch_clear_words(G, 2 * kBarrierWords, s);
      if (rc != MQ_OK) return rc;
      rc = launch_absmax_quantize_pack_fused(A, M, d, 8, Q, sA, qA, s);
    } else {
      rc = launch_absmax_quantize_pack_fused(A, M, d, 8, Q, sA, qA, s, G, kBarrierWords);
    }
    q_used = rc == MQ_OK;
  }
  if (rc == MQ_ERR_UNSUPPORTED) rc = launch_absmax_quantize_pack(A, M, d, 8, part1, sA, qA, s, G, kBarrierWords);
  if (rc != MQ_OK) return rc;
  // a4 + a5, first pass: only the abs-max of relu(A W1 + b1) leaves the chip
  GemmArgs g1{};
  g1.qA = qA; g1.packedW = packedW1; g1.bits = 8; g1.M = M; g1.N = f; g1.K = d;
  g1.sA = sA; g1.sW = sW1; g1.bias = b1; g1.relu = 1;
  // when the first product's result is at most one tile per resident workgroup, one launch does both
  // passes with the sums held in registers across a grid-wide barrier
  if (q_used) {
    g1.clear_words = Q;        // the quantizer is done with them: left zero for the next call
    g1.nclear = kBarrierWords;
  }
  rc = g_ffn_single_pass ? launch_gemm_requant_coop(g1, sH, qH, G, s) : MQ_ERR_UNSUPPORTED;
  g1.clear_words = nullptr;
  g1.nclear = 0;
  if (rc == MQ_ERR_UNSUPPORTED) {
    if (q_used) {              // nobody else zeroes the quantizer's words on this path
      rc = launch_clear_words(Q, kBarrierWords, s);
      if (rc != MQ_OK) return rc;
    }
    rc = launch_gemm_amax_partial(g1, part2, s);
    if (rc != MQ_OK) return rc;
    // second pass: the same sums again, quantized with the multiplier now known, stored as packed int8
    rc = launch_gemm_requant(g1, part2, sH, qH, s);
  }
  if (rc != MQ_OK) return rc;
  // second product with the float epilogue
  GemmArgs g2{};
  g2.qA = qH; g2.packedW = packedW2; g2.bits = 8; g2.M = M; g2.N = d; g2.K = f;
  g2.sA = sH; g2.sW = sW2; g2.bias = b2; g2.relu = 0; g2.Y = Y;
  return launch_gemm_packed(g2, kEpiDequant, s);
}
}  // namespace

int mq_ffn_i8_f32(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
                  const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
                  void* ws, size_t ws_bytes, void* stream) {
  return ffn_i8_run(A, M, d, f, packedW1, sW1, b1, packedW2, sW2, b2, Y, ws, ws_bytes, stream, false);
}

int mq_ffn_ws_prepare(void* ws, size_t ws_bytes, size_t M, size_t d, size_t f, void* stream) {
  if (ws == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, f, d)) return MQ_ERR_SHAPE;
  if (!aligned(ws, 256)) return MQ_ERR_ALIGN;
  const FfnWs L(M, d, f);
  if (ws_bytes < L.total) return MQ_ERR_WORKSPACE;
  return launch_clear_words(reinterpret_cast<unsigned*>(static_cast<uint8_t*>(ws) + L.off_bar), 2 * kBarrierWords,
                            as_stream(stream));
}

int mq_ffn_i8_f32_prepared(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
                           const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
                           void* ws, size_t ws_bytes, void* stream) {
  return ffn_i8_run(A, M, d, f, packedW1, sW1, b1, packedW2, sW2, b2, Y, ws, ws_bytes, stream, true);
}

namespace mq {
namespace {
// Scratch layout of mq_ffn_i16_f32.
struct Ffn16Ws {
  size_t off_part, off_scal, off_bar, off_qA, off_H, off_qH, total;
  Ffn16Ws(size_t M, size_t d, size_t f) {
    off_part = 0;
    off_scal = round_up(kAbsmaxPartials * sizeof(float), 256);
    off_bar = off_scal + 256;                                        // agreement words of the one-kernel quantizer
    off_qA = off_bar + round_up(kBarrierWords * sizeof(unsigned), 256);
    off_H = round_up(off_qA + PackedDims(16, M, d).total_bytes(), 256);
    off_qH = round_up(off_H + M * f * sizeof(float), 256);
    total = round_up(off_qH + PackedDims(16, M, f).total_bytes(), 256);
  }
};
}  // namespace
}  // namespace mq

size_t mq_ffn_i16_ws_bytes(size_t M, size_t d, size_t f) {
  if (!dims_ok(M, f, d)) return 0;
  return Ffn16Ws(M, d, f).total;
}

int mq_ffn_i16_f32(const float* A, size_t M, size_t d, size_t f, const void* packedW1, const float* sW1,
                   const float* b1, const void* packedW2, const float* sW2, const float* b2, float* Y,
                   void* ws, size_t ws_bytes, void* stream) {
  if (A == nullptr || packedW1 == nullptr || sW1 == nullptr || packedW2 == nullptr || sW2 == nullptr ||
      Y == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, f, d)) return MQ_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(packedW1, 16) || !aligned(packedW2, 16) || !aligned(ws, 256) ||
      !aligned(sW1, 4) || !aligned(sW2, 4) || !aligned(Y, 4))
    return MQ_ERR_ALIGN;
  if ((b1 != nullptr && !aligned(b1, 4)) || (b2 != nullptr && !aligned(b2, 4))) return MQ_ERR_ALIGN;
  const Ffn16Ws L(M, d, f);
  if (ws_bytes < L.total) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  uint8_t* base = static_cast<uint8_t*>(ws);
  float* part = reinterpret_cast<float*>(base + L.off_part);
  float* sA = reinterpret_cast<float*>(base + L.off_scal);
  float* sH = sA + 1;
  float* hmax = sA + 2;                       // max|H|: kHmaxSlots words raised by the first product's workgroups
  constexpr unsigned kHmaxSlots = 32;
  uint8_t* qA = base + L.off_qA;
  float* H = reinterpret_cast<float*>(base + L.off_H);
  uint8_t* qH = base + L.off_qH;
  // a1 + a2 on the input.  Where the tensor fits the registers of one resident grid it is read once: a small launch
  // clears the agreement words and max|H|, then one kernel finds max|A| across the grid and converts from registers;
  // otherwise two passes (partial maxima, then the quantizer), the first of which zeroes max|H|.
  unsigned* bar = reinterpret_cast<unsigned*>(base + L.off_bar);
  static_assert(sizeof(float) * 3 <= 256, "max|H| sits right in front of the agreement words");
  int rc = MQ_ERR_UNSUPPORTED;
  if (g_ffn_single_pass && M * d >= ((size_t)1 << 20)) {
    // hmax is the third float of the 256 bytes in front of `bar`: one clearing launch covers both
    rc = launch_clear_words(reinterpret_cast<unsigned*>(hmax), (unsigned)((L.off_bar - L.off_scal) / 4 - 2 + kBarrierWords), s);
    if (rc != MQ_OK) return rc;
    rc = launch_absmax_quantize_pack_fused(A, M, d, 16, bar, sA, qA, s);
  }
  if (rc == MQ_ERR_UNSUPPORTED)
    rc = launch_absmax_quantize_pack(A, M, d, 16, part, sA, qA, s, reinterpret_cast<unsigned*>(hmax), kHmaxSlots);
  if (rc != MQ_OK) return rc;
  // a4 + a5: H = relu(A W1 + b1) in binary32, max|H| as a by-product of the epilogue
  GemmArgs g1{};
  g1.qA = qA;
  g1.packedW = packedW1; g1.bits = 16; g1.M = M; g1.N = f; g1.K = d;
  g1.sA = sA; g1.sW = sW1; g1.bias = b1; g1.relu = 1; g1.Y = H; g1.out_amax = hmax; g1.amax_slots = kHmaxSlots;
  rc = launch_gemm_packed(g1, kEpiDequant, s);
  if (rc != MQ_OK) return rc;
  // a1 + a2 on H: the multiplier comes from the maxima already there (kernels that do not know about the slots
  // raise the first word only; the others then stay zero)
  rc = launch_quantize_pack_partials(H, M, f, 16, hmax, kHmaxSlots, sH, qH, s);
  if (rc != MQ_OK) return rc;
  GemmArgs g2{};
  g2.qA = qH;
  g2.packedW = packedW2; g2.bits = 16; g2.M = M; g2.N = d; g2.K = f;
  g2.sA = sH; g2.sW = sW2; g2.bias = b2; g2.relu = 0; g2.Y = Y;
  return launch_gemm_packed(g2, kEpiDequant, s);
}

size_t mq_ffn_i16_fixed_ws_bytes(size_t M, size_t d, size_t f) {
  if (!dims_ok(M, f, d)) return 0;
  return round_up(PackedDims(16, M, d).total_bytes(), 256) + round_up(PackedDims(16, M, f).total_bytes(), 256);
}

int mq_ffn_i16_fixed_f32(const float* A, size_t M, size_t d, size_t f, const float* sA, const void* packedW1,
                         const float* sW1, const float* b1, const float* sH, const void* packedW2, const float* sW2,
                         const float* b2, float* Y, void* ws, size_t ws_bytes, void* stream) {
  if (A == nullptr || sA == nullptr || packedW1 == nullptr || sW1 == nullptr || sH == nullptr || packedW2 == nullptr ||
      sW2 == nullptr || Y == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  if (!dims_ok(M, f, d)) return MQ_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(packedW1, 16) || !aligned(packedW2, 16) || !aligned(ws, 256) || !aligned(sA, 4) ||
      !aligned(sW1, 4) || !aligned(sH, 4) || !aligned(sW2, 4) || !aligned(Y, 4))
    return MQ_ERR_ALIGN;
  if ((b1 != nullptr && !aligned(b1, 4)) || (b2 != nullptr && !aligned(b2, 4))) return MQ_ERR_ALIGN;
  if (ws_bytes < mq_ffn_i16_fixed_ws_bytes(M, d, f)) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  uint8_t* qA = static_cast<uint8_t*>(ws);
  uint8_t* qH = qA + round_up(PackedDims(16, M, d).total_bytes(), 256);
  // quant_int(A) with the given multiplier, product + b1 + ReLU re-quantized with the given multiplier in the
  // epilogue (H goes to memory once, as packed 16-bit values), product + b2
  int rc = launch_quantize_pack(A, M, d, 16, sA, qA, s);
  if (rc != MQ_OK) return rc;
  GemmArgs g1{};
  g1.qA = qA; g1.packedW = packedW1; g1.bits = 16; g1.M = M; g1.N = f; g1.K = d;
  g1.sA = sA; g1.sW = sW1; g1.bias = b1; g1.relu = 1;
  rc = launch_gemm_requant_fixed_i16(g1, sH, qH, s);
  if (rc != MQ_OK) return rc;
  GemmArgs g2{};
  g2.qA = qH; g2.packedW = packedW2; g2.bits = 16; g2.M = M; g2.N = d; g2.K = f;
  g2.sA = sH; g2.sW = sW2; g2.bias = b2; g2.relu = 0; g2.Y = Y;
  return launch_gemm_packed(g2, kEpiDequant, s);
}

size_t mq_linear_ws_bytes(int bits, size_t M, size_t K) {
  if (!bits_ok(bits) || M == 0 || K == 0 || M >= kMaxDim || K >= kMaxDim || M > kMaxElems / K) return 0;
  return LinearWs(bits, M, K).total;
}

int mq_linear_f32(const float* A, size_t M, size_t K, const float* sA_or_null, const void* packedW,
                  const float* sW, int bits, size_t N, const float* bias, int relu, float* Y,
                  float* out_amax, void* ws, size_t ws_bytes, void* stream) {
  if (!bits_ok(bits)) return MQ_ERR_DTYPE;
  if (A == nullptr || packedW == nullptr || sW == nullptr || Y == nullptr || ws == nullptr) return MQ_ERR_NULL;
  if (!dims_ok(M, N, K)) return MQ_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(packedW, 16) || !aligned(ws, 16) || !aligned(sW, 4) || !aligned(Y, 4))
    return MQ_ERR_ALIGN;
  if ((sA_or_null != nullptr && !aligned(sA_or_null, 4)) || (bias != nullptr && !aligned(bias, 4)) ||
      (out_amax != nullptr && !aligned(out_amax, 4)))
    return MQ_ERR_ALIGN;
  const LinearWs L(bits, M, K);
  if (ws_bytes < L.total) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  uint8_t* base = static_cast<uint8_t*>(ws);
  float* scale = reinterpret_cast<float*>(base + L.off_scale);
  float* part = reinterpret_cast<float*>(base + L.off_part);
  void* q = base + L.off_q;
  const float* sA = sA_or_null;
  GemmArgs a{};
  a.packedW = packedW; a.bits = bits; a.M = M; a.N = N; a.K = K;
  a.sW = sW; a.bias = bias; a.relu = relu != 0; a.Y = Y; a.out_amax = out_amax;
  int rc;
  if (bits == 8 && gemm_small_f32_supported(M, N, K)) {
    // decode-sized input: quant_int happens inside the product's operand fetch (same arithmetic, same
    // results), one launch with a given multiplier, two with abs-max
    if (sA != nullptr) return launch_gemm_small_f32(A, sA, 0, nullptr, a, s);
    unsigned np = 0;
    rc = launch_absmax_partials(A, M * K, part, &np, s);
    if (rc != MQ_OK) return rc;
    return launch_gemm_small_f32(A, part, np, scale, a, s);
  }
  // general case: quant_int straight into fragment order, then the packed product
  if (sA == nullptr) {
    rc = launch_absmax_quantize_pack(A, M, K, bits, part, scale, q, s);
    sA = scale;
  } else {
    rc = launch_quantize_pack(A, M, K, bits, sA, q, s);
  }
  if (rc != MQ_OK) return rc;
  a.qA = q; a.sA = sA;
  return launch_gemm_packed(a, kEpiDequant, s);
}

/* ---- float glue of the averaging-attention decode step -------------------- */

int mq_running_average_f32(const float* g_prev, const float* x, size_t n, int t, float* g, void* stream) {
  if (g_prev == nullptr || x == nullptr || g == nullptr) return MQ_ERR_NULL;
  if (n == 0 || n > kMaxElems || t < 1) return MQ_ERR_SHAPE;
  if (!aligned(g_prev, 4) || !aligned(x, 4) || !aligned(g, 4)) return MQ_ERR_ALIGN;
  return launch_running_average(g_prev, x, n, t, g, as_stream(stream));
}

int mq_concat2_f32(const float* a, size_t da, const float* b, size_t db, size_t M, float* out, void* stream) {
  if (a == nullptr || b == nullptr || out == nullptr) return MQ_ERR_NULL;
  if (M == 0 || da == 0 || db == 0 || M >= kMaxDim || da >= kMaxDim || db >= kMaxDim) return MQ_ERR_SHAPE;
  if (!aligned(a, 4) || !aligned(b, 4) || !aligned(out, 4)) return MQ_ERR_ALIGN;
  return launch_concat2(a, da, b, db, M, out, as_stream(stream));
}

int mq_add_layer_norm_f32(const float* a, const float* r, const float* gamma, const float* beta, size_t M, size_t d,
                          float eps, float* y, void* stream) {
  if (a == nullptr || r == nullptr || gamma == nullptr || beta == nullptr || y == nullptr) return MQ_ERR_NULL;
  if (M == 0 || d == 0 || M >= kMaxDim || d >= kMaxDim || !(eps >= 0.0f)) return MQ_ERR_SHAPE;
  if (!aligned(a, 4) || !aligned(r, 4) || !aligned(gamma, 4) || !aligned(beta, 4) || !aligned(y, 4)) return MQ_ERR_ALIGN;
  return launch_add_layer_norm(a, r, gamma, beta, M, d, eps, y, as_stream(stream));
}

int mq_gate_mix_layer_norm_f32(const float* x, const float* f, const float* z, const float* gamma, const float* beta,
                               size_t M, size_t d, float eps, float* y, void* stream) {
  if (x == nullptr || f == nullptr || z == nullptr || gamma == nullptr || beta == nullptr || y == nullptr)
    return MQ_ERR_NULL;
  if (M == 0 || d == 0 || M >= kMaxDim || d >= kMaxDim / 2 || !(eps >= 0.0f)) return MQ_ERR_SHAPE;
  if (!aligned(x, 4) || !aligned(f, 4) || !aligned(z, 4) || !aligned(gamma, 4) || !aligned(beta, 4) || !aligned(y, 4))
    return MQ_ERR_ALIGN;
  return launch_gate_mix_layer_norm(x, f, z, gamma, beta, M, d, eps, y, as_stream(stream));
}

int mq_cross_attention_f32(const float* q, const float* K, const float* V, size_t M, size_t S, size_t d, int heads,
                           float* ctx, void* stream) {
  if (q == nullptr || K == nullptr || V == nullptr || ctx == nullptr) return MQ_ERR_NULL;
  if (M == 0 || S == 0 || d == 0 || heads <= 0 || M >= kMaxDim || S >= kMaxDim || d >= kMaxDim || d % (size_t)heads != 0)
    return MQ_ERR_SHAPE;
  if (!aligned(q, 4) || !aligned(K, 4) || !aligned(V, 4) || !aligned(ctx, 4)) return MQ_ERR_ALIGN;
  return launch_cross_attention(q, K, V, M, S, d, heads, ctx, as_stream(stream));
}

namespace mq {
namespace {
// Scratch layout of mq_aan_layer_f32: quantizer partials, two multipliers, one packed 8-bit activation
// buffer sized for the widest product input, and the float intermediates of the layer.
struct AanWs {
  size_t off_part, off_gpart, off_xpart, off_hpart, off_hpart2, off_scal, off_q, off_hid, off_f, off_cat, off_z, off_y1, off_qv, off_ctx, off_o, off_y2, off_ff, total;
  AanWs(size_t M, size_t d, size_t ffn, size_t aan_ffn) {
    const size_t widest = ffn > aan_ffn ? (ffn > 2 * d ? ffn : 2 * d) : (aan_ffn > 2 * d ? aan_ffn : 2 * d);
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o = round_up(o + bytes, 256); return at; };
    off_part = take(kAbsmaxPartials * sizeof(float));
    off_gpart = take((running_average_partials(M * d) > M ? running_average_partials(M * d) : M) * sizeof(float));
    off_xpart = take(running_average_partials(M * d) * sizeof(float));
    off_hpart = take(kAbsmaxPartials * sizeof(float));
    off_hpart2 = take(kAbsmaxPartials * sizeof(float));
    off_scal = take(256);
    off_q = take(PackedDims(8, M, widest).total_bytes());
    off_hid = take(M * (ffn > aan_ffn ? ffn : aan_ffn) * sizeof(float));
    off_f = take(M * d * sizeof(float));
    off_cat = take(M * 2 * d * sizeof(float));
    off_z = take(M * 2 * d * sizeof(float));
    off_y1 = take(M * d * sizeof(float));
    off_qv = take(M * d * sizeof(float));
    off_ctx = take(M * d * sizeof(float));
    off_o = take(M * d * sizeof(float));
    off_y2 = take(M * d * sizeof(float));
    off_ff = take(M * d * sizeof(float));
    total = o;
  }
};
bool product_ok(const mq_product& p) {
  return p.packed != nullptr && p.scale != nullptr && aligned(p.packed, 16) && aligned(p.scale, 4) &&
         (p.bias == nullptr || aligned(p.bias, 4));
}
bool norm_ok(const mq_norm& n) { return n.gamma != nullptr && n.beta != nullptr && aligned(n.gamma, 4) && aligned(n.beta, 4); }
}  // namespace
}  // namespace mq

size_t mq_aan_layer_ws_bytes(size_t M, size_t d, size_t ffn, size_t aan_ffn) {
  if (!dims_ok(M, ffn, d) || !dims_ok(M, aan_ffn, d) || !dims_ok(M, 2 * d, 2 * d)) return 0;
  return AanWs(M, d, ffn, aan_ffn).total;
}

int mq_aan_layer_f32(const mq_aan_layer* P, const float* x, const float* g_prev, int t, const float* K, const float* V,
                     size_t M, size_t S, int heads, int use_ffn, int use_gate, float eps, float* y, float* g_out,
                     void* ws, size_t ws_bytes, void* stream) {
  if (P == nullptr || x == nullptr || g_prev == nullptr || K == nullptr || V == nullptr || y == nullptr ||
      g_out == nullptr || ws == nullptr)
    return MQ_ERR_NULL;
  const size_t d = P->d, ffn = P->ffn, aan_ffn = P->aan_ffn;
  if (!dims_ok(M, ffn, d) || !dims_ok(M, aan_ffn, d) || !dims_ok(M, 2 * d, 2 * d) || S == 0 || S >= kMaxDim || t < 1 ||
      heads <= 0 || d % (size_t)heads != 0 || !(eps >= 0.0f))
    return MQ_ERR_SHAPE;
  if (!product_ok(P->ctx_q) || !product_ok(P->ctx_o) || !product_ok(P->ffn1) || !product_ok(P->ffn2) ||
      !norm_ok(P->ln1) || !norm_ok(P->ln2) || !norm_ok(P->ln3))
    return MQ_ERR_NULL;
  if (use_ffn && (!product_ok(P->aan_ffn1) || !product_ok(P->aan_ffn2))) return MQ_ERR_NULL;
  if (use_gate && !product_ok(P->aan_gate)) return MQ_ERR_NULL;
  if (!aligned(x, 16) || !aligned(g_prev, 4) || !aligned(K, 4) || !aligned(V, 4) || !aligned(y, 4) ||
      !aligned(g_out, 16) || !aligned(ws, 256))
    return MQ_ERR_ALIGN;
  const AanWs L(M, d, ffn, aan_ffn);
  if (ws_bytes < L.total) return MQ_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  uint8_t* base = static_cast<uint8_t*>(ws);
  float* part = reinterpret_cast<float*>(base + L.off_part);
  float* sA = reinterpret_cast<float*>(base + L.off_scal);
  void* qbuf = base + L.off_q;
  auto fbuf = [&](size_t off) { return reinterpret_cast<float*>(base + off); };
  float *hid = fbuf(L.off_hid), *f = fbuf(L.off_f), *cat = fbuf(L.off_cat), *z = fbuf(L.off_z), *y1 = fbuf(L.off_y1),
        *qv = fbuf(L.off_qv), *ctx = fbuf(L.off_ctx), *o = fbuf(L.off_o), *y2 = fbuf(L.off_y2), *ff = fbuf(L.off_ff);
  float* gpart = reinterpret_cast<float*>(base + L.off_gpart);
  float* hpart = reinterpret_cast<float*>(base + L.off_hpart);
  float* hpart2 = reinterpret_cast<float*>(base + L.off_hpart2);
  float* xpart = reinterpret_cast<float*>(base + L.off_xpart);
  float* hmax = sA + 1;           // three words: max|.| of three products' outputs where no per-workgroup maxima are
                                  // available, cleared by the first kernel
  // One parameter product: quant_int of the input with its own abs-max multiplier, dot'_int, bias (+ReLU).
  // The kernel that produced the input has already left partial maxima of it (np of them at `partials`), so the
  // quantizer needs no abs-max pass of its own; inputs with more rows than the quantizer reduces per block take
  // the separate pass.  want_max: the product that follows needs max|Y|; it is left as *out_np partial maxima at
  // *out_partials (one per workgroup, no atomics) where the decode-sized kernels run, else in the word hword.
  const float* out_partials = nullptr;
  size_t out_np = 0;
  auto product = [&](const float* A, size_t Kdim, const mq_product& W, size_t N, int relu, float* Y,
                     const float* partials, size_t np, bool want_max, float* hword, float* out_buf) -> int {
    int rc;
    GemmArgs g{};
    g.packedW = W.packed; g.bits = 8; g.M = M; g.N = N; g.K = Kdim;
    g.sW = W.scale; g.bias = W.bias; g.relu = relu; g.Y = Y;
    out_partials = nullptr; out_np = 0;
    if (partials != nullptr && np <= kAbsmaxPartials && gemm_small_f32_supported(M, N, Kdim)) {
      // short K: quant_int inside the product's operand fetch, no quantizing launch
      if (want_max) {
        const size_t wg = gemm_small_f32_partials(M, N, Kdim);
        if (wg <= kAbsmaxPartials) { g.partial = out_buf; out_partials = out_buf; out_np = wg; }
        else { g.out_amax = hword; out_partials = hword; out_np = 1; }
      }
      return launch_gemm_small_f32(A, partials, (unsigned)np, sA, g, s);
    }
    if (partials != nullptr && np <= kAbsmaxPartials)
      rc = launch_quantize_pack_partials(A, M, Kdim, 8, partials, (unsigned)np, sA, qbuf, s);
    else
      rc = launch_absmax_quantize_pack(A, M, Kdim, 8, part, sA, qbuf, s);
    if (rc != MQ_OK) return rc;
    g.qA = qbuf; g.sA = sA;
    if (want_max && M <= 512 && gemm_small_partials(M, N, Kdim) <= kAbsmaxPartials) {
      // decode-sized: the split-K kernel leaves one maximum per workgroup
      g.partial = out_buf; out_partials = out_buf; out_np = gemm_small_partials(M, N, Kdim);
      return launch_gemm_small(g, kEpiDequant, s);
    }
    if (want_max) { g.out_amax = hword; out_partials = hword; out_np = 1; }
    return launch_gemm_packed(g, kEpiDequant, s);
  };
  const size_t np_avg = running_average_partials(M * d);
  int rc = launch_running_average(g_prev, x, M * d, t, g_out, s, gpart, reinterpret_cast<unsigned*>(hmax), 3, xpart);
  if (rc != MQ_OK) return rc;
  const float* fpath = g_out;
  const float* fpart = gpart;     // partial maxima of |f|
  size_t fnp = np_avg;
  if (use_ffn) {
    if ((rc = product(g_out, d, P->aan_ffn1, aan_ffn, 1, hid, gpart, np_avg, true, hmax, hpart)) != MQ_OK) return rc;
    const float* hp = out_partials;
    const size_t hn = out_np;
    if ((rc = product(hid, aan_ffn, P->aan_ffn2, d, 0, f, hp, hn, use_gate != 0, hmax + 2, hpart2)) != MQ_OK) return rc;
    fpath = f;
    fpart = out_partials;
    fnp = out_np;
  }
  if (use_gate) {
    GemmArgs gg{};
    gg.packedW = P->aan_gate.packed; gg.bits = 8; gg.M = M; gg.N = 2 * d; gg.K = 2 * d;
    gg.sW = P->aan_gate.scale; gg.bias = P->aan_gate.bias; gg.relu = 0; gg.Y = z;
    if (gemm_small_f32_supported(M, 2 * d, 2 * d) && d % 4 == 0 && fpart != nullptr && fnp >= 1) {
      // the gate's input [x, f] is read from its two pieces (with their partial maxima) inside the product
      // kernel: the concatenation is never stored and its launch disappears
      rc = launch_gemm_small_f32_pair(x, d, xpart, (unsigned)np_avg, fpath, fpart, (unsigned)fnp, sA, gg, s);
      if (rc != MQ_OK) return rc;
    } else {
      if ((rc = launch_concat2(x, d, fpath, d, M, cat, s, gpart)) != MQ_OK) return rc;
      if ((rc = product(cat, 2 * d, P->aan_gate, 2 * d, 0, z, gpart, M, false, nullptr, nullptr)) != MQ_OK) return rc;
    }
    rc = launch_gate_mix_layer_norm(x, fpath, z, P->ln1.gamma, P->ln1.beta, M, d, eps, y1, s, gpart);
  } else {
    rc = launch_add_layer_norm(fpath, x, P->ln1.gamma, P->ln1.beta, M, d, eps, y1, s, gpart);
  }
  if (rc != MQ_OK) return rc;
  if ((rc = product(y1, d, P->ctx_q, d, 0, qv, gpart, M, false, nullptr, nullptr)) != MQ_OK) return rc;
  if ((rc = launch_cross_attention(qv, K, V, M, S, d, heads, ctx, s, gpart)) != MQ_OK) return rc;
  if ((rc = product(ctx, d, P->ctx_o, d, 0, o, gpart, M, false, nullptr, nullptr)) != MQ_OK) return rc;
  if ((rc = launch_add_layer_norm(o, y1, P->ln2.gamma, P->ln2.beta, M, d, eps, y2, s, gpart)) != MQ_OK) return rc;
  if ((rc = product(y2, d, P->ffn1, ffn, 1, hid, gpart, M, true, hmax + 1, hpart)) != MQ_OK) return rc;
  const float* hp2 = out_partials;
  const size_t hn2 = out_np;
  if ((rc = product(hid, ffn, P->ffn2, d, 0, ff, hp2, hn2, false, nullptr, nullptr)) != MQ_OK) return rc;
  return launch_add_layer_norm(ff, y2, P->ln3.gamma, P->ln3.beta, M, d, eps, y, s);
}

}  // extern "C"
