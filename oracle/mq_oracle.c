/*
 * mq_oracle.c -- plain CPU oracle for the low-precision matrix-product path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
 * compute; it is slow on purpose (scalar loops, no blocking, no SIMD
 * intrinsics, no BLAS) so that every function can be checked against the paper
 * by eye.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  It shares no code, header, table or helper with the HIP
 * library and neither side includes or imports the other.
 *
 * What the path computes (arxiv 1805.12096):
 *   quant_int   Section 4.2 "Quantization and integer products": multiply by a
 *               quantization multiplier, round to a signed integer; 8-bit
 *               values end up in [-127, 127], 16-bit in [-32767, 32767].
 *   dot'_int    Section 4.3 "Memoization": the integer product of two already
 *               quantized tensors, A times the transpose of B (both operands
 *               contiguous along the contracted index), with 32-bit sums
 *               (Section 4.2).
 *   epilogue    The integer product stands in for the float product (Sections
 *               4.3, 4.4), so its sums are scaled back to float and the bias
 *               is added; outputs are neither clipped nor quantized (4.2).
 *   arg-max     Section 2.3 "Decoding with small beams": with beam size 1 no
 *               softmax is evaluated, the word with the highest activation is
 *               taken.
 *
 * Precision.  The inputs are binary32 and the quantized tensors have to be
 * reproducible bit for bit, so the quantizer's arithmetic is fixed to binary32
 * with round-to-nearest-even: one multiply, one rint, one clamp.  The integer
 * product is exact (64-bit sums) and then reduced modulo 2^32, which is what a
 * 32-bit accumulator without saturation holds whatever the summation order
 * (Section 4.2 notes that no saturating 32-bit add exists on the paper's
 * machine).  The epilogue is one binary32 divide for the inverse scale and one
 * fused multiply-add per output.
 *
 * Pins (tests/test_oracle_pins.py): hand-computed dyadic quantization cases,
 * brute force with unbounded Python integers, closed forms (constant matrices,
 * identity, the 32767*32767*K wrap), numpy's int64 product, the closed-form
 * quantization error bound against an fp64 product of the real inputs, fp64
 * evaluation of the epilogue, numpy.argmax with planted winners and ties.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Largest magnitude quant_int may produce: Section 4.2 scales 8-bit values to
 * [-127, 127]; the 16-bit range is taken symmetric in the same way. */
static int qmax_of(int bits) { return bits == 8 ? 127 : (bits == 16 ? 32767 : 0); }

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void orc_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* max_i |x_i| over the finite-or-infinite entries; NaNs are skipped and
 * counted.  The maximum of a set of floats is exact and order free. */
float orc_absmax_f32(const float* x, size_t n, uint64_t* nan_count) {
  float amax = 0.0f;
  uint64_t nans = 0;
  for (size_t i = 0; i < n; ++i) {
    float v = x[i];
    if (v != v) { ++nans; continue; }
    float a = fabsf(v);
    if (a > amax) amax = a;
  }
  if (nan_count) *nan_count = nans;
  return amax;
}

/* Per-tensor multiplier that maps the largest magnitude onto Qmax: one
 * correctly rounded binary32 division.  An all-zero tensor gets 1. */
float orc_scale_from_amax(float amax, int bits) {
  float q = (float)qmax_of(bits);
  if (!(amax > 0.0f)) return 1.0f;
  return q / amax;
}

/* quant_int (Section 4.2): q = clamp(round_half_even(x * s), -Qmax, +Qmax).
 * NaN products (NaN input, or inf * 0) become 0 and are counted.
 * q is int8_t[n] for bits == 8, int16_t[n] for bits == 16. */
int orc_quant_int(const float* x, size_t n, int bits, float s, void* q, uint64_t* nan_count) {
  const int qm = qmax_of(bits);
  if (qm == 0) return -1;
  const float lim = (float)qm;
  uint64_t nans = 0;
  for (size_t i = 0; i < n; ++i) {
    volatile float t = x[i] * s; /* one binary32 multiply, never contracted */
    float r = rintf(t);          /* round half to even (default rounding mode) */
    int v;
    if (r != r) { v = 0; ++nans; }
    else if (r > lim) v = qm;
    else if (r < -lim) v = -qm;
    else v = (int)r;
    if (bits == 8) ((int8_t*)q)[i] = (int8_t)v;
    else ((int16_t*)q)[i] = (int16_t)v;
  }
  if (nan_count) *nan_count = nans;
  return 0;
}

/* dot'_int (Section 4.3): acc[m][n] = sum_k qA[m][k] * qB[n][k], A is [M x K],
 * B is [N x K], both row-major, i.e. A times B transposed.  The sum is taken
 * exactly in 64 bits and stored modulo 2^32 (two's complement).  overflow_count
 * receives the number of outputs whose exact sum does not fit 32 bits. */
int orc_dot_int(const void* qA, const void* qB, int bits, size_t M, size_t N, size_t K,
                int32_t* acc, uint64_t* overflow_count) {
  if (qmax_of(bits) == 0) return -1;
  uint64_t over = 0;
  const int8_t* a8 = (const int8_t*)qA;
  const int8_t* b8 = (const int8_t*)qB;
  const int16_t* a16 = (const int16_t*)qA;
  const int16_t* b16 = (const int16_t*)qB;
#pragma omp parallel for schedule(static) reduction(+ : over)
  for (ptrdiff_t m = 0; m < (ptrdiff_t)M; ++m) {
    for (size_t n = 0; n < N; ++n) {
      int64_t sum = 0;
      if (bits == 8) {
        for (size_t k = 0; k < K; ++k) sum += (int64_t)a8[m * K + k] * (int64_t)b8[n * K + k];
      } else {
        for (size_t k = 0; k < K; ++k) sum += (int64_t)a16[m * K + k] * (int64_t)b16[n * K + k];
      }
      uint32_t low = (uint32_t)((uint64_t)sum & 0xFFFFFFFFu);
      int32_t wrapped;
      memcpy(&wrapped, &low, sizeof wrapped);
      if ((int64_t)wrapped != sum) ++over;
      acc[m * N + n] = wrapped;
    }
  }
  if (overflow_count) *overflow_count = over;
  return 0;
}

/* Epilogue: y = fma((float)acc, u, bias[n]) with u = 1 / (sA * sW), then
 * max(y, 0) if relu.  bias may be NULL (treated as 0). */
int orc_dequant_bias(const int32_t* acc, size_t M, size_t N, float sA, float sW,
                     const float* bias, int relu, float* Y) {
  volatile float p = sA * sW;
  volatile float u = 1.0f / p;
  for (size_t m = 0; m < M; ++m) {
    for (size_t n = 0; n < N; ++n) {
      float b = bias ? bias[n] : 0.0f;
      float y = fmaf((float)acc[m * N + n], u, b);
      if (relu) y = (y > 0.0f) ? y : 0.0f;
      Y[m * N + n] = y;
    }
  }
  return 0;
}

/* Greedy arg-max on the integer sums (Section 2.3; no softmax): the smallest
 * column index holding the row maximum, and that maximum scaled to float.
 * Valid on integers because u > 0 is one scalar per product. */
int orc_argmax_i32(const int32_t* acc, size_t M, size_t N, float sA, float sW,
                   int32_t* tok, float* maxlogit) {
  if (N == 0) return -1;
  volatile float p = sA * sW;
  volatile float u = 1.0f / p;
  for (size_t m = 0; m < M; ++m) {
    int32_t best = acc[m * N];
    size_t arg = 0;
    for (size_t n = 1; n < N; ++n) {
      if (acc[m * N + n] > best) { best = acc[m * N + n]; arg = n; }
    }
    tok[m] = (int32_t)arg;
    volatile float v = (float)best * u;
    maxlogit[m] = v;
  }
  return 0;
}

/* Arg-max on float activations (used when an output bias is present):
 * smallest index of the row maximum. */
int orc_argmax_f32(const float* Y, size_t M, size_t N, int32_t* tok, float* maxval) {
  if (N == 0) return -1;
  for (size_t m = 0; m < M; ++m) {
    float best = Y[m * N];
    size_t arg = 0;
    for (size_t n = 1; n < N; ++n) {
      if (Y[m * N + n] > best) { best = Y[m * N + n]; arg = n; }
    }
    tok[m] = (int32_t)arg;
    maxval[m] = best;
  }
  return 0;
}
