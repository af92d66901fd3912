// Floating-point glue between the integer products of one greedy decode step of the averaging
// attention decoder (arxiv 1805.12096, Section 3.2: the decoder's self-attention is replaced by a
// cumulative uniform average that is updated from the last step only, followed by a feed-forward
// network and a gate; Section 3.1: source attention and the position-wise feed-forward block; every
// sub-layer ends in residual + layer normalisation).  All tensors are binary32, a decode step has a
// few hundred rows of model width, so every kernel here is one short pass over a few 100 KB: one
// workgroup per sentence, the row staged in LDS, reductions inside the workgroup.
#include "mq_internal.h"

namespace mq {

namespace {

constexpr int kT = 256;              // threads per workgroup
constexpr int kMaxRow = 8192;        // floats of a row kept in LDS (32 KB)
constexpr int kMaxScores = 4096;     // heads x source positions kept in LDS

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// sum over the workgroup; every thread gets the result.  `red` holds kT / 64 floats.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum_f(v);
  __syncthreads();                               // `red` may still be read from the call before
  if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int k = 1; k < kT / kWave; ++k) r += red[k];
  return r;
}

// max over the workgroup of a non-negative value, to partial[blockIdx.x] (for the abs-max of the tensor
// this kernel writes, so that the quantizer of the next product needs no pass of its own)
__device__ __forceinline__ void block_absmax_out(float v, float* red, float* __restrict__ partial) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  __syncthreads();
  if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = red[0];
#pragma unroll
    for (int k = 1; k < kT / kWave; ++k) r = fmaxf(r, red[k]);
    partial[blockIdx.x] = r;
  }
}

__global__ __launch_bounds__(kT) void k_running_average(const float* __restrict__ g_prev, const float* __restrict__ x,
                                                        size_t n, float tm1, float t, float* __restrict__ g,
                                                        float* __restrict__ partial, unsigned* __restrict__ clear,
                                                        unsigned nclear) {
  __shared__ float red[kT / kWave];
  const size_t i = (size_t)blockIdx.x * kT + threadIdx.x;
  float v = 0.f;
  if (i < n) {
    v = __fdiv_rn(__fmaf_rn(tm1, g_prev[i], x[i]), t);
    g[i] = v;
  }
  if (clear != nullptr && blockIdx.x == 0 && threadIdx.x < nclear) clear[threadIdx.x] = 0u;   // later kernels' maxima
  if (partial != nullptr) block_absmax_out(fabsf(v), red, partial);       // fmaxf drops NaN
}

__global__ __launch_bounds__(kT) void k_concat2(const float* __restrict__ a, unsigned da, const float* __restrict__ b,
                                                unsigned db, float* __restrict__ out, float* __restrict__ partial) {
  __shared__ float red[kT / kWave];
  const size_t m = blockIdx.x;
  float mx = 0.f;
  for (unsigned j = threadIdx.x; j < da + db; j += kT) {
    const float v = j < da ? a[m * da + j] : b[m * db + (j - da)];
    out[m * (da + db) + j] = v;
    mx = fmaxf(mx, fabsf(v));
  }
  if (partial != nullptr) block_absmax_out(mx, red, partial);
}

__device__ __forceinline__ float sigmoidf_(float z) { return __fdiv_rn(1.0f, 1.0f + expf(-z)); }

// One workgroup per row: h = GATED ? sigmoid(z[:d]) x + sigmoid(z[d:]) f : a;  y = LN(h + r) gamma + beta with
// the biased variance, mean and variance as two passes over the row held in LDS.
template <bool GATED>
__global__ __launch_bounds__(kT) void k_layer_norm(const float* __restrict__ a, const float* __restrict__ f,
                                                   const float* __restrict__ z, const float* __restrict__ r,
                                                   const float* __restrict__ gamma, const float* __restrict__ beta,
                                                   unsigned d, float eps, float* __restrict__ y,
                                                   float* __restrict__ partial) {
  __shared__ float row[kMaxRow];
  __shared__ float red[kT / kWave];
  const size_t m = blockIdx.x;
  float s = 0.f;
  for (unsigned j = threadIdx.x; j < d; j += kT) {
    float h;
    if (GATED) {
      const float x = a[m * d + j];
      h = sigmoidf_(z[m * 2 * d + j]) * x + sigmoidf_(z[m * 2 * d + d + j]) * f[m * d + j];
    } else {
      h = a[m * d + j];
    }
    h += r[m * d + j];
    row[j] = h;
    s += h;
  }
  const float mu = block_sum(s, red) / (float)d;
  float q = 0.f;
  for (unsigned j = threadIdx.x; j < d; j += kT) {
    const float c = row[j] - mu;
    q += c * c;
  }
  const float var = block_sum(q, red) / (float)d;
  const float inv = __fdiv_rn(1.0f, sqrtf(var + eps));
  float mx = 0.f;
  for (unsigned j = threadIdx.x; j < d; j += kT) {
    const float v = (row[j] - mu) * inv * gamma[j] + beta[j];
    y[m * d + j] = v;
    mx = fmaxf(mx, fabsf(v));
  }
  if (partial != nullptr) block_absmax_out(mx, red, partial);
}

// One workgroup per sentence.  Scores of all heads and source positions into LDS (one wave per (head,
// position) pair at a time, lanes over the head's width), softmax per head, then the context: thread j
// of the model width sums p[s] V[s][j] over the source positions.
__global__ __launch_bounds__(kT) void k_cross_attention(const float* __restrict__ q, const float* __restrict__ K,
                                                        const float* __restrict__ V, unsigned S, unsigned d,
                                                        unsigned heads, float* __restrict__ ctx,
                                                        float* __restrict__ partial) {
  __shared__ float sc[kMaxScores];
  __shared__ float red[kT / kWave];
  const size_t m = blockIdx.x;
  const unsigned dh = d / heads;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const float scale = __fdiv_rn(1.0f, sqrtf((float)dh));
  const float* qm = q + m * d;
  const float* Km = K + m * S * d;
  const float* Vm = V + m * S * d;
  for (unsigned p = wave; p < heads * S; p += kT / kWave) {
    const unsigned h = p / S, s = p % S;
    float acc = 0.f;
    for (unsigned j = lane; j < dh; j += kWave) acc = fmaf(qm[h * dh + j], Km[s * d + h * dh + j], acc);
    acc = wave_sum_f(acc);
    if (lane == 0) sc[p] = acc * scale;
  }
  __syncthreads();
  // softmax over the S positions of each head: one wave per head at a time
  for (unsigned h = wave; h < heads; h += kT / kWave) {
    float mx = -INFINITY;
    for (unsigned s = lane; s < S; s += kWave) mx = fmaxf(mx, sc[h * S + s]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    float sum = 0.f;
    for (unsigned s = lane; s < S; s += kWave) {
      const float e = expf(sc[h * S + s] - mx);
      sc[h * S + s] = e;
      sum += e;
    }
    sum = wave_sum_f(sum);
    const float inv = __fdiv_rn(1.0f, sum);
    for (unsigned s = lane; s < S; s += kWave) sc[h * S + s] *= inv;
  }
  __syncthreads();
  float mx = 0.f;
  for (unsigned j = threadIdx.x; j < d; j += kT) {
    const unsigned h = j / dh;
    float acc = 0.f;
    for (unsigned s = 0; s < S; ++s) acc = fmaf(sc[h * S + s], Vm[s * d + j], acc);
    ctx[m * d + j] = acc;
    mx = fmaxf(mx, fabsf(acc));
  }
  if (partial != nullptr) block_absmax_out(mx, red, partial);
}

}  // namespace

// The launchers' optional `partial` receives one max|output| per workgroup (glue_partials(...) of them).
size_t running_average_partials(size_t n) { return (n + kT - 1) / kT; }

int launch_running_average(const float* g_prev, const float* x, size_t n, int t, float* g, hipStream_t s, float* partial,
                           unsigned* clear, unsigned nclear) {
  const size_t blocks = (n + kT - 1) / kT;
  if (blocks > 0x7FFFFFFFull || nclear > (unsigned)kT) return MQ_ERR_SHAPE;
  hipLaunchKernelGGL(k_running_average, dim3((unsigned)blocks), dim3(kT), 0, s, g_prev, x, n, (float)(t - 1), (float)t, g,
                     partial, clear, nclear);
  return check_hip(hipGetLastError());
}

int launch_concat2(const float* a, size_t da, const float* b, size_t db, size_t M, float* out, hipStream_t s,
                   float* partial) {
  hipLaunchKernelGGL(k_concat2, dim3((unsigned)M), dim3(kT), 0, s, a, (unsigned)da, b, (unsigned)db, out, partial);
  return check_hip(hipGetLastError());
}

int launch_add_layer_norm(const float* a, const float* r, const float* gamma, const float* beta, size_t M, size_t d,
                          float eps, float* y, hipStream_t s, float* partial) {
  if (d > (size_t)kMaxRow) return MQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((k_layer_norm<false>), dim3((unsigned)M), dim3(kT), 0, s, a, (const float*)nullptr,
                     (const float*)nullptr, r, gamma, beta, (unsigned)d, eps, y, partial);
  return check_hip(hipGetLastError());
}

int launch_gate_mix_layer_norm(const float* x, const float* f, const float* z, const float* gamma, const float* beta,
                               size_t M, size_t d, float eps, float* y, hipStream_t s, float* partial) {
  if (d > (size_t)kMaxRow) return MQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((k_layer_norm<true>), dim3((unsigned)M), dim3(kT), 0, s, x, f, z, x, gamma, beta, (unsigned)d, eps, y,
                     partial);
  return check_hip(hipGetLastError());
}

int launch_cross_attention(const float* q, const float* K, const float* V, size_t M, size_t S, size_t d, int heads,
                           float* ctx, hipStream_t s, float* partial) {
  if ((size_t)heads * S > (size_t)kMaxScores) return MQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_cross_attention, dim3((unsigned)M), dim3(kT), 0, s, q, K, V, (unsigned)S, (unsigned)d,
                     (unsigned)heads, ctx, partial);
  return check_hip(hipGetLastError());
}

}  // namespace mq
