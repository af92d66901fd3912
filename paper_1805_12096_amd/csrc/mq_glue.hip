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
                                                        unsigned nclear, float* __restrict__ partial_x) {
  __shared__ float red[kT / kWave];
  const size_t i = (size_t)blockIdx.x * kT + threadIdx.x;
  float v = 0.f, xv = 0.f;
  if (i < n) {
    xv = x[i];
    v = __fdiv_rn(__fmaf_rn(tm1, g_prev[i], xv), t);
    g[i] = v;
  }
  if (clear != nullptr && blockIdx.x == 0 && threadIdx.x < nclear) clear[threadIdx.x] = 0u;   // later kernels' maxima
  if (partial != nullptr) block_absmax_out(fabsf(v), red, partial);       // fmaxf drops NaN
  // max|x| as well (the gate's product takes [x, f] as its input and needs the maximum of both halves)
  if (partial_x != nullptr) block_absmax_out(fabsf(xv), red, partial_x);
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
// position) pair, lanes over the head's width, four pairs per trip so that four rows of K are in flight
// per wave instead of one: the loop is bound by memory latency, not by arithmetic), softmax per head, then
// the context: thread j of the model width sums p[s] V[s][j] over the source positions.
constexpr int kTA = 512;             // threads of the attention kernel

__global__ __launch_bounds__(kTA) void k_cross_attention(const float* __restrict__ q, const float* __restrict__ K,
                                                         const float* __restrict__ V, unsigned S, unsigned d,
                                                         unsigned heads, float* __restrict__ ctx,
                                                         float* __restrict__ partial) {
  __shared__ float sc[kMaxScores];
  __shared__ float red[kTA / kWave];
  constexpr unsigned NWV = kTA / kWave;
  const size_t m = blockIdx.x;
  const unsigned dh = d / heads;
  const unsigned lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const float scale = __fdiv_rn(1.0f, sqrtf((float)dh));
  const float* qm = q + m * d;
  const float* Km = K + m * S * d;
  const float* Vm = V + m * S * d;
  const unsigned pairs = heads * S;
  for (unsigned p0 = wave; p0 < pairs; p0 += 4 * NWV) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (unsigned j = lane; j < dh; j += kWave) {
      float kv[4], qv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const unsigned p = p0 + u * NWV;
        const unsigned pc = p < pairs ? p : p0;                 // past the end: a valid pair again, result unused
        const unsigned h = pc / S, s = pc % S;
        kv[u] = Km[(size_t)s * d + h * dh + j];
        qv[u] = qm[h * dh + j];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = fmaf(qv[u], kv[u], acc[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float t = wave_sum_f(acc[u]);
      const unsigned p = p0 + u * NWV;
      if (lane == 0 && p < pairs) sc[p] = t * scale;
    }
  }
  __syncthreads();
  // softmax over the S positions of each head: one wave per head at a time
  for (unsigned h = wave; h < heads; h += NWV) {
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
  for (unsigned j = threadIdx.x; j < d; j += kTA) {
    const unsigned h = j / dh;
    float acc = 0.f;
    unsigned s = 0;
    for (; s + 4 <= S; s += 4) {                                   // four rows of V in flight
      const float v0 = Vm[(size_t)s * d + j], v1 = Vm[(size_t)(s + 1) * d + j], v2 = Vm[(size_t)(s + 2) * d + j],
                  v3 = Vm[(size_t)(s + 3) * d + j];
      acc = fmaf(sc[h * S + s], v0, acc);
      acc = fmaf(sc[h * S + s + 1], v1, acc);
      acc = fmaf(sc[h * S + s + 2], v2, acc);
      acc = fmaf(sc[h * S + s + 3], v3, acc);
    }
    for (; s < S; ++s) acc = fmaf(sc[h * S + s], Vm[(size_t)s * d + j], acc);
    ctx[m * d + j] = acc;
    mx = fmaxf(mx, fabsf(acc));
  }
  if (partial != nullptr) {
    // (the helper is written for kT threads; here the workgroup is kTA wide)
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    __syncthreads();
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
      float r = red[0];
#pragma unroll
      for (unsigned k = 1; k < NWV; ++k) r = fmaxf(r, red[k]);
      partial[blockIdx.x] = r;
    }
  }
}

// The same for the usual shapes (model width a multiple of 256, head width a power of two between 4 and 256):
// every load is a float4, a wave reads whole 1 KB pieces of a K row and all heads' partial dot products of one
// source position come out of one pass; the context phase splits the source positions over thread groups so
// that every thread has several rows of V in flight.
template <int CH>      // CH = d / 256: float4 pieces of a row per lane
__global__ __launch_bounds__(kTA) void k_cross_attention_fast(const float* __restrict__ q, const float* __restrict__ K,
                                                              const float* __restrict__ V, unsigned S, unsigned heads,
                                                              float* __restrict__ ctx, float* __restrict__ partial) {
  constexpr unsigned d = 256u * CH;
  constexpr unsigned NWV = kTA / kWave;
  constexpr unsigned COLS = d / 4;                 // float4 columns of a row
  constexpr unsigned SG = kTA / COLS;              // groups of threads that share the source positions
  static_assert(kTA % COLS == 0 && SG >= 1, "context phase layout");
  __shared__ float sc[kMaxScores];
  __shared__ float4 part[SG > 1 ? kTA : 1];
  __shared__ float red[NWV];
  const size_t m = blockIdx.x;
  const unsigned dh = d / heads, grp = dh / 4;     // lanes per head inside a 256-float piece
  const unsigned lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const float scale = __fdiv_rn(1.0f, sqrtf((float)dh));
  const float4* q4 = reinterpret_cast<const float4*>(q + m * d);
  const float4* K4 = reinterpret_cast<const float4*>(K + m * S * d);
  const float4* V4 = reinterpret_cast<const float4*>(V + m * S * d);
  float4 qr[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) qr[c] = q4[c * 64 + lane];
  for (unsigned s0 = wave; s0 < S; s0 += 4 * NWV) {
    float4 kr[4][CH];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const unsigned s = s0 + u * NWV < S ? s0 + u * NWV : s0;       // past the end: a valid row again, result unused
#pragma unroll
      for (int c = 0; c < CH; ++c) kr[u][c] = K4[(size_t)s * COLS + c * 64 + lane];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const unsigned s = s0 + u * NWV;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        float a = fmaf(qr[c].x, kr[u][c].x, fmaf(qr[c].y, kr[u][c].y, fmaf(qr[c].z, kr[u][c].z, qr[c].w * kr[u][c].w)));
        for (unsigned off = grp / 2; off >= 1; off >>= 1) a += __shfl_xor(a, off, kWave);
        const unsigned h = (c * 256 + 4 * lane) / dh;
        if (s < S && lane % grp == 0) sc[h * S + s] = a * scale;
      }
    }
  }
  __syncthreads();
  for (unsigned h = wave; h < heads; h += NWV) {
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
  const unsigned col = threadIdx.x % COLS, sg = threadIdx.x / COLS;
  const unsigned h = (4 * col) / dh;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  unsigned s = sg;
  for (; s + 3 * SG < S; s += 4 * SG) {
    const float4 v0 = V4[(size_t)s * COLS + col], v1 = V4[(size_t)(s + SG) * COLS + col],
                 v2 = V4[(size_t)(s + 2 * SG) * COLS + col], v3 = V4[(size_t)(s + 3 * SG) * COLS + col];
    const float p0 = sc[h * S + s], p1 = sc[h * S + s + SG], p2 = sc[h * S + s + 2 * SG], p3 = sc[h * S + s + 3 * SG];
    acc.x = fmaf(p3, v3.x, fmaf(p2, v2.x, fmaf(p1, v1.x, fmaf(p0, v0.x, acc.x))));
    acc.y = fmaf(p3, v3.y, fmaf(p2, v2.y, fmaf(p1, v1.y, fmaf(p0, v0.y, acc.y))));
    acc.z = fmaf(p3, v3.z, fmaf(p2, v2.z, fmaf(p1, v1.z, fmaf(p0, v0.z, acc.z))));
    acc.w = fmaf(p3, v3.w, fmaf(p2, v2.w, fmaf(p1, v1.w, fmaf(p0, v0.w, acc.w))));
  }
  for (; s < S; s += SG) {
    const float4 v0 = V4[(size_t)s * COLS + col];
    const float p0 = sc[h * S + s];
    acc.x = fmaf(p0, v0.x, acc.x);
    acc.y = fmaf(p0, v0.y, acc.y);
    acc.z = fmaf(p0, v0.z, acc.z);
    acc.w = fmaf(p0, v0.w, acc.w);
  }
  float mx = 0.f;
  if constexpr (SG > 1) {
    part[threadIdx.x] = acc;
    __syncthreads();
    if (sg == 0) {
#pragma unroll
      for (unsigned g = 1; g < SG; ++g) {
        const float4 o = part[g * COLS + col];
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
      }
    }
  }
  if (sg == 0) {
    reinterpret_cast<float4*>(ctx + m * d)[col] = acc;
    mx = fmaxf(fmaxf(fabsf(acc.x), fabsf(acc.y)), fmaxf(fabsf(acc.z), fabsf(acc.w)));
  }
  if (partial != nullptr) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    __syncthreads();
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
      float r = red[0];
#pragma unroll
      for (unsigned k = 1; k < NWV; ++k) r = fmaxf(r, red[k]);
      partial[blockIdx.x] = r;
    }
  }
}

}  // namespace

// The launchers' optional `partial` receives one max|output| per workgroup (glue_partials(...) of them).
size_t running_average_partials(size_t n) { return (n + kT - 1) / kT; }

int launch_running_average(const float* g_prev, const float* x, size_t n, int t, float* g, hipStream_t s, float* partial,
                           unsigned* clear, unsigned nclear, float* partial_x) {
  const size_t blocks = (n + kT - 1) / kT;
  if (blocks > 0x7FFFFFFFull || nclear > (unsigned)kT) return MQ_ERR_SHAPE;
  hipLaunchKernelGGL(k_running_average, dim3((unsigned)blocks), dim3(kT), 0, s, g_prev, x, n, (float)(t - 1), (float)t, g,
                     partial, clear, nclear, partial_x);
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
  const size_t dh = d / (size_t)heads;
  const bool pow2 = (dh & (dh - 1)) == 0;
  const bool vec_ok = (reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V) |
                       reinterpret_cast<uintptr_t>(ctx)) % 16 == 0;
  if (vec_ok && pow2 && dh >= 4 && dh <= 256 && (d == 256 || d == 512 || d == 1024)) {
    if (d == 256)
      hipLaunchKernelGGL((k_cross_attention_fast<1>), dim3((unsigned)M), dim3(kTA), 0, s, q, K, V, (unsigned)S,
                         (unsigned)heads, ctx, partial);
    else if (d == 512)
      hipLaunchKernelGGL((k_cross_attention_fast<2>), dim3((unsigned)M), dim3(kTA), 0, s, q, K, V, (unsigned)S,
                         (unsigned)heads, ctx, partial);
    else
      hipLaunchKernelGGL((k_cross_attention_fast<4>), dim3((unsigned)M), dim3(kTA), 0, s, q, K, V, (unsigned)S,
                         (unsigned)heads, ctx, partial);
    return check_hip(hipGetLastError());
  }
  hipLaunchKernelGGL(k_cross_attention, dim3((unsigned)M), dim3(kTA), 0, s, q, K, V, (unsigned)S, (unsigned)d,
                     (unsigned)heads, ctx, partial);
  return check_hip(hipGetLastError());
}

}  // namespace mq
