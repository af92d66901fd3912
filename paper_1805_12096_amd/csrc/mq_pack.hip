// Memoized quant_int(B^T) (arxiv 1805.12096, Section 4.3): quantize a float
// parameter once, transposed to [N x K], and store it in the fragment order the
// MFMA kernels consume.  Runs once per parameter, off the decode path, so the
// kernels here favour clarity: every thread produces one 16-byte lane slot.
#include "mq_internal.h"

namespace mq {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ int quant1(float x, float s, float lim) {
  const float r = rintf(__fmul_rn(x, s));
  const float c = fminf(fmaxf(r, -lim), lim);
  return (r != r) ? 0 : (int)c;
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void k_prepare(const float* __restrict__ B, int transposed,
                                                      size_t N, size_t K,
                                                      const float* __restrict__ scale,
                                                      uint8_t* __restrict__ packed) {
  const PackedDims d(BITS, N, K);
  const float s = *scale;
  const float lim = BITS == 8 ? 127.0f : 32767.0f;
  const size_t nslots = d.nblocks * d.kfrags * kWave;
  for (size_t slot = (size_t)blockIdx.x * kThreads + threadIdx.x; slot < nslots;
       slot += (size_t)gridDim.x * kThreads) {
    const int lane = (int)(slot % kWave);
    const size_t frag = slot / kWave;
    const size_t nb = frag / d.kfrags, kb = frag % d.kfrags;
    const size_t n = nb * kFragRows + lane % 32;
    const size_t k0 = kb * kFragK + 16 * (lane / 32);
    uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const size_t k = k0 + j;
      if (n < N && k < K) {
        const float x = transposed ? B[n * K + k] : B[k * N + n];
        const int q = quant1(x, s, lim);
        if (BITS == 8) {
          lo[j / 4] |= (uint32_t)(q & 0xFF) << (8 * (j % 4));
        } else {
          // q = 256 * h + l + 128 with h = q >> 8 and l = (q & 255) - 128, both int8
          hi[j / 4] |= (uint32_t)((q >> 8) & 0xFF) << (8 * (j % 4));
          lo[j / 4] |= (uint32_t)((q & 0xFF) ^ 0x80) << (8 * (j % 4));
        }
      }
    }
    uint8_t* dst = packed + d.frag_offset(nb, kb) + (size_t)lane * 16;
    if (BITS == 8) {
      *reinterpret_cast<uint4*>(dst) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    } else {
      *reinterpret_cast<uint4*>(dst) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      *reinterpret_cast<uint4*>(dst + kFragBytes) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
  }
}

// 16-bit only: colsum[n] = sum_k quant(Wt[n][k]) for n < N, 0 for padding rows.
__global__ __launch_bounds__(kThreads) void k_colsum(const float* __restrict__ B, int transposed,
                                                     size_t N, size_t K, size_t Np,
                                                     const float* __restrict__ scale,
                                                     int32_t* __restrict__ colsum) {
  const float s = *scale;
  const int lane = threadIdx.x % kWave;
  const size_t wave = (size_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
  const size_t nwaves = (size_t)gridDim.x * (kThreads / kWave);
  for (size_t n = wave; n < Np; n += nwaves) {
    int sum = 0;
    if (n < N)
      for (size_t k = lane; k < K; k += kWave)
        sum += quant1(transposed ? B[n * K + k] : B[k * N + n], s, 32767.0f);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, kWave);
    if (lane == 0) colsum[n] = sum;
  }
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void k_unpack(const uint8_t* __restrict__ packed, size_t N,
                                                     size_t K, void* __restrict__ q) {
  const PackedDims d(BITS, N, K);
  const size_t total = N * K;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (size_t)gridDim.x * kThreads) {
    const size_t n = i / K, k = i % K;
    const size_t nb = n / kFragRows, kb = k / kFragK;
    const int kk = (int)(k % kFragK);
    const int lane = (int)(n % kFragRows) + 32 * (kk / 16);
    const uint8_t* src = packed + d.frag_offset(nb, kb) + (size_t)lane * 16 + kk % 16;
    if (BITS == 8) {
      reinterpret_cast<int8_t*>(q)[i] = (int8_t)src[0];
    } else {
      const int h = (int8_t)src[0];
      const int l = (int8_t)src[kFragBytes];
      reinterpret_cast<int16_t*>(q)[i] = (int16_t)(256 * h + l + 128);
    }
  }
}

unsigned grid_for(size_t items) {
  size_t g = (items + kThreads - 1) / kThreads;
  if (g < 1) g = 1;
  if (g > 8192) g = 8192;
  return (unsigned)g;
}

}  // namespace

int launch_prepare(const float* B, int transposed, size_t N, size_t K, int bits, const float* scale,
                   void* packed, hipStream_t s) {
  const PackedDims d(bits, N, K);
  const unsigned grid = grid_for(d.nblocks * d.kfrags * kWave);
  uint8_t* p = static_cast<uint8_t*>(packed);
  if (bits == 8) {
    hipLaunchKernelGGL(k_prepare<8>, dim3(grid), dim3(kThreads), 0, s, B, transposed, N, K, scale, p);
  } else {
    hipLaunchKernelGGL(k_prepare<16>, dim3(grid), dim3(kThreads), 0, s, B, transposed, N, K, scale, p);
    int32_t* colsum = reinterpret_cast<int32_t*>(p + d.plane_bytes());
    const unsigned g2 = grid_for(d.Np * kWave);
    hipLaunchKernelGGL(k_colsum, dim3(g2), dim3(kThreads), 0, s, B, transposed, N, K, d.Np, scale, colsum);
  }
  return check_hip(hipGetLastError());
}

int launch_unpack(const void* packed, int bits, size_t N, size_t K, void* q, hipStream_t s) {
  const unsigned grid = grid_for(N * K);
  const uint8_t* p = static_cast<const uint8_t*>(packed);
  if (bits == 8) hipLaunchKernelGGL(k_unpack<8>, dim3(grid), dim3(kThreads), 0, s, p, N, K, q);
  else hipLaunchKernelGGL(k_unpack<16>, dim3(grid), dim3(kThreads), 0, s, p, N, K, q);
  return check_hip(hipGetLastError());
}

}  // namespace mq
