// quant_int on gfx950: per-tensor abs-max, multiplier, and the float -> int8 /
// int16 conversion (arxiv 1805.12096, Section 4.2).  All three are bound by HBM
// traffic: wide coalesced loads, one pass each.
#include "mq_grid_max.h"
#include "mq_internal.h"

namespace mq {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__global__ void k_fill_u32(uint32_t* p, uint32_t v) { *p = v; }
// Pseudo-random bytes (a hash of the word index): operand contents for timing runs.  The matrix units draw more
// power on varied operands than on constant ones and clock lower, so constant fill ranks tile variants wrongly.
__global__ void k_fill_pattern(uint32_t* p, size_t nwords, uint32_t seed) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride) {
    uint32_t x = (uint32_t)i * 2654435761u + seed;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16;
    p[i] = x;
  }
}

__global__ void k_clear_words(uint32_t* p, unsigned n) {
  for (unsigned i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

// |x| of a non-NaN float orders like its bit pattern, so the grid-wide maximum
// is an integer atomicMax.  fmaxf drops NaN operands.
// Workgroups of 1024 threads, at most 512 of them: every workgroup may end in one atomic on the same word,
// and those are served one after the other (2048 small workgroups ending together took 25 us for that alone).
constexpr int kAbsmaxThreads = 1024;
__global__ __launch_bounds__(kAbsmaxThreads) void k_absmax(const float* __restrict__ x, size_t n,
                                                           uint32_t* __restrict__ amax_bits) {
  constexpr int kThreads = kAbsmaxThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  const size_t nvec = n / 4;
  const float4* xv = reinterpret_cast<const float4*>(x);
  float m0 = 0.f, m1 = 0.f, m2 = 0.f, m3 = 0.f;
  size_t i = tid;
  for (; i + 3 * nthreads < nvec; i += 4 * nthreads) {
    float4 a = xv[i], b = xv[i + nthreads], c = xv[i + 2 * nthreads], d = xv[i + 3 * nthreads];
    m0 = fmaxf(m0, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
    m1 = fmaxf(m1, fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w))));
    m2 = fmaxf(m2, fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))));
    m3 = fmaxf(m3, fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w))));
  }
  for (; i < nvec; i += nthreads) {
    float4 a = xv[i];
    m0 = fmaxf(m0, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
  }
  for (size_t j = nvec * 4 + tid; j < n; j += nthreads) m1 = fmaxf(m1, fabsf(x[j]));
  float m = wave_max(fmaxf(fmaxf(m0, m1), fmaxf(m2, m3)));
  __shared__ float part[kThreads / kWave];
  const int lane = threadIdx.x % kWave, w = threadIdx.x / kWave;
  if (lane == 0) part[w] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = part[0];
#pragma unroll
    for (int k = 1; k < kThreads / kWave; ++k) r = fmaxf(r, part[k]);
    // the running maximum only grows: a block that cannot raise it skips the (serialising) atomic
    const uint32_t bits = __float_as_uint(r);
    if (bits > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits, bits);
  }
}

__global__ void k_scale(const float* __restrict__ amax, float qmax, float* __restrict__ scale) {
  const float a = *amax;
  *scale = (a > 0.0f) ? __fdiv_rn(qmax, a) : 1.0f;
}

// One element of quant_int: binary32 multiply, round half to even, symmetric
// clamp; NaN becomes 0.
__device__ __forceinline__ int quant1(float x, float s, float lim) {
  const float r = rintf(__fmul_rn(x, s));
  const float c = fminf(fmaxf(r, -lim), lim);
  return (r != r) ? 0 : (int)c;
}

__device__ __forceinline__ uint32_t pack4_i8(int a, int b, int c, int d) {
  return (uint32_t)(a & 0xFF) | ((uint32_t)(b & 0xFF) << 8) | ((uint32_t)(c & 0xFF) << 16) |
         ((uint32_t)(d & 0xFF) << 24);
}
__device__ __forceinline__ uint32_t pack2_i16(int a, int b) {
  return (uint32_t)(a & 0xFFFF) | ((uint32_t)(b & 0xFFFF) << 16);
}

// Flat conversion, 8 elements per thread and step: two 16-byte loads, one 8-byte
// (int8) or 16-byte (int16) store.
template <int BITS>
__global__ __launch_bounds__(kThreads) void k_quantize_flat(const float* __restrict__ x, size_t n,
                                                            const float* __restrict__ scale,
                                                            void* __restrict__ qv) {
  const float s = *scale;
  const float lim = BITS == 8 ? 127.0f : 32767.0f;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  const size_t nvec = n / 8;
  const float4* xv = reinterpret_cast<const float4*>(x);
  for (size_t i = tid; i < nvec; i += nthreads) {
    const float4 a = xv[2 * i], b = xv[2 * i + 1];
    const int q0 = quant1(a.x, s, lim), q1 = quant1(a.y, s, lim), q2 = quant1(a.z, s, lim),
              q3 = quant1(a.w, s, lim), q4 = quant1(b.x, s, lim), q5 = quant1(b.y, s, lim),
              q6 = quant1(b.z, s, lim), q7 = quant1(b.w, s, lim);
    if (BITS == 8) {
      uint2 o;
      o.x = pack4_i8(q0, q1, q2, q3);
      o.y = pack4_i8(q4, q5, q6, q7);
      reinterpret_cast<uint2*>(qv)[i] = o;
    } else {
      uint4 o;
      o.x = pack2_i16(q0, q1);
      o.y = pack2_i16(q2, q3);
      o.z = pack2_i16(q4, q5);
      o.w = pack2_i16(q6, q7);
      reinterpret_cast<uint4*>(qv)[i] = o;
    }
  }
  for (size_t j = nvec * 8 + tid; j < n; j += nthreads) {
    const int q = quant1(x[j], s, lim);
    if (BITS == 8) reinterpret_cast<int8_t*>(qv)[j] = (int8_t)q;
    else reinterpret_cast<int16_t*>(qv)[j] = (int16_t)q;
  }
}

// Row-wise conversion that also produces sum_c q[r][c]: one wavefront per row.
template <int BITS, bool VEC>
__global__ __launch_bounds__(kThreads) void k_quantize_rows(const float* __restrict__ x, size_t rows,
                                                            size_t cols, const float* __restrict__ scale,
                                                            void* __restrict__ qv,
                                                            int32_t* __restrict__ rowsum) {
  const float s = *scale;
  const float lim = BITS == 8 ? 127.0f : 32767.0f;
  const int lane = threadIdx.x % kWave;
  const size_t wave = (size_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
  const size_t nwaves = (size_t)gridDim.x * (kThreads / kWave);
  for (size_t r = wave; r < rows; r += nwaves) {
    const float* xr = x + r * cols;
    int sum = 0;
    if (VEC) {  // cols % 8 == 0 and 16-byte aligned rows
      const float4* xv = reinterpret_cast<const float4*>(xr);
      for (size_t i = lane; i < cols / 8; i += kWave) {
        const float4 a = xv[2 * i], b = xv[2 * i + 1];
        const int q0 = quant1(a.x, s, lim), q1 = quant1(a.y, s, lim), q2 = quant1(a.z, s, lim),
                  q3 = quant1(a.w, s, lim), q4 = quant1(b.x, s, lim), q5 = quant1(b.y, s, lim),
                  q6 = quant1(b.z, s, lim), q7 = quant1(b.w, s, lim);
        sum += q0 + q1 + q2 + q3 + q4 + q5 + q6 + q7;
        if (BITS == 8) {
          uint2 o;
          o.x = pack4_i8(q0, q1, q2, q3);
          o.y = pack4_i8(q4, q5, q6, q7);
          reinterpret_cast<uint2*>(reinterpret_cast<int8_t*>(qv) + r * cols)[i] = o;
        } else {
          uint4 o;
          o.x = pack2_i16(q0, q1);
          o.y = pack2_i16(q2, q3);
          o.z = pack2_i16(q4, q5);
          o.w = pack2_i16(q6, q7);
          reinterpret_cast<uint4*>(reinterpret_cast<int16_t*>(qv) + r * cols)[i] = o;
        }
      }
    } else {
      for (size_t c = lane; c < cols; c += kWave) {
        const int q = quant1(xr[c], s, lim);
        sum += q;
        if (BITS == 8) reinterpret_cast<int8_t*>(qv)[r * cols + c] = (int8_t)q;
        else reinterpret_cast<int16_t*>(qv)[r * cols + c] = (int16_t)q;
      }
    }
    sum = wave_sum(sum);
    if (lane == 0) rowsum[r] = sum;
  }
}

unsigned grid_for(size_t work_items, size_t per_block, unsigned cap) {
  size_t g = (work_items + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (unsigned)g;
}

}  // namespace

int launch_absmax(const float* x, size_t n, float* amax, hipStream_t s) {
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(1), 0, s, reinterpret_cast<uint32_t*>(amax), 0u);
  // 16 floats per thread and pass; at most two workgroups per compute unit
  const unsigned grid = grid_for(n, (size_t)kAbsmaxThreads * 16, 512);
  hipLaunchKernelGGL(k_absmax, dim3(grid), dim3(kAbsmaxThreads), 0, s, x, n, reinterpret_cast<uint32_t*>(amax));
  return check_hip(hipGetLastError());
}

int launch_scale(const float* amax, int bits, float* scale, hipStream_t s) {
  hipLaunchKernelGGL(k_scale, dim3(1), dim3(1), 0, s, amax, (float)qmax_of(bits), scale);
  return check_hip(hipGetLastError());
}

int launch_quantize(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                    void* q, int32_t* rowsum, hipStream_t s) {
  if (rowsum == nullptr) {
    const size_t n = rows * cols;
    const unsigned grid = grid_for(n, (size_t)kThreads * 8, 4096);
    if (bits == 8)
      hipLaunchKernelGGL(k_quantize_flat<8>, dim3(grid), dim3(kThreads), 0, s, x, n, scale, q);
    else
      hipLaunchKernelGGL(k_quantize_flat<16>, dim3(grid), dim3(kThreads), 0, s, x, n, scale, q);
  } else {
    const bool vec = (cols % 8 == 0);
    const unsigned grid = grid_for(rows, kThreads / kWave, 4096);
    if (bits == 8) {
      if (vec) hipLaunchKernelGGL((k_quantize_rows<8, true>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, q, rowsum);
      else hipLaunchKernelGGL((k_quantize_rows<8, false>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, q, rowsum);
    } else {
      if (vec) hipLaunchKernelGGL((k_quantize_rows<16, true>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, q, rowsum);
      else hipLaunchKernelGGL((k_quantize_rows<16, false>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, q, rowsum);
    }
  }
  return check_hip(hipGetLastError());
}

}  // namespace mq

// ---------------------------------------------------------------------------
// quant_int straight into the fragment order the product kernels read (the
// same layout as a prepared parameter, see PackedDims): the activations then
// reach LDS by plain linear copies.  Eight lanes share a row and walk along K
// four floats at a time, so reads are whole 128-byte lines and each store
// instruction writes two 128-byte runs.
namespace mq {
namespace {

// Abs-max without atomics or initialisation: block b writes its maximum to partial[b];
// the consumer reduces the few hundred values itself (block_max_of_partials).
__global__ __launch_bounds__(kThreads) void k_absmax_partial(const float* __restrict__ x, size_t n,
                                                             float* __restrict__ partial, unsigned* clear, unsigned nclear) {
  if (clear != nullptr && blockIdx.x == 0)                 // a later kernel's counters
    for (unsigned i = threadIdx.x; i < nclear; i += kThreads) clear[i] = 0u;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  const size_t nvec = n / 4;
  const float4* xv = reinterpret_cast<const float4*>(x);
  float m0 = 0.f, m1 = 0.f;
  size_t i = tid;
  for (; i + nthreads < nvec; i += 2 * nthreads) {
    const float4 a = xv[i], b = xv[i + nthreads];
    m0 = fmaxf(m0, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
    m1 = fmaxf(m1, fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w))));
  }
  for (; i < nvec; i += nthreads) {
    const float4 a = xv[i];
    m0 = fmaxf(m0, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
  }
  for (size_t j = nvec * 4 + tid; j < n; j += nthreads) m1 = fmaxf(m1, fabsf(x[j]));
  const float m = wave_max(fmaxf(m0, m1));
  __shared__ float part[kThreads / kWave];
  const int lane = threadIdx.x % kWave, w = threadIdx.x / kWave;
  if (lane == 0) part[w] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = part[0];
#pragma unroll
    for (int k = 1; k < kThreads / kWave; ++k) r = fmaxf(r, part[k]);
    partial[blockIdx.x] = r;
  }
}

// Maximum of `count` partial maxima, computed redundantly by every block that needs it.
__device__ __forceinline__ float block_max_of_partials(const float* __restrict__ partial, unsigned count) {
  float m = 0.f;
  for (unsigned i = threadIdx.x; i < count; i += kThreads) m = fmaxf(m, partial[i]);
  m = wave_max(m);
  __shared__ float red[kThreads / kWave];
  if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = m;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int k = 1; k < kThreads / kWave; ++k) r = fmaxf(r, red[k]);
  return r;
}

// FROM_PARTIALS: `scale` holds `npartial` partial abs-maxima instead of the multiplier; the
// multiplier Qmax / max is formed here (one correctly rounded division) and block 0 also
// publishes it in scale_out[0] for the product kernels that follow.
template <int BITS, bool VEC, bool FROM_PARTIALS>
__global__ __launch_bounds__(kThreads) void k_quantize_pack(const float* __restrict__ x, size_t rows,
                                                            size_t cols, const float* __restrict__ scale,
                                                            uint8_t* __restrict__ packed, unsigned ksplit,
                                                            unsigned npartial, float* __restrict__ scale_out) {
  const PackedDims d(BITS, rows, cols);
  float s;
  if (FROM_PARTIALS) {
    const float amax = block_max_of_partials(scale, npartial);
    s = (amax > 0.0f) ? __fdiv_rn(BITS == 8 ? 127.0f : 32767.0f, amax) : 1.0f;
    if (blockIdx.x == 0 && threadIdx.x == 0) *scale_out = s;
  } else {
    s = *scale;
  }
  const float lim = BITS == 8 ? 127.0f : 32767.0f;
  const int lane = threadIdx.x % kWave;
  const int sub = lane % 8;                       // which 4 floats of a 32-element fragment row
  const size_t wave = (size_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
  const size_t nwaves = (size_t)gridDim.x * (kThreads / kWave);
  const size_t row_groups = d.Np / 8;
  const size_t per = (d.kfrags + ksplit - 1) / ksplit;   // fragments along K per work item
  // fragments [part * per, ...) of row group rg; returns the lane's share of the rows' sums (16 bit)
  auto convert = [&](size_t rg, size_t part) -> int {
    const size_t row = rg * 8 + lane / 8;
    const size_t kb_end = (part + 1) * per < d.kfrags ? (part + 1) * per : d.kfrags;
    const size_t nb = row / kFragRows;
    const int slot = (int)(row % kFragRows) + 32 * (sub / 4);
    int sum = 0;
    // four fragments per trip: all four loads are issued before the first conversion, so several
    // 128-byte lines per row are in flight instead of one
    for (size_t kb0 = part * per; kb0 < kb_end; kb0 += 4) {
      float4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const size_t k = (kb0 + j) * kFragK + 4 * sub;
        v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (kb0 + j < kb_end && row < rows) {
          if (VEC) {
            if (k < cols) v[j] = *reinterpret_cast<const float4*>(x + row * cols + k);
          } else {
            const float* xr = x + row * cols;
            if (k + 0 < cols) v[j].x = xr[k + 0];
            if (k + 1 < cols) v[j].y = xr[k + 1];
            if (k + 2 < cols) v[j].z = xr[k + 2];
            if (k + 3 < cols) v[j].w = xr[k + 3];
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (kb0 + j >= kb_end) break;
        const int q0 = quant1(v[j].x, s, lim), q1 = quant1(v[j].y, s, lim), q2 = quant1(v[j].z, s, lim),
                  q3 = quant1(v[j].w, s, lim);
        uint8_t* dst = packed + d.frag_offset(nb, kb0 + j) + (size_t)slot * 16 + 4 * (sub % 4);
        if (BITS == 8) {
          *reinterpret_cast<uint32_t*>(dst) = pack4_i8(q0, q1, q2, q3);
        } else {
          sum += q0 + q1 + q2 + q3;
          // q = 256 h + l + 128: high bytes, and low bytes with the top bit flipped
          *reinterpret_cast<uint32_t*>(dst) = pack4_i8(q0 >> 8, q1 >> 8, q2 >> 8, q3 >> 8);
          *reinterpret_cast<uint32_t*>(dst + kFragBytes) = pack4_i8(q0, q1, q2, q3) ^ 0x80808080u;
        }
      }
    }
    if (BITS == 16) {
      sum += __shfl_xor(sum, 1, kWave);
      sum += __shfl_xor(sum, 2, kWave);
      sum += __shfl_xor(sum, 4, kWave);
    }
    return sum;
  };
  if (BITS == 16 && ksplit > 1) {
    // 16 bit, long rows: the workgroup's waves share a row group, each takes its part of K (four times the loads in
    // flight of one wave per row group, which leaves a chip with a thousand row groups at four waves per compute
    // unit), and the rows' sums meet in LDS.  ksplit is the number of waves of the workgroup here.
    __shared__ int s_part[kThreads / kWave][8];
    const int w = threadIdx.x / kWave;
    for (size_t rg = blockIdx.x; rg < row_groups; rg += gridDim.x) {
      const int sum = convert(rg, (size_t)w);
      if (sub == 0) s_part[w][lane / 8] = sum;
      __syncthreads();
      if (w == 0 && sub == 0) {
        int total = 0;
#pragma unroll
        for (int k = 0; k < kThreads / kWave; ++k) total += s_part[k][lane / 8];
        reinterpret_cast<int32_t*>(packed + d.plane_bytes())[rg * 8 + lane / 8] = total;
      }
      __syncthreads();
    }
    return;
  }
  for (size_t item = wave; item < row_groups * ksplit; item += nwaves) {
    const size_t rg = item / ksplit, part = item % ksplit;
    const int sum = convert(rg, part);
    // 16 bit here: one wave owns whole rows
    if (BITS == 16 && sub == 0) reinterpret_cast<int32_t*>(packed + d.plane_bytes())[rg * 8 + lane / 8] = sum;
  }
}


// abs-max + quant_int in ONE launch for tensors whose elements all fit the registers of one resident
// grid: every wave loads its share (8 rows x 4 NI fragments), the workgroups agree on max|x| (see
// mq_grid_max.h), and the share is converted from registers.  Same work split, rounding and layout as
// k_quantize_pack; x is read once instead of twice and one kernel boundary disappears.
template <int BITS, bool VEC, int NI>
__global__ __launch_bounds__(512) void k_absmax_quantize_pack(const float* __restrict__ x, size_t rows, size_t cols,
                                                              uint8_t* __restrict__ packed, unsigned ksplit,
                                                              unsigned* barrier, unsigned long long ticks,
                                                              float* __restrict__ scale_out, unsigned* clear_words,
                                                              unsigned nclear, int self_clean) {
  constexpr int kW = 512 / kWave;
  // words a LATER kernel's agreement wants zero (not the ones used below): a caller that keeps its agreement
  // areas clean from call to call has this kernel and the next one clear each other's
  if (clear_words != nullptr && blockIdx.x == 0)
    for (unsigned i = threadIdx.x; i < nclear; i += 512) clear_words[i] = 0u;
  const PackedDims d(BITS, rows, cols);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int sub = lane % 8;                       // which 4 floats of a 32-element fragment row
  const size_t row_groups = d.Np / 8;
  const size_t per = (d.kfrags + ksplit - 1) / ksplit;   // fragments along K per wave, at most 4 NI
  const size_t item = (size_t)blockIdx.x * kW + wave;
  const bool active = item < row_groups * ksplit;
  const size_t rg = item / ksplit, part = item % ksplit;
  const size_t row = rg * 8 + lane / 8;
  const size_t kb_begin = part * per;
  const size_t kb_end = (part + 1) * per < d.kfrags ? (part + 1) * per : d.kfrags;
  float4 v[NI][4];
  float m = 0.f;
#pragma unroll
  for (int t = 0; t < NI; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const size_t kb = kb_begin + 4 * t + j;
      const size_t k = kb * kFragK + 4 * sub;
      v[t][j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (active && kb < kb_end && row < rows) {
        if (VEC) {
          if (k < cols) v[t][j] = *reinterpret_cast<const float4*>(x + row * cols + k);
        } else {
          const float* xr = x + row * cols;
          if (k + 0 < cols) v[t][j].x = xr[k + 0];
          if (k + 1 < cols) v[t][j].y = xr[k + 1];
          if (k + 2 < cols) v[t][j].z = xr[k + 2];
          if (k + 3 < cols) v[t][j].w = xr[k + 3];
        }
      }
    }
#pragma unroll
  for (int t = 0; t < NI; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      m = fmaxf(m, fmaxf(fmaxf(fabsf(v[t][j].x), fabsf(v[t][j].y)), fmaxf(fabsf(v[t][j].z), fabsf(v[t][j].w))));
  m = __uint_as_float(wave_max_u32(__float_as_uint(m)));      // m >= 0 and never NaN (fmaxf drops NaN operands)
  __shared__ float red[kW];
  if (lane == 0) red[wave] = m;
  __syncthreads();
  if (wave == 0) {
    float b = red[0];
#pragma unroll
    for (int w = 1; w < kW; ++w) b = fmaxf(b, red[w]);
    if (lane == 0) grid_max_publish(barrier, b);
    const float amax = grid_max_collect(barrier, ticks);
    if (lane == 0) red[0] = amax;
  }
  __syncthreads();
  const float amax = red[0];
  // self_clean: the agreement area is left all zero.  Every workgroup but the first is done with it here (its
  // count goes out now and is looked at after the stores); the first still has to look at the sticky word.
  unsigned retired_before = 0u;
  if (self_clean && blockIdx.x != 0 && threadIdx.x == 0) retired_before = grid_max_retire(barrier);
  const float lim = BITS == 8 ? 127.0f : 32767.0f;
  const float s = (amax > 0.0f) ? __fdiv_rn(lim, amax) : 1.0f;
  int sum = 0;
  if (active) {
    const size_t nb = row / kFragRows;
    const int slot = (int)(row % kFragRows) + 32 * (sub / 4);
#pragma unroll
    for (int t = 0; t < NI; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const size_t kb = kb_begin + 4 * t + j;
        if (kb < kb_end) {
          const int q0 = quant1(v[t][j].x, s, lim), q1 = quant1(v[t][j].y, s, lim), q2 = quant1(v[t][j].z, s, lim),
                    q3 = quant1(v[t][j].w, s, lim);
          uint8_t* dst = packed + d.frag_offset(nb, kb) + (size_t)slot * 16 + 4 * (sub % 4);
          if (BITS == 8) {
            *reinterpret_cast<uint32_t*>(dst) = pack4_i8(q0, q1, q2, q3);
          } else {
            sum += q0 + q1 + q2 + q3;
            // q = 256 h + l + 128: high bytes, and low bytes with the top bit flipped
            *reinterpret_cast<uint32_t*>(dst) = pack4_i8(q0 >> 8, q1 >> 8, q2 >> 8, q3 >> 8);
            *reinterpret_cast<uint32_t*>(dst + kFragBytes) = pack4_i8(q0, q1, q2, q3) ^ 0x80808080u;
          }
        }
      }
  }
  if (BITS == 16) {
    sum += __shfl_xor(sum, 1, kWave);
    sum += __shfl_xor(sum, 2, kWave);
    sum += __shfl_xor(sum, 4, kWave);
    if (ksplit > 1) {
      // the ksplit waves that share a row group sit side by side in the workgroup (ksplit divides its eight waves):
      // their parts of the rows' sums meet in LDS
      __shared__ int s_rowpart[kW][8];
      if (sub == 0) s_rowpart[wave][lane / 8] = sum;
      __syncthreads();
      if (active && part == 0 && sub == 0) {
        int total = 0;
        for (unsigned j = 0; j < ksplit; ++j) total += s_rowpart[wave + j][lane / 8];
        reinterpret_cast<int32_t*>(packed + d.plane_bytes())[row] = total;
      }
    } else if (active && sub == 0) {
      reinterpret_cast<int32_t*>(packed + d.plane_bytes())[row] = sum;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *scale_out = grid_max_failed(barrier) ? __builtin_nanf("") : s;
    if (self_clean) retired_before = grid_max_retire(barrier);
  }
  if (self_clean) {
    __shared__ unsigned last;
    if (threadIdx.x == 0) last = retired_before == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (last != 0u)
      for (unsigned i = threadIdx.x; i < kBarrierWords; i += 512) barrier[i] = 0u;
  }
}

}  // namespace

int launch_quantize_pack(const float* x, size_t rows, size_t cols, int bits, const float* scale,
                         void* packed, hipStream_t s) {
  const PackedDims d(bits, rows, cols);
  const size_t row_groups = d.Np / 8;
  // 8-bit: split K so that even a 300-row batch fills the chip; 16-bit: rows of 512 elements or more are shared by the
  // waves of a workgroup (their sums meet in LDS), shorter ones stay whole
  unsigned ksplit = 1;
  if (bits == 8) {
    while (row_groups * ksplit < 2048 && ksplit * 4 <= d.kfrags) ksplit *= 2;
  } else if (d.kfrags >= 16) {
    ksplit = kThreads / kWave;
  }
  const unsigned grid = bits == 16 && ksplit > 1 ? grid_for(row_groups, 1, 8192) : grid_for(row_groups * ksplit, kThreads / kWave, 8192);
  uint8_t* p = static_cast<uint8_t*>(packed);
  const bool vec = cols % 4 == 0;
  float* none = nullptr;
  if (bits == 8) {
    if (vec) hipLaunchKernelGGL((k_quantize_pack<8, true, false>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, p, ksplit, 0u, none);
    else hipLaunchKernelGGL((k_quantize_pack<8, false, false>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, p, ksplit, 0u, none);
  } else {
    if (vec) hipLaunchKernelGGL((k_quantize_pack<16, true, false>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, p, ksplit, 0u, none);
    else hipLaunchKernelGGL((k_quantize_pack<16, false, false>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, scale, p, ksplit, 0u, none);
  }
  return check_hip(hipGetLastError());
}

int launch_fill_pattern(void* p, size_t bytes, unsigned seed, hipStream_t s) {
  const size_t nwords = bytes / 4;
  if (nwords == 0) return MQ_OK;
  const unsigned grid = grid_for(nwords, 256 * 8, 2048);
  hipLaunchKernelGGL(k_fill_pattern, dim3(grid), dim3(256), 0, s, static_cast<uint32_t*>(p), nwords, seed);
  return check_hip(hipGetLastError());
}

int launch_clear_words(unsigned* p, unsigned n, hipStream_t s) {
  hipLaunchKernelGGL(k_clear_words, dim3(1), dim3(256), 0, s, reinterpret_cast<uint32_t*>(p), n);
  return check_hip(hipGetLastError());
}

// quant_int into the packed layout with the multiplier formed in the kernel from `npartials` partial
// maxima (one is enough: a single max|x| in device memory); scale_out[0] receives the multiplier.
int launch_quantize_pack_partials(const float* x, size_t rows, size_t cols, int bits, const float* partials,
                                  unsigned npartials, float* scale_out, void* packed, hipStream_t s) {
  const unsigned g1 = npartials;
  const PackedDims d(bits, rows, cols);
  const size_t row_groups = d.Np / 8;
  unsigned ksplit = 1;
  if (bits == 8) {
    while (row_groups * ksplit < 2048 && ksplit * 4 <= d.kfrags) ksplit *= 2;
  } else if (d.kfrags >= 16) {
    ksplit = kThreads / kWave;      // the workgroup's waves share a row group
  }
  const unsigned grid = bits == 16 && ksplit > 1 ? grid_for(row_groups, 1, 8192) : grid_for(row_groups * ksplit, kThreads / kWave, 8192);
  uint8_t* p = static_cast<uint8_t*>(packed);
  const bool vec = cols % 4 == 0;
  if (bits == 8) {
    if (vec) hipLaunchKernelGGL((k_quantize_pack<8, true, true>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, partials, p, ksplit, g1, scale_out);
    else hipLaunchKernelGGL((k_quantize_pack<8, false, true>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, partials, p, ksplit, g1, scale_out);
  } else {
    if (vec) hipLaunchKernelGGL((k_quantize_pack<16, true, true>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, partials, p, ksplit, g1, scale_out);
    else hipLaunchKernelGGL((k_quantize_pack<16, false, true>), dim3(grid), dim3(kThreads), 0, s, x, rows, cols, partials, p, ksplit, g1, scale_out);
  }
  return check_hip(hipGetLastError());
}

namespace {
template <int BITS, bool VEC, int NI>
int launch_fused_one(const float* x, size_t rows, size_t cols, uint8_t* packed, unsigned ksplit, unsigned grid,
                     unsigned* barrier, float* scale_out, hipStream_t s, unsigned* clear_words, unsigned nclear,
                     int self_clean) {
  auto kern = k_absmax_quantize_pack<BITS, VEC, NI>;
  static int max_blocks = -1;       // workgroups the device can hold at once, asked once
  if (max_blocks < 0) {
    int per_cu = 0, dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern), 512, 0) != hipSuccess)
      return MQ_ERR_HIP;
    max_blocks = per_cu * cus;
  }
  if (grid > (unsigned)max_blocks) return MQ_ERR_UNSUPPORTED;     // the grid-wide wait needs every workgroup resident
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 0, s, x, rows, cols, packed, ksplit, barrier, barrier_timeout_ticks(),
                     scale_out, clear_words, nclear, self_clean);
  return check_hip(hipGetLastError());
}

template <int BITS, bool VEC>
int launch_fused_ni(int ni, const float* x, size_t rows, size_t cols, uint8_t* packed, unsigned ksplit, unsigned grid,
                    unsigned* barrier, float* scale_out, hipStream_t s, unsigned* clear_words, unsigned nclear,
                    int self_clean) {
  switch (ni) {
    case 1: return launch_fused_one<BITS, VEC, 1>(x, rows, cols, packed, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean);
    case 2: return launch_fused_one<BITS, VEC, 2>(x, rows, cols, packed, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean);
    case 4: return launch_fused_one<BITS, VEC, 4>(x, rows, cols, packed, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean);
    default: return launch_fused_one<BITS, VEC, 8>(x, rows, cols, packed, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean);
  }
}
}  // namespace

// abs-max + quant_int into the packed layout in ONE launch, for tensors small enough to sit in the
// registers of one resident grid (at most 256 workgroups of 8 waves, at most 32 fragments along K per
// wave): MQ_ERR_UNSUPPORTED otherwise, nothing launched.  The kBarrierWords words at `barrier` must be
// zero when the kernel starts.  scale_out[0] receives the multiplier (NaN if the grid-wide wait failed).
int launch_absmax_quantize_pack_fused(const float* x, size_t rows, size_t cols, int bits, unsigned* barrier,
                                      float* scale_out, void* packed, hipStream_t s, unsigned* clear_words,
                                      unsigned nclear, int self_clean) {
  const PackedDims d(bits, rows, cols);
  const size_t row_groups = d.Np / 8;
  const size_t max_waves = (size_t)kBarrierSlots * (512 / kWave);
  if (row_groups > max_waves) return MQ_ERR_UNSUPPORTED;
  // split K as far as one trip of four fragments per wave allows while the waves still fit; 16 bit: at most over
  // the eight waves of a workgroup, where the parts of a row's sum meet in LDS
  unsigned ksplit = 1;
  while (row_groups * ksplit * 2 <= max_waves && (d.kfrags + 2 * ksplit - 1) / (2 * ksplit) >= 4 &&
         (bits == 8 || ksplit * 2 <= 512 / kWave))
    ksplit *= 2;
  const size_t per = (d.kfrags + ksplit - 1) / ksplit;
  if (per > 32) return MQ_ERR_UNSUPPORTED;
  const int ni = per <= 4 ? 1 : per <= 8 ? 2 : per <= 16 ? 4 : 8;
  const unsigned grid = (unsigned)((row_groups * ksplit + 512 / kWave - 1) / (512 / kWave));
  uint8_t* p = static_cast<uint8_t*>(packed);
  const bool vec = cols % 4 == 0;
  if (bits == 8) {
    return vec ? launch_fused_ni<8, true>(ni, x, rows, cols, p, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean)
               : launch_fused_ni<8, false>(ni, x, rows, cols, p, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean);
  }
  return vec ? launch_fused_ni<16, true>(ni, x, rows, cols, p, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean)
             : launch_fused_ni<16, false>(ni, x, rows, cols, p, ksplit, grid, barrier, scale_out, s, clear_words, nclear, self_clean);
}

// abs-max + quant_int into the packed layout in two launches, no atomics, no fill:
// partial maxima to `partials` (kAbsmaxPartials floats), then quantization with the multiplier
// formed from them; scale_out[0] receives the multiplier.
// Partial maxima of |x| only (at most kAbsmaxPartials of them); *count receives how many were written.
int launch_absmax_partials(const float* x, size_t n, float* partials, unsigned* count, hipStream_t s) {
  const unsigned g1 = grid_for(n, (size_t)kThreads * 8, kAbsmaxPartials);
  hipLaunchKernelGGL(k_absmax_partial, dim3(g1), dim3(kThreads), 0, s, x, n, partials, (unsigned*)nullptr, 0u);
  *count = g1;
  return check_hip(hipGetLastError());
}

int launch_absmax_quantize_pack(const float* x, size_t rows, size_t cols, int bits, float* partials,
                                float* scale_out, void* packed, hipStream_t s, unsigned* clear, unsigned nclear) {
  const size_t n = rows * cols;
  const unsigned g1 = grid_for(n, (size_t)kThreads * 8, kAbsmaxPartials);
  hipLaunchKernelGGL(k_absmax_partial, dim3(g1), dim3(kThreads), 0, s, x, n, partials, clear, nclear);
  return launch_quantize_pack_partials(x, rows, cols, bits, partials, g1, scale_out, packed, s);
}

}  // namespace mq
