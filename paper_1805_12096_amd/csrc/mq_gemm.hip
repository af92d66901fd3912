// dot'_int on gfx950 (arxiv 1805.12096, Sections 4.2 and 4.3): C = qA . Wt^T with
// 32-bit sums on the int8 matrix cores (v_mfma_i32_32x32x32_i8), and the fused
// epilogues: raw sums, dequantize + bias (+ReLU) (+abs-max of the result), and
// the beam-1 arg-max of Section 2.3.
//
// Both operands are contiguous along K, so a fragment for the 32x32x32 MFMA is
// "lane l holds 16 consecutive bytes of row l % 32 starting at 16 (l / 32)" for
// either operand.  Because the same rule serves A and Wt, the two can swap roles
// in the instruction: (a = A, b = Wt) puts consecutive n on consecutive lanes
// (coalesced stores of Y), (a = Wt, b = A) puts all candidates n of one sentence
// into the registers of one lane (arg-max without cross-lane traffic).
//
// 16-bit operands run as four 8-bit products.  With q = 256 h + l + 128,
// h = q >> 8, l = (q & 255) - 128 (both fit int8 for every int16 q):
//   sum_k a b = 2^16 sum(ha hb) + 2^8 sum(ha lb + la hb) + sum(la lb)
//               + 128 (sum_k a + sum_k b) - 16384 K          (mod 2^32)
// The three partial sums stay below 2^31 for K <= 2^16, so only the final
// combination wraps, exactly as a 32-bit accumulator would.
#include <type_traits>

#include "mq_internal.h"

namespace mq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;               // contracted elements staged per step
constexpr int kLdsStride = kBK + 16;  // bytes per staged row; odd multiple of 16 => conflict-free b128 reads

struct Params {
  const uint8_t* qA;
  const int32_t* rowsumA;
  const uint8_t* packedW;
  unsigned M, N, K;
  unsigned tiles_n;
  int32_t* C;
  const float* sA;
  const float* sW;
  const float* bias;
  int relu;
  float* Y;
  float* out_amax;
  unsigned long long* keys;
};

__device__ __forceinline__ v4i as_v4i(uint4 v) {
  v4i r;
  r.x = (int)v.x; r.y = (int)v.y; r.z = (int)v.z; r.w = (int)v.w;
  return r;
}

// 8 consecutive int16 (two dwords pairs) -> 4 high bytes and 4 low bytes per dword pair
__device__ __forceinline__ void split16(uint32_t d0, uint32_t d1, uint32_t& hi, uint32_t& lo) {
  hi = ((d0 >> 8) & 0xFFu) | ((d0 >> 24) << 8) | (((d1 >> 8) & 0xFFu) << 16) | ((d1 >> 24) << 24);
  lo = ((d0 & 0xFFu) | (((d0 >> 16) & 0xFFu) << 8) | ((d1 & 0xFFu) << 16) | (((d1 >> 16) & 0xFFu) << 24)) ^
       0x80808080u;
}

template <int BITS, int BM, int BN, int WM, int WN, int EPI, bool KVEC>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm(const Params p) {
  constexpr int NT = WM * WN * 64;
  constexpr int NPL = BITS == 16 ? 2 : 1;
  constexpr int TM = BM / WM / 32;
  constexpr int TN = BN / WN / 32;
  constexpr int NACC = BITS == 16 ? 3 : 1;
  constexpr int CHUNKS = BM * (kBK / 16);
  constexpr int CPT = (CHUNKS + NT - 1) / NT;
  constexpr bool SWAP = EPI == kEpiArgmax;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");

  __shared__ __attribute__((aligned(16))) uint8_t lds[2][NPL][BM][kLdsStride];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = tid / 64;
  const int wm = wave / WN, wn = wave % WN;
  const unsigned tile_m = blockIdx.x / p.tiles_n, tile_n = blockIdx.x % p.tiles_n;
  const unsigned m0 = tile_m * BM, n0 = tile_n * BN;
  const PackedDims d(BITS, p.N, p.K);
  const unsigned KT = (unsigned)(d.Kp / kBK);

  // ---- staging of A: global -> registers -> LDS ---------------------------
  uint4 stage[CPT][NPL];
  auto load_a = [&](unsigned kt) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * NT;
      const unsigned row = m0 + c / (kBK / 16);
      const unsigned k = kt * kBK + (c % (kBK / 16)) * 16;
      uint4 v0 = make_uint4(0, 0, 0, 0), v1 = make_uint4(0, 0, 0, 0);
      if (c < CHUNKS && row < p.M && k < p.K) {
        if (KVEC) {
          const uint4* src = reinterpret_cast<const uint4*>(p.qA + ((size_t)row * p.K + k) * (BITS / 8));
          v0 = src[0];
          if (BITS == 16) v1 = src[1];
        } else {
          uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            if (k + j < p.K) {
              if (BITS == 8) {
                w[j / 4] |= (uint32_t)p.qA[(size_t)row * p.K + k + j] << (8 * (j % 4));
              } else {
                const uint16_t e = reinterpret_cast<const uint16_t*>(p.qA)[(size_t)row * p.K + k + j];
                w[j / 2] |= (uint32_t)e << (16 * (j % 2));
              }
            }
          }
          v0 = make_uint4(w[0], w[1], w[2], w[3]);
          v1 = make_uint4(w[4], w[5], w[6], w[7]);
        }
      }
      if constexpr (BITS == 8) {
        stage[i][0] = v0;
      } else {
        uint4 hi, lo;
        split16(v0.x, v0.y, hi.x, lo.x);
        split16(v0.z, v0.w, hi.y, lo.y);
        split16(v1.x, v1.y, hi.z, lo.z);
        split16(v1.z, v1.w, hi.w, lo.w);
        stage[i][0] = hi;
        stage[i][NPL - 1] = lo;
      }
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * NT;
      if (c < CHUNKS) {
#pragma unroll
        for (int pl = 0; pl < NPL; ++pl)
          *reinterpret_cast<uint4*>(&lds[buf][pl][c / (kBK / 16)][(c % (kBK / 16)) * 16]) = stage[i][pl];
      }
    }
  };

  // ---- fragments of the packed parameter straight from global memory ------
  size_t wfrag[TN];
#pragma unroll
  for (int nt = 0; nt < TN; ++nt) {
    size_t nb = (size_t)(n0 + (wn * TN + nt) * 32) / 32;
    if (nb >= d.nblocks) nb = d.nblocks - 1;  // overhanging tile: loads stay in bounds, results are masked
    wfrag[nt] = d.frag_offset(nb, 0) + (size_t)lane * 16;
  }
  uint4 bw[2][TN][2][NPL];
  auto load_b = [&](int set, unsigned kt) {
#pragma unroll
    for (int nt = 0; nt < TN; ++nt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int pl = 0; pl < NPL; ++pl)
          bw[set][nt][ks][pl] = *reinterpret_cast<const uint4*>(
              p.packedW + wfrag[nt] + ((size_t)(kt * 2 + ks) * NPL + pl) * kFragBytes);
  };

  v16i acc[TM][TN][NACC];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int c = 0; c < NACC; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][b][c][r] = 0;

  // One staged step.  SET is both the LDS buffer and the register set of Wt
  // fragments, a compile-time constant so the fragments stay in registers.
  auto step = [&](auto set_c, unsigned kt) {
    constexpr int set = decltype(set_c)::value;
    store_a(set);
    __syncthreads();
    if (kt + 1 < KT) {
      load_a(kt + 1);
      load_b(set ^ 1, kt + 1);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      v4i af[TM][NPL];
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int pl = 0; pl < NPL; ++pl)
          af[mt][pl] = as_v4i(*reinterpret_cast<const uint4*>(
              &lds[set][pl][(wm * TM + mt) * 32 + lane % 32][ks * 32 + 16 * (lane / 32)]));
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
          if constexpr (BITS == 8) {
            const v4i a = af[mt][0], b = as_v4i(bw[set][nt][ks][0]);
            acc[mt][nt][0] = SWAP ? __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, acc[mt][nt][0], 0, 0, 0)
                                  : __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[mt][nt][0], 0, 0, 0);
          } else {
            const v4i ah = af[mt][0], al = af[mt][NPL - 1];
            const v4i bh = as_v4i(bw[set][nt][ks][0]), bl = as_v4i(bw[set][nt][ks][NPL - 1]);
            acc[mt][nt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bh, acc[mt][nt][0], 0, 0, 0);
            acc[mt][nt][NACC - 2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bl, acc[mt][nt][NACC - 2], 0, 0, 0);
            acc[mt][nt][NACC - 2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bh, acc[mt][nt][NACC - 2], 0, 0, 0);
            acc[mt][nt][NACC - 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bl, acc[mt][nt][NACC - 1], 0, 0, 0);
          }
        }
    }
  };

  // Two LDS buffers: step kt writes buffer kt % 2 while stragglers may still
  // read buffer (kt - 1) % 2; the barrier inside step kt + 1 orders the reuse.
  load_a(0);
  load_b(0, 0);
  for (unsigned kt = 0; kt < KT; kt += 2) {
    step(std::integral_constant<int, 0>{}, kt);
    if (kt + 1 < KT) step(std::integral_constant<int, 1>{}, kt + 1);
  }

  // ---- epilogues -----------------------------------------------------------
  // Result layout of the 32x32 MFMA: register r of lane l holds element
  // (i, j) = (8 (r / 4) + 4 (l / 32) + r % 4, l % 32); i runs over the rows of
  // the `a` operand, j over the rows of the `b` operand.
  const int lj = lane % 32, lh = lane / 32;

  if (EPI == kEpiArgmax) {
    // a = Wt: i is the candidate n, j is the sentence m.  Each lane scans its
    // own candidates in increasing n, so '>' keeps the smallest index.
    __shared__ unsigned long long best_keys[BM];
    __syncthreads();
    for (int i = tid; i < BM; i += NT) best_keys[i] = 0ull;
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      int best = 0;
      unsigned bestn = 0xFFFFFFFFu;
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned n = n0 + (wn * TN + nt) * 32 + 8 * (r / 4) + 4 * lh + r % 4;
          const int v = acc[mt][nt][0][r];
          if (n < p.N && (bestn == 0xFFFFFFFFu || v > best)) { best = v; bestn = n; }
        }
      // key orders by sum first, then by smaller index; 0 means "no candidate"
      unsigned long long key = 0ull;
      if (bestn != 0xFFFFFFFFu)
        key = ((unsigned long long)((unsigned)best ^ 0x80000000u) << 32) | (unsigned long long)(0xFFFFFFFFu - bestn);
      const unsigned long long other = __shfl_xor(key, 32, 64);
      if (other > key) key = other;
      if (lh == 0 && key != 0ull) atomicMax(&best_keys[(wm * TM + mt) * 32 + lj], key);
    }
    __syncthreads();
    for (int i = tid; i < BM; i += NT) {
      const unsigned m = m0 + i;
      const unsigned long long key = best_keys[i];
      if (m < p.M && key != 0ull) {
        // the global maximum only grows, so a stale smaller-or-equal value can be skipped safely
        if (key > __atomic_load_n(&p.keys[m], __ATOMIC_RELAXED)) atomicMax(&p.keys[m], key);
      }
    }
    return;
  }

  float u = 0.f, local_amax = 0.f;
  if (EPI == kEpiDequant) u = __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
  const int32_t* colsum = reinterpret_cast<const int32_t*>(p.packedW + d.plane_bytes());

#pragma unroll
  for (int nt = 0; nt < TN; ++nt) {
    const unsigned n = n0 + (wn * TN + nt) * 32 + lj;
    const bool n_ok = n < p.N;
    float bias = 0.f;
    unsigned corr_n = 0;
    if (EPI == kEpiDequant && p.bias != nullptr && n_ok) bias = p.bias[n];
    if (BITS == 16 && n_ok) corr_n = 128u * (unsigned)colsum[n] - 16384u * p.K;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const unsigned m = m0 + (wm * TM + mt) * 32 + 8 * (r / 4) + 4 * lh + r % 4;
        if (!n_ok || m >= p.M) continue;
        int v;
        if constexpr (BITS == 8) {
          v = acc[mt][nt][0][r];
        } else {
          const unsigned t = ((unsigned)acc[mt][nt][0][r] << 16) + ((unsigned)acc[mt][nt][NACC - 2][r] << 8) +
                             (unsigned)acc[mt][nt][NACC - 1][r] + 128u * (unsigned)p.rowsumA[m] + corr_n;
          v = (int)t;
        }
        if (EPI == kEpiRaw) {
          p.C[(size_t)m * p.N + n] = v;
        } else {
          float y = fmaf((float)v, u, bias);
          if (p.relu) y = (y > 0.0f) ? y : 0.0f;
          p.Y[(size_t)m * p.N + n] = y;
          local_amax = fmaxf(local_amax, fabsf(y));
        }
      }
  }
  if (EPI == kEpiDequant && p.out_amax != nullptr) {
    // block-wide maximum, then at most one atomic per block; the running
    // maximum only grows, so a block that cannot raise it skips the atomic.
    __shared__ float wave_amax[WM * WN];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) local_amax = fmaxf(local_amax, __shfl_xor(local_amax, off, 64));
    if (lane == 0) wave_amax[wave] = local_amax;
    __syncthreads();
    if (tid == 0) {
      float m = wave_amax[0];
#pragma unroll
      for (int w = 1; w < WM * WN; ++w) m = fmaxf(m, wave_amax[w]);
      unsigned* dst = reinterpret_cast<unsigned*>(p.out_amax);
      const unsigned bits = __float_as_uint(m);
      if (bits > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, bits);
    }
  }
}

__global__ void k_argmax_init(unsigned long long* keys, unsigned M) {
  const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < M) keys[i] = 0ull;
}

__global__ void k_argmax_finish(const unsigned long long* __restrict__ keys, unsigned M,
                                const float* __restrict__ sA, const float* __restrict__ sW,
                                int32_t* __restrict__ tok, float* __restrict__ maxlogit) {
  const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M) return;
  const float u = __fdiv_rn(1.0f, __fmul_rn(*sA, *sW));
  const unsigned long long key = keys[i];
  const int best = (int)((unsigned)(key >> 32) ^ 0x80000000u);
  const unsigned n = 0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull);
  tok[i] = (int32_t)n;
  maxlogit[i] = __fmul_rn((float)best, u);
}

template <int BITS, int BM, int BN, int WM, int WN, int EPI>
int launch_tiles(const GemmArgs& a, hipStream_t s) {
  Params p;
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.rowsumA = a.rowsumA;
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y;
  p.out_amax = a.out_amax; p.keys = a.keys;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  const dim3 grid((unsigned)(tiles_m * tiles_n)), block(WM * WN * 64);
  if (a.K % 16 == 0)
    hipLaunchKernelGGL((k_gemm<BITS, BM, BN, WM, WN, EPI, true>), grid, block, 0, s, p);
  else
    hipLaunchKernelGGL((k_gemm<BITS, BM, BN, WM, WN, EPI, false>), grid, block, 0, s, p);
  return check_hip(hipGetLastError());
}

}  // namespace

int launch_gemm(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  if (a.bits == 8) {
    switch (epi) {
      case kEpiRaw: return launch_tiles<8, 128, 128, 2, 2, kEpiRaw>(a, s);
      case kEpiDequant: return launch_tiles<8, 128, 128, 2, 2, kEpiDequant>(a, s);
      case kEpiArgmax: return launch_tiles<8, 128, 128, 2, 2, kEpiArgmax>(a, s);
    }
  } else {
    switch (epi) {
      case kEpiRaw: return launch_tiles<16, 128, 128, 2, 2, kEpiRaw>(a, s);
      case kEpiDequant: return launch_tiles<16, 128, 128, 2, 2, kEpiDequant>(a, s);
      case kEpiArgmax: return MQ_ERR_DTYPE;
    }
  }
  return MQ_ERR_UNSUPPORTED;
}

int launch_argmax_init(unsigned long long* keys, size_t M, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_init, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, s, keys, (unsigned)M);
  return check_hip(hipGetLastError());
}

int launch_argmax_finish(const unsigned long long* keys, size_t M, const float* sA, const float* sW,
                         int32_t* tok, float* maxlogit, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_finish, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, s, keys,
                     (unsigned)M, sA, sW, tok, maxlogit);
  return check_hip(hipGetLastError());
}

}  // namespace mq
