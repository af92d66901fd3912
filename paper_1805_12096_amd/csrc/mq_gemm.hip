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

#include "mq_gemm_common.h"

namespace mq {

namespace {

constexpr int kBK = 64;               // contracted elements staged per step
constexpr int kLdsStride = kBK + 16;  // bytes per staged row; odd multiple of 16 => conflict-free b128 reads

// Four consecutive int16 (two dwords) -> their 4 high bytes and their 4 low bytes
// (low bytes with the top bit flipped, i.e. minus 128 as signed bytes).
__device__ __forceinline__ uint32_t hi_bytes(uint32_t d0, uint32_t d1) {
  return ((d0 >> 8) & 0xFFu) | ((d0 >> 24) << 8) | (((d1 >> 8) & 0xFFu) << 16) | ((d1 >> 24) << 24);
}
__device__ __forceinline__ uint32_t lo_bytes(uint32_t d0, uint32_t d1) {
  return ((d0 & 0xFFu) | (((d0 >> 16) & 0xFFu) << 8) | ((d1 & 0xFFu) << 16) | (((d1 >> 16) & 0xFFu) << 24)) ^
         0x80808080u;
}

template <int BITS, int BM, int BN, int WM, int WN, int EPI, bool KVEC>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm(const Params p) {
  constexpr int NT = WM * WN * 64;
  constexpr int NPL = BITS == 16 ? 2 : 1;
  constexpr int TM = BM / WM / 32;
  constexpr int TN = BN / WN / 32;
  constexpr int NACC = BITS == 16 ? 3 : 1;
  constexpr int CHUNKS_A = BM * (kBK / 16);
  constexpr int CPT_A = (CHUNKS_A + NT - 1) / NT;
  constexpr int NB = BN / 32;                          // parameter row blocks per tile
  constexpr int CHUNKS_B = NB * 2 * NPL * 64;          // 16-byte chunks of one staged step
  constexpr int CPT_B = (CHUNKS_B + NT - 1) / NT;
  constexpr int A_STAGE = NPL * BM * kLdsStride;       // bytes
  constexpr int B_STAGE = CHUNKS_B * 16;
  constexpr bool SWAP = EPI == kEpiArgmax;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");
  static_assert(CHUNKS_A % NT == 0 && CHUNKS_B % NT == 0, "staging must divide evenly over the threads");

  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* const ldsA = smem;                  // [2][NPL][BM][kLdsStride]
  uint8_t* const ldsB = smem + 2 * A_STAGE;    // [2][NB][2][NPL][1024], fragment order as in global memory

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = tid / 64;
  const int wm = wave / WN, wn = wave % WN;
  unsigned tile_m, tile_n;
  tile_coords(p.tiles_m, p.tiles_n, BM >= 1024 ? 1u : 1024u / BM, tile_m, tile_n);
  const unsigned m0 = tile_m * BM, n0 = tile_n * BN;
  const PackedDims d(BITS, p.N, p.K);
  const unsigned KT = (unsigned)(d.Kp / kBK);

  // ---- staging: global -> registers -> LDS ---------------------------------
  u4 stage_a[CPT_A][NPL];
  u4 stage_b[CPT_B];
  auto load_a = [&](unsigned kt) {
#pragma unroll
    for (int i = 0; i < CPT_A; ++i) {
      const int c = tid + i * NT;
      const unsigned row = m0 + c / (kBK / 16);
      const unsigned k = kt * kBK + (c % (kBK / 16)) * 16;
      const u4 zero = {0u, 0u, 0u, 0u};
      u4 v0 = zero, v1 = zero;
      const bool valid = c < CHUNKS_A && row < p.M && k < p.K;
      if constexpr (KVEC) {
        // Always load from an in-bounds address (row and k clamped).  What lies
        // outside needs no zeroing: rows >= M are never stored, and elements
        // k >= K meet the zero padding of the packed parameter.
        const unsigned rc = row < p.M ? row : p.M - 1;
        const unsigned kc = k < p.K ? k : p.K - 16;
        const u4* src = reinterpret_cast<const u4*>(p.qA + ((size_t)rc * p.K + kc) * (BITS / 8));
        v0 = src[0];
        if (BITS == 16) v1 = src[1];
      } else if (valid) {
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
        v0 = u4{w[0], w[1], w[2], w[3]};
        v1 = u4{w[4], w[5], w[6], w[7]};
      }
      if constexpr (BITS == 8) {
        stage_a[i][0] = v0;
      } else {
        const u4 hi = {hi_bytes(v0.x, v0.y), hi_bytes(v0.z, v0.w), hi_bytes(v1.x, v1.y), hi_bytes(v1.z, v1.w)};
        const u4 lo = {lo_bytes(v0.x, v0.y), lo_bytes(v0.z, v0.w), lo_bytes(v1.x, v1.y), lo_bytes(v1.z, v1.w)};
        stage_a[i][0] = hi;
        stage_a[i][NPL - 1] = lo;
      }
    }
  };
  // One staged step of the parameter is, per row block, 2 * NPL consecutive
  // fragments in global memory; LDS keeps the same order, so the copy is linear.
  size_t b_src[CPT_B];
#pragma unroll
  for (int i = 0; i < CPT_B; ++i) {
    const int c = tid + i * NT;
    size_t nb = (size_t)n0 / 32 + c / (2 * NPL * 64);
    if (nb >= d.nblocks) nb = d.nblocks - 1;  // overhanging tile: loads stay in bounds, results are masked
    b_src[i] = d.frag_offset(nb, 0) + (size_t)(c % (2 * NPL * 64)) * 16;
  }
  auto load_b = [&](unsigned kt) {
#pragma unroll
    for (int i = 0; i < CPT_B; ++i)
      stage_b[i] = *reinterpret_cast<const u4*>(p.packedW + b_src[i] + (size_t)kt * (2 * NPL * kFragBytes));
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CPT_A; ++i) {
      const int c = tid + i * NT;
#pragma unroll
      for (int pl = 0; pl < NPL; ++pl)
        *reinterpret_cast<u4*>(ldsA + buf * A_STAGE + (pl * BM + c / (kBK / 16)) * kLdsStride +
                                  (c % (kBK / 16)) * 16) = stage_a[i][pl];
    }
#pragma unroll
    for (int i = 0; i < CPT_B; ++i) {
      const int c = tid + i * NT;
      *reinterpret_cast<u4*>(ldsB + buf * B_STAGE + c * 16) = stage_b[i];
    }
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

  auto compute = [&](int buf) {
    const uint8_t* a_base = ldsA + buf * A_STAGE + ((wm * TM) * 32 + lane % 32) * kLdsStride + 16 * (lane / 32);
    const uint8_t* b_base = ldsB + buf * B_STAGE + (wn * TN) * (2 * NPL * kFragBytes) + lane * 16;
    // All fragment reads of the step are issued before the first MFMA so that
    // LDS latency is paid once per step, not once per fragment.
    v4i af[2][TM][NPL], bf[2][TN][NPL];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int pl = 0; pl < NPL; ++pl)
          af[ks][mt][pl] = as_v4i(*reinterpret_cast<const u4*>(a_base + (pl * BM + mt * 32) * kLdsStride + ks * 32));
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
#pragma unroll
        for (int pl = 0; pl < NPL; ++pl)
          bf[ks][nt][pl] = as_v4i(*reinterpret_cast<const u4*>(b_base + ((nt * 2 + ks) * NPL + pl) * kFragBytes));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
          if constexpr (BITS == 8) {
            const v4i a = af[ks][mt][0], b = bf[ks][nt][0];
            acc[mt][nt][0] = SWAP ? __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, acc[mt][nt][0], 0, 0, 0)
                                  : __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[mt][nt][0], 0, 0, 0);
          } else {
            const v4i ah = af[ks][mt][0], al = af[ks][mt][NPL - 1];
            const v4i bh = bf[ks][nt][0], bl = bf[ks][nt][NPL - 1];
            acc[mt][nt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bh, acc[mt][nt][0], 0, 0, 0);
            acc[mt][nt][NACC - 2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bl, acc[mt][nt][NACC - 2], 0, 0, 0);
            acc[mt][nt][NACC - 2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bh, acc[mt][nt][NACC - 2], 0, 0, 0);
            acc[mt][nt][NACC - 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bl, acc[mt][nt][NACC - 1], 0, 0, 0);
          }
        }
    }
  };

  // Two LDS stages.  While step kt is multiplied out of stage kt % 2, the
  // global loads of step kt + 1 are in flight into registers; they are written
  // to the other stage after the multiply, and one barrier per step orders both
  // the reuse of that stage and the visibility of the new data.
  load_a(0);
  load_b(0);
  store_stage(0);
  __syncthreads();
  for (unsigned kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) {
      load_a(kt + 1);
      load_b(kt + 1);
    }
    compute(cur);
    if (more) store_stage(cur ^ 1);
    __syncthreads();
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

  const int32_t* colsum = reinterpret_cast<const int32_t*>(p.packedW + d.plane_bytes());
  store_epilogue<BITS, TM, TN, NACC, EPI, WM * WN>(acc, p, m0 + wm * TM * 32, n0 + wn * TN * 32, p.rowsumA, colsum);
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

template <int BITS, int BM, int BN, int WM, int WN>
constexpr size_t smem_bytes() {
  constexpr int NPL = BITS == 16 ? 2 : 1;
  return 2 * (size_t)(NPL * BM * kLdsStride) + 2 * (size_t)((BN / 32) * 2 * NPL * 64 * 16);
}

template <int BITS, int BM, int BN, int WM, int WN, int EPI, bool KVEC>
int launch_one(const Params& p, dim3 grid, hipStream_t s) {
  constexpr size_t smem = smem_bytes<BITS, BM, BN, WM, WN>();
  auto kern = k_gemm<BITS, BM, BN, WM, WN, EPI, KVEC>;
  static bool attr_done = false;   // raising the dynamic LDS limit is needed once per kernel
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(WM * WN * 64), smem, s, p);
  return check_hip(hipGetLastError());
}

template <int BITS, int BM, int BN, int WM, int WN, int EPI>
int launch_tiles(const GemmArgs& a, hipStream_t s) {
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.rowsumA = a.rowsumA;
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y;
  p.out_amax = a.out_amax; p.keys = a.keys; p.partial = nullptr; p.npartial = 0; p.s_out = nullptr; p.packed_out = nullptr;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  const dim3 grid((unsigned)(tiles_m * tiles_n));
  if (a.K % 16 == 0) return launch_one<BITS, BM, BN, WM, WN, EPI, true>(p, grid, s);
  return launch_one<BITS, BM, BN, WM, WN, EPI, false>(p, grid, s);
}

template <int BITS, int EPI>
int launch_variant(const GemmArgs& a, int variant, hipStream_t s) {
  if constexpr (BITS == 8) {
    switch (variant) {
      case 1: return launch_tiles<8, 128, 128, 2, 2, EPI>(a, s);
      case 2: return launch_tiles<8, 256, 128, 2, 2, EPI>(a, s);
      case 3: return launch_tiles<8, 256, 256, 2, 2, EPI>(a, s);
      case 4: return launch_tiles<8, 128, 256, 2, 2, EPI>(a, s);
      default: return MQ_ERR_UNSUPPORTED;
    }
  } else {
    switch (variant) {
      case 1: return launch_tiles<16, 128, 128, 2, 2, EPI>(a, s);
      case 2: return launch_tiles<16, 64, 64, 2, 2, EPI>(a, s);
      default: return MQ_ERR_UNSUPPORTED;
    }
  }
}

int g_forced_variant = 0;

// Tile choice by shape: the large tile when it still yields at least one tile
// per compute unit, the small one otherwise.
int pick_variant(const GemmArgs& a) {
  if (g_forced_variant > 0) return g_forced_variant;
  if (a.bits == 16) return 1;
  const size_t t256 = ((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (t256 >= 256) return 3;
  const size_t t2 = ((a.M + 255) / 256) * ((a.N + 127) / 128);
  if (t2 >= 256) return 2;
  return 1;
}

}  // namespace

void set_forced_variant(int v) { g_forced_variant = v; }
int forced_variant() { return g_forced_variant; }

int launch_gemm(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  const int v = pick_variant(a);
  if (a.bits == 8) {
    switch (epi) {
      case kEpiRaw: return launch_variant<8, kEpiRaw>(a, v, s);
      case kEpiDequant: return launch_variant<8, kEpiDequant>(a, v, s);
      case kEpiArgmax: return launch_tiles<8, 128, 128, 2, 2, kEpiArgmax>(a, s);
    }
  } else {
    switch (epi) {
      case kEpiRaw: return launch_variant<16, kEpiRaw>(a, v, s);
      case kEpiDequant: return launch_variant<16, kEpiDequant>(a, v, s);
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
