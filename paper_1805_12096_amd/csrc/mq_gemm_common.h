// Pieces shared by the product kernels: register vector types, kernel
// parameters, the block-to-tile map and the store epilogues.
#pragma once

#include <type_traits>

#include "mq_internal.h"

namespace mq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));   // 16 bytes as a first-class register value

struct Params {
  const uint8_t* qA;        // row-major activations (row-major kernel) or packed activations (packed kernel)
  const int32_t* rowsumA;   // 16 bit: sum_k qA[m][k]
  const uint8_t* packedW;
  unsigned M, N, K;
  unsigned tiles_m, tiles_n;
  int32_t* C;
  const float* sA;
  const float* sW;
  const float* bias;
  int relu;
  float* Y;
  float* out_amax;
  unsigned long long* keys;
  // fused-FFN epilogues (packed kernel only)
  float* partial;           // abs-max partials: written (one per block) or read (npartial of them)
  unsigned npartial;
  float* s_out;             // multiplier formed from the partials, published by block 0
  uint8_t* packed_out;      // output written as packed 8-bit activations [M x N]
  unsigned* barrier;        // kBarrierWords words of the single-pass epilogue's grid-wide barrier, zero at start
  unsigned long long barrier_ticks;   // longest wait there, in ticks of the 100 MHz wall clock
  unsigned* clear_words;    // single-pass epilogue: nclear words that workgroup 0 zeroes at its start (or null)
  unsigned nclear;
  unsigned amax_slots;      // out_amax is that many words, workgroup b raises word b % amax_slots (0 or 1: one word)
};

__device__ __forceinline__ v4i as_v4i(u4 v) { return __builtin_bit_cast(v4i, v); }

// Block index -> tile.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2; giving every XCD one contiguous run of tiles (n fastest)
// makes the blocks that run together on an XCD share A row panels and the
// parameter in that XCD's L2.
__device__ __forceinline__ unsigned xcd_remap(unsigned bid, unsigned total) {
  const unsigned q = total / 8, r = total % 8, x = bid % 8, idx = bid / 8;
  return x * q + (x < r ? x : r) + idx;
}

// Tile coordinates of a block.  After the XCD remap, consecutive tile numbers
// walk down a band of GM tile rows before moving to the next tile column, so
// the ~32 blocks resident on one XCD cover a GM x (32 / GM) patch of the
// result: each A row panel and each parameter panel they stream is then shared
// by several of them in that XCD's L2 instead of being fetched once per block.
__device__ __forceinline__ void tile_coords(unsigned tiles_m, unsigned tiles_n, unsigned GM, unsigned& tile_m,
                                            unsigned& tile_n) {
  const unsigned t = xcd_remap(blockIdx.x, gridDim.x);
  const unsigned band = t / (GM * tiles_n), in_band = t % (GM * tiles_n);
  const unsigned first = band * GM;
  const unsigned rows = tiles_m - first < GM ? tiles_m - first : GM;
  tile_m = first + in_band % rows;
  tile_n = in_band / rows;
}

// max |y| over the workgroup's results -> the caller's word: block-wide maximum, then at most one atomic per
// block; the running maximum only grows, so a block that cannot raise it skips the atomic.  Every thread of the
// workgroup must call this.
template <int NWAVES>
__device__ __forceinline__ void publish_block_amax(const Params& p, float local_amax) {
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  __shared__ float wave_amax[NWAVES];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) local_amax = fmaxf(local_amax, __shfl_xor(local_amax, off, 64));
  if (lane == 0) wave_amax[wave] = local_amax;
  __syncthreads();
  if (threadIdx.x == 0) {
    float m = wave_amax[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) m = fmaxf(m, wave_amax[w]);
    // same-address atomics are served one after the other (about 12 ns each): a thousand workgroups on one word
    // cost 12 us, on 32 words next to nothing
    unsigned* dst = reinterpret_cast<unsigned*>(p.out_amax) + (p.amax_slots > 1 ? blockIdx.x % p.amax_slots : 0);
    const unsigned bits = __float_as_uint(m);
    if (bits > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, bits);
  }
}

// Raw-sum and dequantizing epilogues for a wave that holds TM x TN result tiles
// of the 32x32 MFMA with (a = activations, b = parameter): register r of lane l
// is element (i, j) = (8 (r / 4) + 4 (l / 32) + r % 4, l % 32) of its tile, i
// along M, j along N.  wave_m0 / wave_n0 are the wave's first row / column.
// 16-bit sums are recombined here from the three partial accumulators:
//   acc = 2^16 hh + 2^8 mid + ll + 128 (rowsum[m] + colsum[n]) - 16384 K  (mod 2^32).
// bias_pre (optional): this lane's TN biases (0 where there is none), fetched by the caller before its main
// loop so that the epilogue does not start with a memory round trip.
// row_base / col_base: index of rowsum[0] / colsum[0] (a caller that has copied its tile's sums to LDS before its
// main loop, for the same reason, passes the tile's origin; sums of rows and columns past the end must then be there
// too, as zeros).
// u_pre (optional): the dequantization factor 1 / (sA sW), for a caller that runs the epilogue once per tile of several
// (the two loads here wait for every load the wave has in flight).
// amax_acc (optional): this thread's running max |y|; with it the epilogue only updates it, and the caller publishes
// the workgroup's maximum once, after its last tile (publish_block_amax).
template <int BITS, int TM, int TN, int NACC, int EPI, int NWAVES>
__device__ __forceinline__ void store_epilogue(v16i (&acc)[TM][TN][NACC], const Params& p, unsigned wave_m0,
                                               unsigned wave_n0, const int32_t* rowsum, const int32_t* colsum,
                                               const float* bias_pre = nullptr, unsigned row_base = 0,
                                               unsigned col_base = 0, const float* u_pre = nullptr,
                                               float* amax_acc = nullptr) {
  const int lane = threadIdx.x % 64;
  const int lj = lane % 32, lh = lane / 32;
  float u = 0.f, local_amax = 0.f;
  if (EPI == kEpiDequant) u = u_pre != nullptr ? *u_pre : __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
  // Addresses split into a wave-uniform part (tile origin, register's row) and a per-lane constant
  // (4 (l / 32) rows down, l % 32 columns right), so that a store needs no per-element arithmetic.
  const size_t lane_off = (size_t)(4 * lh) * p.N + lj;
  // Whole wave tile inside the matrix (the common case): no per-element bounds checks.
  const bool interior = wave_m0 + TM * 32 <= p.M && wave_n0 + TN * 32 <= p.N;
  auto element = [&](int mt, int nt, int r, float bias, unsigned corr_n, unsigned m) -> void {
    int v;
    if constexpr (BITS == 8) {
      v = acc[mt][nt][0][r];
    } else {
      const unsigned t = ((unsigned)acc[mt][nt][0][r] << 16) + ((unsigned)acc[mt][nt][NACC - 2][r] << 8) +
                         (unsigned)acc[mt][nt][NACC - 1][r] + 128u * (unsigned)rowsum[m - row_base] + corr_n;
      v = (int)t;
    }
    const size_t uni = (size_t)(wave_m0 + mt * 32 + 8 * (r / 4) + r % 4) * p.N + wave_n0 + nt * 32;
    if (EPI == kEpiRaw) {
      p.C[uni + lane_off] = v;
    } else {
      float y = fmaf((float)v, u, bias);
      if (p.relu) y = (y > 0.0f) ? y : 0.0f;
      p.Y[uni + lane_off] = y;
      local_amax = fmaxf(local_amax, fabsf(y));
    }
  };
  if (interior && p.N <= (1u << 26)) {
    // The epilogue is bound by vector instructions (a 256 x 128 tile is 64 results per lane with the matrix cores
    // idle), so this path keeps them to a minimum per result: two shift-adds and one three-operand add for the
    // recombination, convert, multiply-add, (maximum for the ReLU,) store.  The tile origin is wave-uniform, so
    // a row's address is scalar arithmetic and the store takes it with one 32-bit lane offset (four rows down and
    // 31 columns right fit 32 bits for N up to 2^26); the ReLU is a maximum with zero under a uniform branch (NaN
    // and -0 come out as 0 either way).
    const unsigned um0 = __builtin_amdgcn_readfirstlane(wave_m0), un0 = __builtin_amdgcn_readfirstlane(wave_n0);
    const uint32_t lane_bytes = ((4u * (unsigned)lh) * p.N + (unsigned)lj) * 4u;
    char* const out = reinterpret_cast<char*>(EPI == kEpiRaw ? static_cast<void*>(p.C) : static_cast<void*>(p.Y)) +
                      ((size_t)um0 * p.N + un0) * 4;
    const size_t row_bytes = (size_t)p.N * 4;
    float bias[TN];
    unsigned corr[TN];
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
      const unsigned n = un0 + nt * 32 + lj;
      bias[nt] = 0.f;
      corr[nt] = 0;
      if (EPI == kEpiDequant) {
        if (bias_pre != nullptr) bias[nt] = bias_pre[nt];
        else if (p.bias != nullptr) bias[nt] = p.bias[n];
      }
      if (BITS == 16) corr[nt] = 128u * (unsigned)colsum[n - col_base] - 16384u * p.K;
    }
    auto rows = [&](auto relu_on) {
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = mt * 32 + 8 * (r / 4) + r % 4;
          char* const rowp = out + row * row_bytes;
          unsigned rs128 = 0;
          if (BITS == 16) rs128 = 128u * (unsigned)rowsum[um0 + row + 4 * lh - row_base];
#pragma unroll
          for (int nt = 0; nt < TN; ++nt) {
            int v;
            if constexpr (BITS == 8) {
              v = acc[mt][nt][0][r];
            } else {
              unsigned t;
              asm("v_lshl_add_u32 %0, %1, 8, %2" : "=v"(t) : "v"(acc[mt][nt][NACC - 2][r]), "v"(acc[mt][nt][NACC - 1][r]));
              asm("v_lshl_add_u32 %0, %1, 16, %2" : "=v"(t) : "v"(acc[mt][nt][0][r]), "v"(t));
              v = (int)(t + rs128 + corr[nt]);
            }
            char* const dst = rowp + nt * 128 + lane_bytes;
            if (EPI == kEpiRaw) {
              *reinterpret_cast<int32_t*>(dst) = v;
            } else {
              float y = fmaf((float)v, u, bias[nt]);
              if (decltype(relu_on)::value) y = __builtin_fmaxf(y, 0.0f);
              *reinterpret_cast<float*>(dst) = y;
              local_amax = fmaxf(local_amax, fabsf(y));
            }
          }
        }
    };
    if (EPI == kEpiDequant && p.relu) rows(std::true_type{});
    else rows(std::false_type{});
  } else {
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
      const unsigned n = wave_n0 + nt * 32 + lj;
      const bool n_ok = n < p.N;
      float bias = 0.f;
      unsigned corr_n = 0;
      if (EPI == kEpiDequant) {
        if (bias_pre != nullptr) bias = bias_pre[nt];
        else if (p.bias != nullptr && n_ok) bias = p.bias[n];
      }
      if (BITS == 16 && n_ok) corr_n = 128u * (unsigned)colsum[n - col_base] - 16384u * p.K;
#pragma unroll
      for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned m = wave_m0 + mt * 32 + 8 * (r / 4) + 4 * lh + r % 4;
          if (n_ok && m < p.M) element(mt, nt, r, bias, corr_n, m);
        }
    }
  }
  if (EPI == kEpiDequant && p.out_amax != nullptr) {
    if (amax_acc != nullptr) *amax_acc = fmaxf(*amax_acc, local_amax);
    else publish_block_amax<NWAVES>(p, local_amax);
  }
}

}  // namespace mq
