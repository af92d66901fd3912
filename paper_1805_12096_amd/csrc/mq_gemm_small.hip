// dot'_int for decode-sized activations (arxiv 1805.12096, Section 4.3: the
// product of two quantized tensors, both contiguous along K; Section 3.2: a
// decoder step multiplies a few hundred rows by every parameter matrix).
//
// With a few hundred rows the whole product is some ten thousand matrix
// instructions, a few per SIMD: time is latency, not throughput.  The tiled
// kernel walks K in a software pipeline, one stage after the other, which is
// the wrong shape for that.  Here the contraction is cut ACROSS the waves of a
// workgroup instead: a workgroup owns a 32- or 64-row by 32-column piece of the
// result, each of its waves takes a contiguous run of K, asks for all of its
// operand fragments at once (one round trip to L2), multiplies, and the partial
// sums meet in LDS.  Integer addition is exact, so the split changes no bit.
// Both operands are in fragment order; a fragment is one coalesced 1 KB read
// straight into the registers the matrix instruction takes.
#include "mq_gemm_common.h"

namespace mq {

namespace {

// TMW: 32-row blocks per workgroup; KS: waves (= parts of K); KW: fragments per operand row block and round.
template <int TMW, int KS, int KW>
__global__ __launch_bounds__(KS * 64) void k_gemm_small(const Params p, const int dequant) {
  extern __shared__ __attribute__((aligned(16))) int part[];      // [KS][TMW * 1024]
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const PackedDims dA(8, p.M, p.K), dW(8, p.N, p.K);
  const unsigned tile_n = blockIdx.x % p.tiles_n, tile_m = blockIdx.x / p.tiles_n;
  const unsigned kfrags = (unsigned)dA.kfrags;
  const unsigned per = (kfrags + KS - 1) / KS;
  const unsigned kb_begin = wave * per;
  const unsigned kb_end = kb_begin + per < kfrags ? kb_begin + per : kfrags;

  // row blocks of the tile; one past the end is clamped (its rows are masked when stored)
  const uint8_t* a_src[TMW];
#pragma unroll
  for (int mt = 0; mt < TMW; ++mt) {
    unsigned rb = tile_m * TMW + mt;
    if (rb >= dA.nblocks) rb = (unsigned)dA.nblocks - 1;
    a_src[mt] = p.qA + dA.frag_offset(rb, 0) + lane * 16;
  }
  const uint8_t* w_src = p.packedW + dW.frag_offset(tile_n, 0) + lane * 16;

  v16i acc[TMW];
#pragma unroll
  for (int mt = 0; mt < TMW; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0;

  for (unsigned kb0 = kb_begin; kb0 < kb_end; kb0 += KW) {
    u4 fa[TMW][KW], fw[KW];
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      // a fragment past this wave's run is read from the run's last one (a valid address) and not used
      const unsigned kb = kb0 + j < kb_end ? kb0 + j : kb_end - 1;
      fw[j] = *reinterpret_cast<const u4*>(w_src + (size_t)kb * kFragBytes);
#pragma unroll
      for (int mt = 0; mt < TMW; ++mt) fa[mt][j] = *reinterpret_cast<const u4*>(a_src[mt] + (size_t)kb * kFragBytes);
    }
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      if (kb0 + j < kb_end) {
#pragma unroll
        for (int mt = 0; mt < TMW; ++mt)
          acc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(fa[mt][j]), as_v4i(fw[j]), acc[mt], 0, 0, 0);
      }
    }
  }

  // partial sums of this wave: element e = (mt * 16 + r) * 64 + lane
  int* mine = part + wave * (TMW * 1024);
#pragma unroll
  for (int mt = 0; mt < TMW; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) mine[(mt * 16 + r) * 64 + lane] = acc[mt][r];
  __syncthreads();

  // Every thread adds up KS partial sums for TMW * 1024 / (KS * 64) elements.  Its elements all have
  // e % 64 == lane, so they share the column n and the bias.
  const int lj = lane % 32, lh = lane / 32;
  const unsigned n = tile_n * 32 + lj;
  const bool n_ok = n < p.N;
  float u = 0.f, bias = 0.f, local_amax = 0.f;
  if (dequant) {
    u = __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
    if (p.bias != nullptr && n_ok) bias = p.bias[n];
  }
  constexpr int PER_THREAD = TMW * 1024 / (KS * 64);
  static_assert(PER_THREAD >= 1 && PER_THREAD * KS * 64 == TMW * 1024, "elements must divide over the threads");
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) {
    const int e = tid + i * KS * 64;
    unsigned v = 0;
#pragma unroll
    for (int w = 0; w < KS; ++w) v += (unsigned)part[w * (TMW * 1024) + e];      // mod 2^32
    const int mt = e / 1024, r = (e / 64) % 16;
    const unsigned m = (tile_m * TMW + mt) * 32 + 8 * (r / 4) + 4 * lh + r % 4;
    if (n_ok && m < p.M) {
      if (dequant) {
        float y = fmaf((float)(int)v, u, bias);
        if (p.relu) y = (y > 0.0f) ? y : 0.0f;
        p.Y[(size_t)m * p.N + n] = y;
        local_amax = fmaxf(local_amax, fabsf(y));
      } else {
        p.C[(size_t)m * p.N + n] = (int)v;
      }
    }
  }
  if (dequant && p.out_amax != nullptr) {
    // block-wide maximum, then at most one atomic per block; the running maximum only grows, so a block
    // that cannot raise it skips the atomic
    __shared__ float wave_amax[KS];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) local_amax = fmaxf(local_amax, __shfl_xor(local_amax, off, 64));
    if (lane == 0) wave_amax[wave] = local_amax;
    __syncthreads();
    if (tid == 0) {
      float mx = wave_amax[0];
#pragma unroll
      for (int w = 1; w < KS; ++w) mx = fmaxf(mx, wave_amax[w]);
      unsigned* dst = reinterpret_cast<unsigned*>(p.out_amax);
      const unsigned bits = __float_as_uint(mx);
      if (bits > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, bits);
    }
  }
}

template <int TMW, int KS, int KW>
int launch_small(const GemmArgs& a, int dequant, hipStream_t s) {
  constexpr size_t smem = (size_t)KS * TMW * 1024 * sizeof(int);
  static_assert(smem <= 128 * 1024, "LDS budget");
  const PackedDims dA(8, a.M, a.K), dW(8, a.N, a.K);
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (dA.nblocks + TMW - 1) / TMW, tiles_n = dW.nblocks;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  auto kern = k_gemm_small<TMW, KS, KW>;
  static bool attr_done = false;
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(KS * 64), smem, s, p, dequant);
  return check_hip(hipGetLastError());
}

template <int TMW>
int launch_small_tmw(const GemmArgs& a, int dequant, size_t kfrags, hipStream_t s) {
  // one round of loads per wave where K allows: 4 waves up to K = 512, 8 up to 2048
  if (kfrags <= 16) return launch_small<TMW, 4, 4>(a, dequant, s);
  if (kfrags <= 32) return launch_small<TMW, 8, 4>(a, dequant, s);
  if (kfrags <= 64) return launch_small<TMW, 8, 8>(a, dequant, s);
  // 16 waves leave 128 registers per lane, too few for the two-row-block form: that one stays at 8 waves
  // and takes several rounds
  if constexpr (TMW == 2) return launch_small<2, 8, 8>(a, dequant, s);
  else return launch_small<1, 16, 8>(a, dequant, s);
}

}  // namespace

// Split-K product for few rows: 8-bit packed operands, raw sums or dequantize + bias (+ReLU) (+max|y|).
// Any shape is computed correctly; it is the fast choice when the result is small.
int launch_gemm_small(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  if (a.bits != 8 || (epi != kEpiRaw && epi != kEpiDequant)) return MQ_ERR_UNSUPPORTED;
  const PackedDims dA(8, a.M, a.K), dW(8, a.N, a.K);
  const int dequant = epi == kEpiDequant;
  // two row blocks per workgroup only when that still leaves a workgroup for every compute unit
  const bool wide = ((dA.nblocks + 1) / 2) * dW.nblocks >= 256;
  return wide ? launch_small_tmw<2>(a, dequant, dA.kfrags, s) : launch_small_tmw<1>(a, dequant, dA.kfrags, s);
}

}  // namespace mq
