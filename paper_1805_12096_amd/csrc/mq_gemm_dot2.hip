// dot'_int for 16-bit operands on the vector ALU instead of the matrix cores (arxiv 1805.12096, Section 4.2: the
// paper's own 16-bit kernel multiplies pairs of 16-bit values and adds them into 32-bit sums with one vector
// instruction; v_dot2c_i32_i16 is this chip's instruction of that kind).  It is the alternative implementation the
// auto-tuner (Section 4.4) ranks against the decomposition onto four 8-bit matrix products: variant 7 of the packed
// 16-bit products.  Same operands (both packed), same results (the exact sums modulo 2^32), any shape.
//
// One wave per workgroup owns a 32 x 32 tile of the result.  Per 32 contracted elements it reads the two byte planes of
// one fragment of each operand (four coalesced 1 KB reads), interleaves the planes back into 16-bit values with byte
// permutes (value = high byte, low byte with its top bit flipped back), parks them in LDS as rows of 16 pairs, and
// every lane then multiplies a 4 x 4 block of the tile out of LDS: 16 pairs x 16 dot instructions.  No plane
// corrections are needed, the sums are those of the 16-bit values themselves.
#include "mq_gemm_common.h"

namespace mq {

namespace {

typedef short v2s __attribute__((ext_vector_type(2)));

constexpr int kRowPairs = 16;            // 32 contracted 16-bit values = 16 dwords per row and K step
constexpr int kRowStride = kRowPairs + 1;   // padded so that the lanes' row starts fall into different banks

// 16 bytes of the high plane and 16 of the low plane (one lane's share of a fragment: 16 consecutive K of one row)
// -> 8 dwords of two 16-bit values each
__device__ __forceinline__ void planes_to_pairs(const u4& hi, const u4& lo, uint32_t (&out)[8]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t l = lo[d] ^ 0x80808080u;       // the low plane stores (q & 255) - 128
    out[2 * d] = __builtin_amdgcn_perm(hi[d], l, 0x05010400u);       // bytes l0 h0 l1 h1
    out[2 * d + 1] = __builtin_amdgcn_perm(hi[d], l, 0x07030602u);   // bytes l2 h2 l3 h3
  }
}

template <int EPI>
__global__ __launch_bounds__(64) void k_gemm_dot2(const Params p) {
  __shared__ uint32_t sA[32 * kRowStride];
  __shared__ uint32_t sB[32 * kRowStride];
  const int lane = threadIdx.x;
  const PackedDims dA(16, p.M, p.K), dW(16, p.N, p.K);
  const unsigned nb = blockIdx.x % p.tiles_n, rb = blockIdx.x / p.tiles_n;
  const int ti = lane / 8, tj = lane % 8;                 // this lane's 4 x 4 block: rows 4 ti .., columns 4 tj ..
  int acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0;
  const uint8_t* srcA = p.qA + dA.frag_offset(rb, 0) + lane * 16;
  const uint8_t* srcB = p.packedW + dW.frag_offset(nb, 0) + lane * 16;
  const unsigned row = lane % 32, half = lane / 32;
  const unsigned KF = (unsigned)dA.kfrags;
  // the next fragments are fetched while the current ones are multiplied
  u4 ah = *reinterpret_cast<const u4*>(srcA), al = *reinterpret_cast<const u4*>(srcA + kFragBytes);
  u4 bh = *reinterpret_cast<const u4*>(srcB), bl = *reinterpret_cast<const u4*>(srcB + kFragBytes);
  for (unsigned kb = 0; kb < KF; ++kb) {
    uint32_t pa[8], pb[8];
    planes_to_pairs(ah, al, pa);
    planes_to_pairs(bh, bl, pb);
    __syncthreads();                                       // the reads of the step before are done
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      sA[row * kRowStride + 8 * half + d] = pa[d];
      sB[row * kRowStride + 8 * half + d] = pb[d];
    }
    if (kb + 1 < KF) {
      const size_t step = (size_t)(kb + 1) * 2 * kFragBytes;
      ah = *reinterpret_cast<const u4*>(srcA + step);
      al = *reinterpret_cast<const u4*>(srcA + step + kFragBytes);
      bh = *reinterpret_cast<const u4*>(srcB + step);
      bl = *reinterpret_cast<const u4*>(srcB + step + kFragBytes);
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kRowPairs; ++c) {
      uint32_t a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = sA[(4 * ti + i) * kRowStride + c];
        b[i] = sB[(4 * tj + i) * kRowStride + c];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_sdot2(__builtin_bit_cast(v2s, a[i]), __builtin_bit_cast(v2s, b[j]), acc[i][j], false);
    }
  }
  // epilogue: raw sums, or y = fma((float) sum, 1 / (sA sW), bias[n]) (+ReLU) (+ max|y| for the caller)
  float u = 0.f, local_amax = 0.f;
  if (EPI == kEpiDequant) u = __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned m = rb * 32 + 4 * ti + i;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const unsigned n = nb * 32 + 4 * tj + j;
      if (m < p.M && n < p.N) {
        if (EPI == kEpiRaw) {
          p.C[(size_t)m * p.N + n] = acc[i][j];
        } else {
          float y = fmaf((float)acc[i][j], u, p.bias != nullptr ? p.bias[n] : 0.0f);
          if (p.relu) y = (y > 0.0f) ? y : 0.0f;
          p.Y[(size_t)m * p.N + n] = y;
          local_amax = fmaxf(local_amax, fabsf(y));
        }
      }
    }
  }
  if (EPI == kEpiDequant && p.out_amax != nullptr) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) local_amax = fmaxf(local_amax, __shfl_xor(local_amax, off, 64));
    if (lane == 0) {
      unsigned* dst = reinterpret_cast<unsigned*>(p.out_amax);
      const unsigned bits = __float_as_uint(local_amax);
      if (bits > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, bits);
    }
  }
}

}  // namespace

int launch_gemm_dot2(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  if (a.bits != 16 || (epi != kEpiRaw && epi != kEpiDequant)) return MQ_ERR_UNSUPPORTED;
  const PackedDims dA(16, a.M, a.K), dW(16, a.N, a.K);
  if (dA.nblocks * dW.nblocks > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  p.tiles_m = (unsigned)dA.nblocks;
  p.tiles_n = (unsigned)dW.nblocks;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  const dim3 grid((unsigned)(dA.nblocks * dW.nblocks));
  if (epi == kEpiRaw) hipLaunchKernelGGL(k_gemm_dot2<kEpiRaw>, grid, dim3(64), 0, s, p);
  else hipLaunchKernelGGL(k_gemm_dot2<kEpiDequant>, grid, dim3(64), 0, s, p);
  return check_hip(hipGetLastError());
}

}  // namespace mq
