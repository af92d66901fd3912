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
// BITS == 16: every fragment is two byte planes (high byte; low byte with its top bit flipped) and a result
// tile takes four products into three accumulators (hh, hl + lh, ll); a wave's partial sum is their
// recombination 2^16 hh + 2^8 mid + ll (mod 2^32), which adds up over the waves like the 8-bit sums, and the
// plane offsets are corrected once at the end: + 128 (rowsum[m] + colsum[n]) - 16384 K.
template <int BITS, int TMW, int KS, int KW>
__global__ __launch_bounds__(KS * 64) void k_gemm_small(const Params p, const int dequant) {
  constexpr int NPL = BITS == 16 ? 2 : 1;
  constexpr int NACC = BITS == 16 ? 3 : 1;
  extern __shared__ __attribute__((aligned(16))) int part[];      // [KS][TMW * 1024]
  const int tid = threadIdx.x, lane = tid % 64;
  // The wave index, and with it the wave's run of K, must be wave-uniform to the COMPILER (scalar registers,
  // scalar branches): a matrix instruction under a lane mask is executed even when the mask is empty.
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const PackedDims dA(BITS, p.M, p.K), dW(BITS, p.N, p.K);
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

  // The epilogue's constants are asked for before the operands: loaded where they are used, they are a memory
  // round trip that nothing hides.  Every element a thread finishes has e % 64 == lane, so they share the
  // column n and the bias.
  const int lj = lane % 32, lh = lane / 32;
  const unsigned n = tile_n * 32 + lj;
  const bool n_ok = n < p.N;
  float u = 0.f, bias = 0.f, local_amax = 0.f;
  if (dequant) {
    u = __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
    if (p.bias != nullptr && n_ok) bias = p.bias[n];
  }

  v16i acc[TMW][NACC];
#pragma unroll
  for (int mt = 0; mt < TMW; ++mt)
#pragma unroll
    for (int c = 0; c < NACC; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][c][r] = 0;

  for (unsigned kb0 = kb_begin; kb0 < kb_end; kb0 += KW) {
    u4 fa[TMW][KW][NPL], fw[KW][NPL];
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      // a fragment past this wave's run is read from the run's last one (a valid address) and not used
      const unsigned kb = kb0 + j < kb_end ? kb0 + j : kb_end - 1;
#pragma unroll
      for (int pl = 0; pl < NPL; ++pl) {
        fw[j][pl] = *reinterpret_cast<const u4*>(w_src + ((size_t)kb * NPL + pl) * kFragBytes);
#pragma unroll
        for (int mt = 0; mt < TMW; ++mt)
          fa[mt][j][pl] = *reinterpret_cast<const u4*>(a_src[mt] + ((size_t)kb * NPL + pl) * kFragBytes);
      }
    }
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      if (kb0 + j < kb_end) {
#pragma unroll
        for (int mt = 0; mt < TMW; ++mt) {
          if constexpr (BITS == 8) {
            acc[mt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(fa[mt][j][0]), as_v4i(fw[j][0]), acc[mt][0], 0, 0, 0);
          } else {
            acc[mt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(fa[mt][j][0]), as_v4i(fw[j][0]), acc[mt][0], 0, 0, 0);
            acc[mt][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(fa[mt][j][0]), as_v4i(fw[j][1]), acc[mt][1], 0, 0, 0);
            acc[mt][2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(fa[mt][j][1]), as_v4i(fw[j][1]), acc[mt][2], 0, 0, 0);
            acc[mt][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(fa[mt][j][1]), as_v4i(fw[j][0]), acc[mt][1], 0, 0, 0);
          }
        }
      }
    }
  }

  // partial sums of this wave: element e = (mt * 16 + r) * 64 + lane
  int* mine = part + wave * (TMW * 1024);
#pragma unroll
  for (int mt = 0; mt < TMW; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      unsigned v = (unsigned)acc[mt][0][r];
      if constexpr (BITS == 16) v = (v << 16) + ((unsigned)acc[mt][1][r] << 8) + (unsigned)acc[mt][2][r];
      mine[(mt * 16 + r) * 64 + lane] = (int)v;
    }
  __syncthreads();

  // Every thread adds up KS partial sums for TMW * 1024 / (KS * 64) elements.
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
      if constexpr (BITS == 16) {
        const int32_t* rowsum = reinterpret_cast<const int32_t*>(p.qA + dA.plane_bytes());
        const int32_t* colsum = reinterpret_cast<const int32_t*>(p.packedW + dW.plane_bytes());
        v += 128u * ((unsigned)rowsum[m] + (unsigned)colsum[n]) - 16384u * p.K;
      }
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
  if (dequant && (p.out_amax != nullptr || p.partial != nullptr)) {
    // block-wide maximum of |y|: one value per workgroup in p.partial (no atomics; the next quantizer reduces
    // them), and/or raised into *p.out_amax with at most one atomic per block; the running maximum only
    // grows, so a block that cannot raise it skips the atomic
    __shared__ float wave_amax[KS];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) local_amax = fmaxf(local_amax, __shfl_xor(local_amax, off, 64));
    if (lane == 0) wave_amax[wave] = local_amax;
    __syncthreads();
    if (tid == 0) {
      float mx = wave_amax[0];
#pragma unroll
      for (int w = 1; w < KS; ++w) mx = fmaxf(mx, wave_amax[w]);
      if (p.partial != nullptr) p.partial[blockIdx.x] = mx;
      if (p.out_amax != nullptr) {
        unsigned* dst = reinterpret_cast<unsigned*>(p.out_amax);
        const unsigned bits = __float_as_uint(mx);
        if (bits > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, bits);
      }
    }
  }
}

template <int BITS, int TMW, int KS, int KW>
int launch_small(const GemmArgs& a, int dequant, hipStream_t s) {
  constexpr size_t smem = (size_t)KS * TMW * 1024 * sizeof(int);
  static_assert(smem <= 128 * 1024, "LDS budget");
  const PackedDims dA(BITS, a.M, a.K), dW(BITS, a.N, a.K);
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (dA.nblocks + TMW - 1) / TMW, tiles_n = dW.nblocks;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  p.partial = a.partial;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  auto kern = k_gemm_small<BITS, TMW, KS, KW>;
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


// quant_int fused into the operand fetch (Section 4.2: activations are quantized on every call): A comes as
// fp32 rows, each lane loads the 16 floats of its fragment slot, multiplies by the multiplier, rounds to
// nearest even, clamps and packs them into the 16 operand bytes.  The multiplier is either given or formed
// here from partial maxima left by the kernel that produced A (127 / max, one correctly rounded division,
// as the separate quantizer does).  Every column block of a row block repeats the conversion of that row
// block; that is cheap next to a launch as long as K is short (the fp32 rows are four times the bytes).
struct SmallF32Params {
  const float* A;            // [M x K] fp32, K a multiple of 32, rows 16-byte aligned; with A2: [M x K1], columns 0 .. K1 - 1
  const float* A2;           // optional second piece [M x (K - K1)]: columns K1 .. K - 1 of the input
  unsigned K1;
  const float* scale;        // multiplier (npartial == 0) or partial maxima
  unsigned npartial;
  const float* scale2;       // more partial maxima (the second piece's), npartial2 of them
  unsigned npartial2;
  float* scale_out;          // receives the multiplier (workgroup 0)
  const uint8_t* packedW;
  unsigned M, N, K, tiles_n;
  const float* sW;
  const float* bias;
  int relu;
  float* Y;
  float* out_amax;
  float* partial_out;        // optional: max|y| of every workgroup
};

__device__ __forceinline__ uint32_t quant_pack4(float4 v, float s) {
  auto q = [&](float x) -> uint32_t {
    const float r = rintf(__fmul_rn(x, s));
    int i;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(i) : "v"(r));      // saturates, NaN -> 0
    return (uint32_t)(min(max(i, -127), 127) & 0xFF);
  };
  return q(v.x) | (q(v.y) << 8) | (q(v.z) << 16) | (q(v.w) << 24);
}

// TNW: 32-column blocks per workgroup; KS waves split K; a round is 4 fragments (128 elements of K).
// Each wave reads its own run of K from the fp32 rows in whole 512-byte pieces (two rows per load
// instruction), converts, and turns the bytes into operand fragments through a private piece of LDS:
// fragment f of a round sits at f * kPitch, K half h of a row at h * kHalf inside it (the paddings
// spread the 4-byte writes of a row over the banks), 16 bytes per row.
template <int TNW, int KS>
__global__ __launch_bounds__(KS * 64) void k_gemm_small_f32(const SmallF32Params p) {
  constexpr int KW = 4;
  constexpr int kHalf = 512 + 16, kPitch = 2 * kHalf;
  extern __shared__ __attribute__((aligned(16))) int part[];      // [KS][TNW * 1024], then the staging pieces
  __shared__ float red[KS];
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);      // scalar, see k_gemm_small
  uint8_t* stage = reinterpret_cast<uint8_t*>(part + KS * TNW * 1024) + wave * (KW * kPitch);
  const PackedDims dW(8, p.N, p.K);
  const unsigned tile_n = blockIdx.x % p.tiles_n, tile_m = blockIdx.x / p.tiles_n;
  const unsigned ksl = p.K / 32;                                  // slices that hold real elements
  const unsigned per = (ksl + KS - 1) / KS;
  const unsigned kb_begin = wave * per;
  const unsigned kb_end = kb_begin + per < ksl ? kb_begin + per : ksl;
  const int lj = lane % 32, lh = lane / 32;

  const uint8_t* w_src[TNW];
#pragma unroll
  for (int c = 0; c < TNW; ++c) {
    unsigned nb = tile_n * TNW + c;
    if (nb >= dW.nblocks) nb = (unsigned)dW.nblocks - 1;
    w_src[c] = p.packedW + dW.frag_offset(nb, 0) + lane * 16;
  }
  // load i of a round: row 2 i + lane / 32 of the tile, floats 4 (lane % 32) .. + 3 of the round's 128
  // (rows past the end repeat the last one; their results are never stored)
  unsigned a_row[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    unsigned row = tile_m * 32 + 2 * i + lh;
    if (row >= p.M) row = p.M - 1;
    a_row[i] = row;
  }
  const unsigned ld1 = p.A2 != nullptr ? p.K1 : p.K, ld2 = p.K - p.K1;
  // where this lane's four bytes of load i go: fragment lj / 8, K half (lj / 4) % 2, row 2 i + lh, byte 4 (lj % 4)
  uint8_t* st_dst = stage + (lj / 8) * kPitch + ((lj / 4) % 2) * kHalf + lh * 16 + 4 * (lj % 4);

  float4 fa[16];
  u4 fw[TNW][KW];
  auto fetch = [&](unsigned kb0) {
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      const unsigned kb = kb0 + j < kb_end ? kb0 + j : kb_end - 1;
#pragma unroll
      for (int c = 0; c < TNW; ++c) fw[c][j] = *reinterpret_cast<const u4*>(w_src[c] + (size_t)kb * kFragBytes);
    }
    // a lane whose fragment lies past the run reads the run's last fragment instead (a valid address, unused)
    const unsigned kb = kb0 + lj / 8 < kb_end ? kb0 + lj / 8 : kb_end - 1;
    const unsigned col = kb * 32 + 4 * (lj % 8);               // this lane's first column of the input
    // two-piece input: the piece, its row stride and the column inside it (K1 is a multiple of 4, so a lane's
    // four floats never straddle the pieces)
    const bool second = p.A2 != nullptr && col >= p.K1;
    const float* base = second ? p.A2 + (col - p.K1) : p.A + col;
    const unsigned ld = second ? ld2 : ld1;
#pragma unroll
    for (int i = 0; i < 16; ++i) fa[i] = *reinterpret_cast<const float4*>(base + (size_t)a_row[i] * ld);
  };
  // the epilogue's constants first (see k_gemm_small): a thread's elements lie in column block
  // c = (i KS 64) / 1024 of the tile, all at column lj of it
  const float sW_pre = *p.sW;
  float bias_pre[TNW];
#pragma unroll
  for (int c = 0; c < TNW; ++c) {
    const unsigned n = (tile_n * TNW + c) * 32 + lj;
    bias_pre[c] = (p.bias != nullptr && n < p.N) ? p.bias[n] : 0.0f;
  }
  if (kb_begin < kb_end) fetch(kb_begin);        // the first round is on its way while the multiplier is formed

  float s;
  if (p.npartial != 0) {
    float m = 0.f;
    for (unsigned i = tid; i < p.npartial; i += KS * 64) m = fmaxf(m, p.scale[i]);
    for (unsigned i = tid; i < p.npartial2; i += KS * 64) m = fmaxf(m, p.scale2[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) red[wave] = m;
    __syncthreads();
    float amax = red[0];
#pragma unroll
    for (int w = 1; w < KS; ++w) amax = fmaxf(amax, red[w]);
    s = (amax > 0.0f) ? __fdiv_rn(127.0f, amax) : 1.0f;
  } else {
    s = *p.scale;
  }
  if (blockIdx.x == 0 && tid == 0 && p.scale_out != nullptr) *p.scale_out = s;

  v16i acc[TNW];
#pragma unroll
  for (int c = 0; c < TNW; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0;
  for (unsigned kb0 = kb_begin; kb0 < kb_end; kb0 += KW) {
    if (kb0 != kb_begin) fetch(kb0);
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<uint32_t*>(st_dst + i * 32) = quant_pack4(fa[i], s);
    // The wave reads back what it wrote itself: LDS operations of one wave complete in order, so the
    // hardware needs no wait.  The compiler does: words are written and 16-byte vectors read, types it may
    // take for non-aliasing, so both sides are fenced against compile-time motion.
    asm volatile("" ::: "memory");
    u4 a[KW];
#pragma unroll
    for (int j = 0; j < KW; ++j) a[j] = *reinterpret_cast<const u4*>(stage + j * kPitch + lh * kHalf + lj * 16);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      if (kb0 + j < kb_end) {
#pragma unroll
        for (int c = 0; c < TNW; ++c)
          acc[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(a[j]), as_v4i(fw[c][j]), acc[c], 0, 0, 0);
      }
    }
  }

  int* mine = part + wave * (TNW * 1024);
#pragma unroll
  for (int c = 0; c < TNW; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) mine[(c * 16 + r) * 64 + lane] = acc[c][r];
  __syncthreads();

  const float u = __fdiv_rn(1.0f, __fmul_rn(s, sW_pre));
  float local_amax = 0.f;
  constexpr int PER_THREAD = TNW * 1024 / (KS * 64);
  static_assert(1024 % (KS * 64) == 0, "a thread's i-th element lies in a column block known at compile time");
  static_assert(PER_THREAD >= 1 && PER_THREAD * KS * 64 == TNW * 1024, "elements must divide over the threads");
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) {
    const int e = tid + i * KS * 64;
    unsigned v = 0;
#pragma unroll
    for (int w = 0; w < KS; ++w) v += (unsigned)part[w * (TNW * 1024) + e];      // mod 2^32
    const int c = e / 1024, r = (e / 64) % 16;
    const unsigned n = (tile_n * TNW + c) * 32 + lj;
    const unsigned m = tile_m * 32 + 8 * (r / 4) + 4 * lh + r % 4;
    if (n < p.N && m < p.M) {
      float y = fmaf((float)(int)v, u, bias_pre[(i * KS * 64) / 1024]);
      if (p.relu) y = (y > 0.0f) ? y : 0.0f;
      p.Y[(size_t)m * p.N + n] = y;
      local_amax = fmaxf(local_amax, fabsf(y));
    }
  }
  if (p.out_amax != nullptr || p.partial_out != nullptr) {
    // as in k_gemm_small: one maximum per workgroup, without atomics, and/or the raised word
    __shared__ float wave_amax[KS];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) local_amax = fmaxf(local_amax, __shfl_xor(local_amax, off, 64));
    if (lane == 0) wave_amax[wave] = local_amax;
    __syncthreads();
    if (tid == 0) {
      float mx = wave_amax[0];
#pragma unroll
      for (int w = 1; w < KS; ++w) mx = fmaxf(mx, wave_amax[w]);
      if (p.partial_out != nullptr) p.partial_out[blockIdx.x] = mx;
      if (p.out_amax != nullptr) {
        unsigned* dst = reinterpret_cast<unsigned*>(p.out_amax);
        const unsigned bits = __float_as_uint(mx);
        if (bits > __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(dst, bits);
      }
    }
  }
}

template <int TNW, int KS>
int launch_small_f32(SmallF32Params p, hipStream_t s) {
  constexpr size_t smem = (size_t)KS * TNW * 1024 * sizeof(int) + (size_t)KS * 4 * 2 * (512 + 16);
  const PackedDims dW(8, p.N, p.K);
  const size_t tiles_m = (p.M + 31) / 32, tiles_n = (dW.nblocks + TNW - 1) / TNW;
  p.tiles_n = (unsigned)tiles_n;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  auto kern = k_gemm_small_f32<TNW, KS>;
  static bool attr_done = false;
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(KS * 64), smem, s, p);
  return check_hip(hipGetLastError());
}

template <int BITS, int TMW>
int launch_small_tmw(const GemmArgs& a, int dequant, size_t kfrags, hipStream_t s) {
  // one round of loads per wave where K allows: 4 waves up to K = 512, 8 up to 2048
  if (kfrags <= 16) return launch_small<BITS, TMW, 4, 4>(a, dequant, s);
  if (kfrags <= 32) return launch_small<BITS, TMW, 8, 4>(a, dequant, s);
  if constexpr (BITS == 16) {
    // two byte planes and three accumulators per tile: four fragments per round, several rounds
    return launch_small<16, TMW, 8, 4>(a, dequant, s);
  } else {
    if (kfrags <= 64) return launch_small<8, TMW, 8, 8>(a, dequant, s);
    // 16 waves leave 128 registers per lane, too few for the two-row-block form: that one stays at 8 waves
    // and takes several rounds
    if constexpr (TMW == 2) return launch_small<8, 2, 8, 8>(a, dequant, s);
    else return launch_small<8, 1, 16, 8>(a, dequant, s);
  }
}

}  // namespace

// Workgroups of launch_gemm_small / launch_gemm_small_f32 for a shape = maxima written to GemmArgs::partial.
size_t gemm_small_partials(size_t M, size_t N, size_t K) {
  const PackedDims dA(8, M, K), dW(8, N, K);
  const bool wide = ((dA.nblocks + 1) / 2) * dW.nblocks >= 256;
  return (wide ? (dA.nblocks + 1) / 2 : dA.nblocks) * dW.nblocks;
}
size_t gemm_small_f32_partials(size_t M, size_t N, size_t K) {
  const PackedDims dW(8, N, K);
  const size_t rbs = (M + 31) / 32;
  const bool wide = rbs * ((dW.nblocks + 1) / 2) >= 160;
  return rbs * (wide ? (dW.nblocks + 1) / 2 : dW.nblocks);
}

// Split-K product for few rows: packed operands of either width, raw sums or dequantize + bias (+ReLU) (+max|y|).
// Any shape is computed correctly; it is the fast choice when the result is small.
int launch_gemm_small(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  if ((a.bits != 8 && a.bits != 16) || (epi != kEpiRaw && epi != kEpiDequant)) return MQ_ERR_UNSUPPORTED;
  const PackedDims dA(a.bits, a.M, a.K), dW(a.bits, a.N, a.K);
  const int dequant = epi == kEpiDequant;
  // two row blocks per workgroup only when that still leaves a workgroup for every compute unit
  const bool wide = ((dA.nblocks + 1) / 2) * dW.nblocks >= 256;
  if (a.bits == 16)
    return wide ? launch_small_tmw<16, 2>(a, dequant, dA.kfrags, s) : launch_small_tmw<16, 1>(a, dequant, dA.kfrags, s);
  return wide ? launch_small_tmw<8, 2>(a, dequant, dA.kfrags, s) : launch_small_tmw<8, 1>(a, dequant, dA.kfrags, s);
}

// Whether quantizing inside the product pays: few rows, K short enough that re-reading the fp32 rows once
// per column tile stays below the cost of a separate quantizing launch.
bool gemm_small_f32_supported(size_t M, size_t N, size_t K) {
  return M >= 1 && M <= 512 && N >= 1 && K >= 32 && K % 32 == 0 && K <= 1024;
}

// quant_int(A) + dot'_int + dequantize + bias (+ReLU) (+max|y|) in one launch; see k_gemm_small_f32.
// scale: the multiplier (npartial == 0) or npartial partial maxima of |A|.
namespace {
int launch_small_f32_any(SmallF32Params p, const GemmArgs& a, hipStream_t s) {
  if (!gemm_small_f32_supported(a.M, a.N, a.K) || a.bits != 8) return MQ_ERR_UNSUPPORTED;
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax; p.partial_out = a.partial;
  const PackedDims dW(8, a.N, a.K);
  const size_t ksl = a.K / 32;
  // two column blocks per workgroup (half the re-reads of A) when that still leaves 160 workgroups; four
  // were slower (7.7 against 6.9 us for 300 x 2048 x 512)
  const bool wide = ((a.M + 31) / 32) * ((dW.nblocks + 1) / 2) >= 160;
  if (wide) {
    if (ksl <= 16) return launch_small_f32<2, 4>(p, s);
    return launch_small_f32<2, 8>(p, s);
  }
  if (ksl <= 16) return launch_small_f32<1, 4>(p, s);
  return launch_small_f32<1, 8>(p, s);
}
}  // namespace

int launch_gemm_small_f32(const float* A, const float* scale, unsigned npartial, float* scale_out, const GemmArgs& a,
                          hipStream_t s) {
  SmallF32Params p{};
  p.A = A; p.scale = scale; p.npartial = npartial; p.scale_out = scale_out;
  return launch_small_f32_any(p, a, s);
}

int launch_gemm_small_f32_pair(const float* A1, size_t K1, const float* part1, unsigned n1, const float* A2,
                               const float* part2, unsigned n2, float* scale_out, const GemmArgs& a, hipStream_t s) {
  if (K1 == 0 || K1 >= a.K || K1 % 4 != 0 || n1 == 0 || n2 == 0) return MQ_ERR_UNSUPPORTED;
  SmallF32Params p{};
  p.A = A1; p.A2 = A2; p.K1 = (unsigned)K1;
  p.scale = part1; p.npartial = n1; p.scale2 = part2; p.npartial2 = n2; p.scale_out = scale_out;
  return launch_small_f32_any(p, a, s);
}

}  // namespace mq
