// dot'_int on packed 8-bit operands with the loading taken off the multiplying waves
// (arxiv 1805.12096, Section 4.3: the product of two quantized tensors, both contiguous along K).
//
// In the tiled kernel of mq_gemm_packed.hip the waves that multiply also issue the stage's direct-to-LDS loads.
// The address unit of a compute unit takes 64 bytes per clock, so the 16 KB of a 128 x 128 stage occupy it for
// 256 clocks -- as long as the step's matrix instructions take -- and a wave whose load waits in that queue cannot
// issue anything else meanwhile.  Here two extra waves per workgroup do nothing but load: they wait for a stage to
// land, meet the others at the step's barrier, and issue the stage that reuses the slot everybody has just left;
// the multiplying waves only read fragments and multiply.  Two loaders, because a wave can have at most 63 loads
// outstanding and a deep pipeline needs more than that in flight.  (Measured against the tiled kernel when that
// one still issued a stage's loads as one burst after the barrier: 1-2 % faster; the tiled kernel has since
// learned to space its loads between its MFMAs, and the auto-tuner decides between the two per shape.)
//
// Same stages, same fragment order, same single barrier per K step and the same epilogue as the tiled kernel.
#include "mq_gemm_common.h"

namespace mq {

namespace {

template <int N>
__device__ __forceinline__ void wait_vmcnt_imm() {
  static_assert(N >= 0 && N <= 63, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);      // vmcnt only
}

__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr int kLoaders = 2;

// BM x BN tile, WM x WN multiplying waves, S stages of one 64-element K step each; EPI: kEpiRaw or kEpiDequant.
template <int BM, int BN, int WM, int WN, int S, int EPI>
__global__ __launch_bounds__((WM * WN + kLoaders) * 64) void k_gemm_prod(const Params p) {
  constexpr int NW = WM * WN;                  // multiplying waves; waves NW, NW + 1 load
  constexpr int TM = BM / WM / 32;
  constexpr int TN = BN / WN / 32;
  constexpr int FPB = 2;                       // fragments per 32-row block and K step
  constexpr int FA = (BM / 32) * FPB;
  constexpr int FB = (BN / 32) * FPB;
  constexpr int LT = FA + FB;                  // fragments per stage
  constexpr int LP = LT / kLoaders;            // per loader
  constexpr int STAGE = LT * kFragBytes;
  static_assert(LT % kLoaders == 0, "stage must divide over the loaders");
  static_assert(S >= 3 && (S - 1) * LP <= 63, "a loader's outstanding loads must fit the counter");
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);     // scalar: roles are scalar branches
  const bool loader = wave >= NW;
  const int wm = loader ? 0 : wave / WN, wn = loader ? 0 : wave % WN;
  unsigned tile_m, tile_n;
  tile_coords(p.tiles_m, p.tiles_n, BM >= 1024 ? 1u : 1024u / BM, tile_m, tile_n);
  const unsigned m0 = tile_m * BM, n0 = tile_n * BN;
  const PackedDims dA(8, p.M, p.K), dW(8, p.N, p.K);
  const unsigned KT = (unsigned)(dA.Kp / 64);

  v16i acc[TM][TN][1];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][0][r] = 0;

  if (loader) {
    // fragments [first, first + LP) of every stage: [0, FA) are A's, the rest the parameter's; row blocks
    // past the end are clamped (their results are masked in the epilogue)
    const int first = (wave - NW) * LP;
    const uint8_t* src[LP];
#pragma unroll
    for (int j = 0; j < LP; ++j) {
      const int i = first + j;
      if (i < FA) {
        size_t blk = (size_t)m0 / 32 + i / FPB;
        if (blk >= dA.nblocks) blk = dA.nblocks - 1;
        src[j] = p.qA + dA.frag_offset(blk, 0) + (size_t)(i % FPB) * kFragBytes + lane * 16;
      } else {
        size_t blk = (size_t)n0 / 32 + (i - FA) / FPB;
        if (blk >= dW.nblocks) blk = dW.nblocks - 1;
        src[j] = p.packedW + dW.frag_offset(blk, 0) + (size_t)((i - FA) % FPB) * kFragBytes + lane * 16;
      }
    }
    auto issue = [&](unsigned kt) {
      uint8_t* dst = smem + (kt % S) * STAGE + first * kFragBytes;
#pragma unroll
      for (int j = 0; j < LP; ++j)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(src[j] + (size_t)kt * (FPB * kFragBytes)),
            (__attribute__((address_space(3))) void*)(dst + j * kFragBytes), 16, 0, 0);
    };
#pragma unroll
    for (int st = 0; st < S - 1; ++st)
      if ((unsigned)st < KT) issue(st);
    // stage 0 (and, for the multiplying waves' first fragment reads, nothing more) has to be there
    if ((unsigned)(S - 2) < KT) wait_vmcnt_imm<(S - 2) * LP>();
    else wait_vmcnt_imm<0>();
    wg_barrier();
    for (unsigned kt = 0; kt < KT; ++kt) {
      // stage kt + 1 must have landed for everybody before the step's barrier; stages kt + 2 .. kt + S - 2
      // may stay in flight (none in the tail)
      if (kt + S - 2 < KT) wait_vmcnt_imm<(S - 3) * LP>();
      else wait_vmcnt_imm<0>();
      wg_barrier();
      // every multiplying wave is past slice 0 of stage kt, so stage kt - 1's slot is free
      if (kt + S - 1 < KT) issue(kt + S - 1);
    }
  } else {
    struct Frags {
      v4i a[TM];
      v4i b[TN];
    };
    constexpr int R = TM + TN;               // fragment reads per K slice
    constexpr int NM = TM * TN;              // MFMAs per K slice
    // r-th fragment read of slice ks of a stage, in the order the MFMAs need them
    auto read_one = [&](Frags& F, const uint8_t* st, int ks, int r) {
      const uint8_t* a_base = st + (wm * TM) * FPB * kFragBytes;
      const uint8_t* b_base = st + (FA + (wn * TN) * FPB) * kFragBytes;
      if (r < 1) {
        F.a[0] = as_v4i(*reinterpret_cast<const u4*>(a_base + ks * kFragBytes));
      } else if (r < 1 + TN) {
        const int nt = r - 1;
        F.b[nt] = as_v4i(*reinterpret_cast<const u4*>(b_base + (nt * 2 + ks) * kFragBytes));
      } else {
        const int mt = 1 + (r - 1 - TN);
        F.a[mt] = as_v4i(*reinterpret_cast<const u4*>(a_base + (mt * 2 + ks) * kFragBytes));
      }
    };
    auto mfma_one = [&](const Frags& F, int i) {
      const int mt = (i / TN) % TM, nt = i % TN;
      acc[mt][nt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[mt], F.b[nt], acc[mt][nt][0], 0, 0, 0);
    };
    // one slice out of `cur` while the reads of the next slice fill `nxt`: an LDS read rides behind each of
    // the first R MFMAs
    auto slice = [&](const Frags& cur, Frags& nxt, const uint8_t* next_stage, int next_ks) {
#pragma unroll
      for (int i = 0; i < (NM > R ? NM : R); ++i) {
        if (i < NM) mfma_one(cur, i);
        if (i < R) read_one(nxt, next_stage, next_ks, i);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    Frags f0, f1;
    wg_barrier();                                    // stage 0 is there
#pragma unroll
    for (int r = 0; r < R; ++r) read_one(f0, smem + lane * 16, 0, r);
    for (unsigned kt = 0; kt < KT; ++kt) {
      const uint8_t* cur = smem + (kt % S) * STAGE + lane * 16;
      const uint8_t* nxt = smem + ((kt + 1) % S) * STAGE + lane * 16;
      slice(f0, f1, cur, 1);                         // slice 0 of stage kt; slice 1's fragments stream in
      wg_barrier();                                  // stage kt + 1 is there; stage kt - 1 is free
      slice(f1, f0, nxt, 0);                         // slice 1; slice 0 of stage kt + 1 streams in (after the
                                                     // last stage: a finished slot again, result unused)
    }
  }

  // loaders pass through the epilogue with a tile origin past the matrix: they store nothing and take part
  // in its barrier
  const unsigned wave_m0 = loader ? p.M : m0 + wm * TM * 32;
  store_epilogue<8, TM, TN, 1, EPI, NW + kLoaders>(acc, p, wave_m0, n0 + wn * TN * 32, nullptr, nullptr);
}

template <int BM, int BN, int WM, int WN, int S, int EPI>
int launch_prod(const GemmArgs& a, hipStream_t s) {
  constexpr size_t smem = (size_t)S * ((BM / 32) + (BN / 32)) * 2 * kFragBytes;
  static_assert(smem <= 160 * 1024, "LDS budget");
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  auto kern = k_gemm_prod<BM, BN, WM, WN, S, EPI>;
  static bool attr_done = false;
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3((WM * WN + kLoaders) * 64), smem, s, p);
  return check_hip(hipGetLastError());
}

}  // namespace

// Variants 11 .. of the packed 8-bit products: `which` = 0: 128 x 128 tile, 8 multiplying waves (64 x 32
// each), 6 stages; 1: 128 x 128, 4 waves (64 x 64), 8 stages; 2: 256 x 128, 8 waves (64 x 64), 5 stages.
int launch_gemm_prod(const GemmArgs& a, Epilogue epi, int which, hipStream_t s) {
  if (a.bits != 8 || (epi != kEpiRaw && epi != kEpiDequant)) return MQ_ERR_UNSUPPORTED;
  const bool raw = epi == kEpiRaw;
  switch (which) {
    case 0: return raw ? launch_prod<128, 128, 2, 4, 6, kEpiRaw>(a, s) : launch_prod<128, 128, 2, 4, 6, kEpiDequant>(a, s);
    case 1: return raw ? launch_prod<128, 128, 2, 2, 8, kEpiRaw>(a, s) : launch_prod<128, 128, 2, 2, 8, kEpiDequant>(a, s);
    case 2: return raw ? launch_prod<256, 128, 4, 2, 5, kEpiRaw>(a, s) : launch_prod<256, 128, 4, 2, 5, kEpiDequant>(a, s);
    default: return MQ_ERR_UNSUPPORTED;
  }
}

}  // namespace mq
