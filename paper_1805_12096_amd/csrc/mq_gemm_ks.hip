// dot'_int on packed 8-bit operands with K split over two wave groups of one workgroup
// (arxiv 1805.12096, Section 4.3: the product of two quantized tensors, both contiguous along K).
//
// For results that only fill the chip with 128 x 128 tiles (the second product of the base FFN block:
// 8192 x 512 gives 256 tiles, one per compute unit) the tiled kernel of mq_gemm_packed.hip runs one wave per
// SIMD: whenever that wave waits -- for its fragments, for the next stage, at the step's barrier -- the
// matrix pipeline of its SIMD idles, and a K step holds only 8 MFMAs per wave between two barriers.
// Here the workgroup has eight waves: two groups of four, each group covering the whole 128 x 128 tile
// (64 x 64 per wave) for every other 64-element K step.  A stage of the ring is 128 elements of K; all eight
// waves load it (4 fragments each, one at a time between their MFMAs), group g multiplies its half.  Per SIMD
// there are now two independent waves, a barrier comes once per 128 elements, and the number of fragment
// reads per MFMA stays that of the 64 x 64 wave tile.  At the end group 1 hands its sums to group 0 through
// LDS (integer addition: the result does not depend on the split) and group 0 runs the shared epilogue.
#include <type_traits>

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

// 128 x 128 tile, 2 groups x (2 x 2) waves, S stages of 128 elements of K; EPI: kEpiRaw or kEpiDequant.
template <int S, int EPI>
__global__ __launch_bounds__(512) void k_gemm_ks(const Params p) {
  constexpr int BM = 128, BN = 128, TM = 2, TN = 2;
  constexpr int NW = 8;
  constexpr int FPB = 4;                       // fragments per 32-row block and stage (4 x 32 elements of K)
  constexpr int L = 4;                         // loads per wave and stage: wave w fetches row block w's fragments
  constexpr int STAGE = 8 * FPB * kFragBytes;  // 4 row blocks of A, 4 of the parameter
  static_assert(S >= 4 && (S - 3) * L + L / 2 <= 63, "ring depth");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const int lane = threadIdx.x % 64;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);     // scalar: the group is a scalar branch
  const int grp = wave / 4, wm = (wave % 4) / 2, wn = wave % 2;
  unsigned tile_m, tile_n;
  tile_coords(p.tiles_m, p.tiles_n, 1024u / BM, tile_m, tile_n);
  const unsigned m0 = tile_m * BM, n0 = tile_n * BN;
  const PackedDims dA(8, p.M, p.K), dW(8, p.N, p.K);
  const unsigned KT = (unsigned)(dA.Kp / 64);  // 64-element K steps
  const unsigned PT = (KT + 1) / 2;            // stages; with KT odd the last one has no second half
  const bool odd = (KT & 1u) != 0;

  // Waves 0..3 fetch A's row blocks, waves 4..7 the parameter's; row blocks past the end are clamped (their
  // results are masked in the epilogue).  Load j of a stage is the block's j-th fragment of that stage.
  const uint8_t* src;
  if (wave < 4) {
    size_t blk = (size_t)m0 / 32 + wave;
    if (blk >= dA.nblocks) blk = dA.nblocks - 1;
    src = p.qA + dA.frag_offset(blk, 0) + lane * 16;
  } else {
    size_t blk = (size_t)n0 / 32 + (wave - 4);
    if (blk >= dW.nblocks) blk = dW.nblocks - 1;
    src = p.packedW + dW.frag_offset(blk, 0) + lane * 16;
  }
  // With KT odd the last stage's fragments 2 and 3 do not exist (they would be the next row block's, or past
  // the buffer): fragments 0 and 1 are fetched again in their place and group 1 multiplies zeros there.
  auto issue_frag = [&](unsigned pt, int j) {
    const int jj = (odd && pt == PT - 1 && j >= 2) ? j - 2 : j;
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(src + ((size_t)pt * FPB + jj) * kFragBytes),
        (__attribute__((address_space(3))) void*)(smem + (pt % S) * STAGE + (wave * FPB + j) * kFragBytes), 16, 0, 0);
  };

  // the dequantizing epilogue's biases: one per lane and column block, in registers across the main loop
  float bias_pre[TN];
  if constexpr (EPI == kEpiDequant) {
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
      const unsigned n = n0 + (wn * TN + nt) * 32 + lane % 32;
      bias_pre[nt] = (p.bias != nullptr && n < p.N) ? p.bias[n] : 0.f;
    }
  }
  v16i acc[TM][TN][1];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][0][r] = 0;

  struct Frags {
    v4i a[TM];
    v4i b[TN];
  };
  constexpr int R = TM + TN, NM = TM * TN;
  // r-th fragment read of this group's slice ks (0 or 1) of a stage, in the order the MFMAs need them
  auto read_one = [&](Frags& F, const uint8_t* st, int ks, int r) {
    const uint8_t* a_base = st + ((wm * TM) * FPB + 2 * grp + ks) * kFragBytes;
    const uint8_t* b_base = st + ((4 + wn * TN) * FPB + 2 * grp + ks) * kFragBytes;
    if (r < 1) F.a[0] = as_v4i(*reinterpret_cast<const u4*>(a_base));
    else if (r < 1 + TN) F.b[r - 1] = as_v4i(*reinterpret_cast<const u4*>(b_base + (r - 1) * FPB * kFragBytes));
    else F.a[r - TN] = as_v4i(*reinterpret_cast<const u4*>(a_base + (r - TN) * FPB * kFragBytes));
  };
  auto mfma_one = [&](const Frags& F, int i) {
    const int mt = i / TN, nt = i % TN;
    acc[mt][nt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[mt], F.b[nt], acc[mt][nt][0], 0, 0, 0);
  };
  // One slice out of `cur` while the reads of the next slice fill `nxt`, one read behind each MFMA; with LOADS,
  // loads [j0, j0 + 2) of stage pt_load go out behind the second and the fourth MFMA.
  auto slice = [&](auto loads_tag, const Frags& cur, Frags& nxt, const uint8_t* next_stage, int next_ks,
                   unsigned pt_load, int j0) {
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      mfma_one(cur, i);
      read_one(nxt, next_stage, next_ks, i);
      if constexpr (decltype(loads_tag)::value) {
        if (i % 2 == 1) issue_frag(pt_load, j0 + i / 2);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_assert(R == NM, "one read per MFMA");

  const bool longk = PT >= (unsigned)(S - 1);
  if (longk) {
#pragma unroll
    for (int st = 0; st < S - 2; ++st)
#pragma unroll
      for (int j = 0; j < L; ++j) issue_frag(st, j);
    // stage S - 2: the first half here, the second behind slice 0 of step 0, as in every later step
    issue_frag(S - 2, 0);
    issue_frag(S - 2, 1);
    wait_vmcnt_imm<(S - 3) * L + L / 2>();
  } else {
#pragma unroll
    for (int st = 0; st < S - 1; ++st)
      if ((unsigned)st < PT)
#pragma unroll
        for (int j = 0; j < L; ++j) issue_frag(st, j);
    wait_vmcnt_imm<0>();
  }
  wg_barrier();
  Frags f0, f1;
#pragma unroll
  for (int r = 0; r < R; ++r) read_one(f0, smem + lane * 16, 0, r);
  const bool kill_last = odd && grp == 1;      // this group's K step of the last stage does not exist
  const v4i zero4 = {0, 0, 0, 0};
  // One stage: slice 0 (slice 1's fragments stream in behind it), the wait for stage pt + 1 and the barrier,
  // slice 1 (slice 0 of stage pt + 1 streams in; after the last stage that reads a finished slot again, unused).
  // Stage pt + S - 1 goes into the slot of stage pt - 1, free once every wave is past this stage's barrier: its
  // first half is issued behind slice 1 (LD1), its second half behind slice 0 of the next stage (LD0).
  auto step = [&](unsigned pt, auto ld0, auto ld1, auto drain) {
    const uint8_t* cur = smem + (pt % S) * STAGE + lane * 16;
    const uint8_t* nxt = smem + ((pt + 1) % S) * STAGE + lane * 16;
    if constexpr (decltype(drain)::value) {
      if (kill_last && pt == PT - 1) {
#pragma unroll
        for (int t = 0; t < TM; ++t) f0.a[t] = zero4;
      }
    }
    slice(ld0, f0, f1, cur, 1, pt + S - 2, 2);
    if constexpr (decltype(drain)::value) {
      wait_vmcnt_imm<0>();
      if (kill_last && pt == PT - 1) {
#pragma unroll
        for (int t = 0; t < TM; ++t) f1.a[t] = zero4;
      }
    } else {
      wait_vmcnt_imm<(S - 3) * L>();
    }
    wg_barrier();
    slice(ld1, f1, f0, nxt, 0, pt + S - 1, 0);
  };
  using T = std::true_type;
  using F = std::false_type;
  unsigned pt = 0;
  if (longk) {
    const unsigned KM = PT - (unsigned)(S - 1);
    for (; pt < KM; ++pt) step(pt, T{}, T{}, F{});
    step(pt, T{}, F{}, F{});
    ++pt;
  }
  for (; pt < PT; ++pt) step(pt, F{}, F{}, T{});

  // group 1's sums go to group 0 through the ring (every load has landed: the last stages waited for all of them)
  wg_barrier();
  v4i* xchg = reinterpret_cast<v4i*>(smem) + (size_t)(wave % 4) * (TM * TN * 4 * 64) + lane;
  if (grp == 1) {
#pragma unroll
    for (int t = 0; t < TM * TN; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const v16i& c = acc[t / TN][t % TN][0];
        xchg[(t * 4 + q) * 64] = v4i{c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]};
      }
  }
  wg_barrier();
  if (grp == 0) {
#pragma unroll
    for (int t = 0; t < TM * TN; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const v4i o = xchg[(t * 4 + q) * 64];
        v16i& c = acc[t / TN][t % TN][0];
        c[4 * q] += o.x; c[4 * q + 1] += o.y; c[4 * q + 2] += o.z; c[4 * q + 3] += o.w;
      }
  }
  // group 1 passes through the epilogue with a tile origin past the matrix: it stores nothing and takes part
  // in the epilogue's barrier
  const unsigned wave_m0 = grp == 0 ? m0 + wm * TM * 32 : p.M;
  store_epilogue<8, TM, TN, 1, EPI, NW>(acc, p, wave_m0, n0 + wn * TN * 32, nullptr, nullptr,
                                        EPI == kEpiDequant ? bias_pre : nullptr);
}

template <int S, int EPI>
int launch_ks(const GemmArgs& a, hipStream_t s) {
  constexpr size_t smem = (size_t)S * 8 * 4 * kFragBytes;
  static_assert(smem <= 160 * 1024, "LDS budget");
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (a.M + 127) / 128, tiles_n = (a.N + 127) / 128;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  auto kern = k_gemm_ks<S, EPI>;
  static bool attr_done = false;
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(512), smem, s, p);
  return check_hip(hipGetLastError());
}

}  // namespace

// Variant 14 of the packed 8-bit products: 128 x 128 tile, K split over two groups of four waves, 4 stages of 128.
int launch_gemm_ks(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  if (a.bits != 8 || (epi != kEpiRaw && epi != kEpiDequant)) return MQ_ERR_UNSUPPORTED;
  return epi == kEpiRaw ? launch_ks<4, kEpiRaw>(a, s) : launch_ks<4, kEpiDequant>(a, s);
}

}  // namespace mq
