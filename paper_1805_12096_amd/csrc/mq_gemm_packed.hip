// dot'_int with BOTH operands in fragment order (arxiv 1805.12096, Section 4.3:
// the product takes two already quantized tensors, each contiguous along K).
// Because activations and parameter share one packed layout, a stage of either
// is a run of 1 KB fragments that the CDNA4 direct-to-LDS load
// (global_load_lds_dwordx4: 64 lanes x 16 bytes land at consecutive LDS
// addresses) copies without touching registers.  That makes a deep software
// pipeline affordable: S stages of LDS, S - 1 of them in flight, which is what
// it takes to cover HBM latency with one or two waves per SIMD.
//
// Synchronisation per K step (one barrier, between the step's two 32-element slices):
//   wait until this wave's loads of stage kt + 1 have landed (vmcnt counts the
//   younger stages that may still be in flight), barrier (now everybody's have,
//   and everybody is done reading stage kt - 1).  The loads that overwrite stage
//   kt - 1's slot are issued one at a time between the MFMAs of the following two
//   slices; fragments are read from LDS one slice ahead of the MFMAs that use them.
// The compiler does not track LDS written by these loads, so the waits are
// explicit and the barrier is fenced against compile-time motion by hand.
#include <type_traits>

#include "mq_gemm_common.h"
#include "mq_grid_max.h"

namespace mq {

namespace {

// kPCoopFast: kPCoop for the common case the launcher can see in advance -- ReLU on and no tile reaching past the
// matrix -- where the re-quantization shrinks to one rounding addition per element (see the store below).
enum PackedEpilogue { kPRaw = 0, kPDequant = 1, kPAmax = 2, kPRequant = 3, kPCoop = 4, kPCoopFast = 5 };

// One element of quant_int (8 bit): binary32 multiply, round half to even, clamp, NaN -> 0.
__device__ __forceinline__ int quant8(float x, float s) {
  const float r = rintf(__fmul_rn(x, s));
  // the hardware conversion saturates and maps NaN to 0, which a C cast does not promise
  int i;
  asm("v_cvt_i32_f32 %0, %1" : "=v"(i) : "v"(r));
  return min(max(i, -127), 127);
}

__device__ __forceinline__ void wait_vmcnt(int n) {
  // s_waitcnt with only vmcnt active: vmcnt is split over bits [3:0] and [15:14]
  switch (n) {
#define MQ_CASE(N) case N: __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | 0x0F70); break;
    MQ_CASE(0) MQ_CASE(1) MQ_CASE(2) MQ_CASE(3) MQ_CASE(4) MQ_CASE(5) MQ_CASE(6) MQ_CASE(7) MQ_CASE(8)
    MQ_CASE(9) MQ_CASE(10) MQ_CASE(11) MQ_CASE(12) MQ_CASE(13) MQ_CASE(14) MQ_CASE(15) MQ_CASE(16)
    MQ_CASE(17) MQ_CASE(18) MQ_CASE(19) MQ_CASE(20) MQ_CASE(21) MQ_CASE(22) MQ_CASE(23) MQ_CASE(24) MQ_CASE(26)
#undef MQ_CASE
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
  }
}

__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int BITS, int BM, int BN, int WM, int WN, int S, int EPI, bool PF = true>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm_pp(const Params p) {
  constexpr int NW = WM * WN;
  constexpr int NPL = BITS == 16 ? 2 : 1;
  constexpr int TM = BM / WM / 32;
  constexpr int TN = BN / WN / 32;
  constexpr int NACC = BITS == 16 ? 3 : 1;
  constexpr int FPB = 2 * NPL;                 // fragments per 32-row block and 64-element K step
  constexpr int FA = (BM / 32) * FPB;          // fragments of A per stage
  constexpr int FB = (BN / 32) * FPB;
  constexpr int L = (FA + FB) / NW;            // direct-to-LDS loads per wave and stage
  constexpr int STAGE = (FA + FB) * kFragBytes;
  static_assert((FA + FB) % NW == 0, "stage must divide evenly over the waves");
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile shape");
  static_assert(S >= 3 && (S - 2) * L <= 24, "wait_vmcnt table");

  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = tid / 64;
  const int wm = wave / WN, wn = wave % WN;
  if constexpr (EPI == kPCoop || EPI == kPCoopFast) {
    // the agreement words of the kernel that ran before this one (a caller that keeps them clean between calls
    // instead of clearing them with a launch of their own): nobody uses them while this kernel runs
    if (p.clear_words != nullptr && blockIdx.x == 0)
      for (unsigned i = tid; i < p.nclear; i += NW * 64) p.clear_words[i] = 0u;
  }
  unsigned tile_m, tile_n;
  tile_coords(p.tiles_m, p.tiles_n, BM >= 1024 ? 1u : 1024u / BM, tile_m, tile_n);
  const unsigned m0 = tile_m * BM, n0 = tile_n * BN;
  const PackedDims dA(BITS, p.M, p.K), dW(BITS, p.N, p.K);
  const unsigned KT = (unsigned)(dA.Kp / 64);
  // the fused epilogues' dequantization factor: its two loads and the division are out of the way early
  float u_early = 0.f;
  if constexpr (EPI == kPAmax || EPI == kPRequant || EPI == kPCoop || EPI == kPCoopFast)
    u_early = __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
  // the tile's biases go to LDS before the main loop: fetched from global memory in the epilogue they are a full
  // memory round trip that nothing hides
  __shared__ float sbias[BN];
  float bias_early = 0.f;
  constexpr bool kBiasLds = BITS == 8 && (EPI == kPAmax || EPI == kPRequant || EPI == kPCoop || EPI == kPCoopFast);
  if constexpr (kBiasLds) {
    static_assert(NW * 64 >= BN, "one thread per column of the tile");
    if (tid < BN && p.bias != nullptr && n0 + tid < p.N) bias_early = p.bias[n0 + tid];
  }
  // 16 bit: the row and column sums the recombination needs (and the re-quantizing epilogue's biases) go to LDS
  // before the main loop as well; fetched in the epilogue they are dependent memory round trips per sub-tile
  __shared__ int32_t s_rowsum[BITS == 16 ? BM : 1];
  __shared__ int32_t s_colsum[BITS == 16 ? BN : 1];
  __shared__ float s_bias16[BITS == 16 && EPI == kPRequant ? BN : 1];
  if constexpr (BITS == 16) {
    const int32_t* rs = reinterpret_cast<const int32_t*>(p.qA + dA.plane_bytes());
    const int32_t* cs = reinterpret_cast<const int32_t*>(p.packedW + dW.plane_bytes());
    for (unsigned i = tid; i < (unsigned)BM; i += NW * 64) s_rowsum[i] = m0 + i < p.M ? rs[m0 + i] : 0;
    for (unsigned i = tid; i < (unsigned)BN; i += NW * 64) s_colsum[i] = n0 + i < p.N ? cs[n0 + i] : 0;
    if constexpr (EPI == kPRequant)
      for (unsigned i = tid; i < (unsigned)BN; i += NW * 64)
        s_bias16[i] = (p.bias != nullptr && n0 + i < p.N) ? p.bias[n0 + i] : 0.0f;
  }
  // the dequantizing epilogue's biases: one per lane and column block, in registers across the main loop
  float bias_pre[TN];
  if constexpr (EPI == kPDequant) {
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
      const unsigned n = n0 + (wn * TN + nt) * 32 + lane % 32;
      bias_pre[nt] = (p.bias != nullptr && n < p.N) ? p.bias[n] : 0.f;
    }
  }

  // Source of this wave's j-th load of a stage: fragment i = wave * L + j of the
  // stage; fragments [0, FA) are A's, the rest the parameter's.  Row blocks past
  // the end are clamped (their results are masked in the epilogue).
  const uint8_t* src[L];
#pragma unroll
  for (int j = 0; j < L; ++j) {
    const int i = wave * L + j;
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
  // this wave's j-th load of stage kt
  auto issue_frag = [&](unsigned kt, int j) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(src[j] + (size_t)kt * (FPB * kFragBytes)),
        (__attribute__((address_space(3))) void*)(smem + (kt % S) * STAGE + (wave * L + j) * kFragBytes), 16, 0, 0);
  };
  auto issue = [&](unsigned kt) {
#pragma unroll
    for (int j = 0; j < L; ++j) issue_frag(kt, j);
  };
  // One load of a stage, without a branch: past the last stage the same instruction re-reads stage 0
  // into a per-wave dummy slot behind the stages, so that every K step issues exactly L loads and the
  // loads can sit between MFMAs (a burst of them right after the barrier stalls in the address queue
  // and holds up the wave's MFMAs with it).
  auto issue_one = [&](unsigned kt, int j) {
    const bool real = kt < KT;
    const unsigned k2 = real ? kt : 0;
    uint8_t* dst = real ? smem + (kt % S) * STAGE + (wave * L + j) * kFragBytes : smem + S * STAGE + wave * kFragBytes;
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(src[j] + (size_t)k2 * (FPB * kFragBytes)),
        (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
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

  // Fragment registers of one 32-element K slice: TM operand fragments of A
  // and TN of the parameter (times two byte planes for 16 bit).
  struct Frags {
    v4i a[TM][NPL];
    v4i b[TN][NPL];
  };
  constexpr int PR = BITS == 16 ? 4 : 1;          // 8-bit products per result tile and K slice
  constexpr int R = (TM + TN) * NPL;              // fragment reads per K slice
  constexpr int NM = TM * TN * PR;                // MFMAs per K slice

  // r-th fragment read of slice ks of a stage, in the order the MFMAs need them:
  // A block 0, every parameter block, then the other A blocks.
  auto read_one = [&](Frags& F, const uint8_t* st, int ks, int r) {
    const uint8_t* a_base = st + (wm * TM) * FPB * kFragBytes;
    const uint8_t* b_base = st + (FA + (wn * TN) * FPB) * kFragBytes;
    if (r < NPL) {
      F.a[0][r] = as_v4i(*reinterpret_cast<const u4*>(a_base + (ks * NPL + r) * kFragBytes));
    } else if (r < NPL + TN * NPL) {
      const int q = r - NPL, nt = q / NPL, pl = q % NPL;
      F.b[nt][pl] = as_v4i(*reinterpret_cast<const u4*>(b_base + ((nt * 2 + ks) * NPL + pl) * kFragBytes));
    } else {
      const int q = r - NPL - TN * NPL, mt = 1 + q / NPL, pl = q % NPL;
      F.a[mt][pl] = as_v4i(*reinterpret_cast<const u4*>(a_base + ((mt * 2 + ks) * NPL + pl) * kFragBytes));
    }
  };
  // i-th MFMA of a slice.  The product index is the slowest, so consecutive
  // instructions never accumulate into the same registers.
  auto mfma_one = [&](const Frags& F, int i) {
    const int pr = i / (TM * TN), mt = (i / TN) % TM, nt = i % TN;
    if constexpr (BITS == 8) {
      // the re-quantizing epilogue wants consecutive n in one lane (4 bytes = one store), i.e. the
      // parameter as operand `a`; everything else wants consecutive n across lanes
      acc[mt][nt][0] = (EPI == kPRequant || EPI == kPCoop || EPI == kPCoopFast)
                           ? __builtin_amdgcn_mfma_i32_32x32x32_i8(F.b[nt][0], F.a[mt][0], acc[mt][nt][0], 0, 0, 0)
                           : __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[mt][0], F.b[nt][0], acc[mt][nt][0], 0, 0, 0);
    } else {
      const int pa = (pr == 0 || pr == 1) ? 0 : NPL - 1;          // hh, hl, lh, ll
      const int pb = (pr == 0 || pr == 2) ? 0 : NPL - 1;
      const int ai = pr == 0 ? 0 : (pr == 3 ? NACC - 1 : NACC - 2);
      // the re-quantizing epilogue wants four consecutive n of one row in a lane: parameter as operand `a`
      acc[mt][nt][ai] = EPI == kPRequant
                            ? __builtin_amdgcn_mfma_i32_32x32x32_i8(F.b[nt][pb], F.a[mt][pa], acc[mt][nt][ai], 0, 0, 0)
                            : __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[mt][pa], F.b[nt][pb], acc[mt][nt][ai], 0, 0, 0);
    }
  };
  // Multiply one slice out of `cur` while the reads of the next slice fill `nxt`:
  // one LDS read rides behind each of the first R MFMAs, and the scheduling
  // fences keep the compiler from regrouping them, so LDS latency hides behind
  // the matrix pipeline instead of stalling it.
  auto slice = [&](const Frags& cur, Frags& nxt, const uint8_t* next_stage, int next_ks) {
#pragma unroll
    for (int i = 0; i < (NM > R ? NM : R); ++i) {
      if (i < NM) mfma_one(cur, i);
      if (i < R) read_one(nxt, next_stage, next_ks, i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // As `slice`, with loads [j0, j1) of stage kt_load issued one at a time, evenly spaced between the MFMAs: a burst
  // of them queues in the address unit (64 bytes per clock) and holds the wave's MFMAs up behind it.
  auto slice_ld = [&](const Frags& cur, Frags& nxt, const uint8_t* next_stage, int next_ks, unsigned kt_load, int j0, int j1) {
    const int nl = j1 - j0;
    const int every = nl > 0 && NM / nl > 0 ? NM / nl : 1;
    int issued = 0;
#pragma unroll
    for (int i = 0; i < (NM > R ? NM : R); ++i) {
      if (i < NM) mfma_one(cur, i);
      if (i < R) read_one(nxt, next_stage, next_ks, i);
      if (i < NM && (i + 1) % every == 0 && issued < nl) {
        issue_frag(kt_load, j0 + issued);
        ++issued;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (; issued < nl; ++issued) issue_frag(kt_load, j0 + issued);
  };

  if constexpr (PF) {
    if (KT >= (unsigned)(S - 1)) {
#pragma unroll
      for (int st = 0; st < S - 2; ++st) issue(st);
      // stage S - 2: the first half here, the second behind slice 0 of step 0, as in every later step
#pragma unroll
      for (int j = 0; j < L / 2; ++j) issue_frag(S - 2, j);
    } else {
#pragma unroll
      for (int st = 0; st < S - 1; ++st)
        if ((unsigned)st < KT) issue(st);
    }
  } else {
#pragma unroll
    for (int st = 0; st < S - 1; ++st)
#pragma unroll
      for (int j = 0; j < L; ++j) issue_one(st, j);
  }
  if constexpr (kBiasLds) {
    if (tid < BN) sbias[tid] = bias_early;      // visible to everybody after the barrier below
  }
  if constexpr (PF) {
    Frags f0, f1;
    const bool longk = KT >= (unsigned)(S - 1);
    if (longk) wait_vmcnt((S - 3) * L + L / 2);      // everything but stage 0 may still be in flight
    else wait_vmcnt(0);
    block_barrier();
#pragma unroll
    for (int r = 0; r < R; ++r) read_one(f0, smem + lane * 16, 0, r);
    // One K step: slice 0 of stage kt (slice 1's fragments stream in behind it), the wait for stage kt + 1 and the
    // barrier, slice 1 (slice 0 of stage kt + 1 streams in; after the last stage that reads a finished slot again and
    // the result is unused).  Stage kt + S - 1 goes into the slot of stage kt - 1, free once every wave is past this
    // step's barrier: its first half is issued behind slice 1 (LD1), its second half behind slice 0 of the next step
    // (LD0), so S - 3 whole stages stay in flight across the wait.  The loop is peeled by what a step issues (all,
    // the last half stage, nothing) so that each body is straight-line code.
    auto step = [&](unsigned kt, auto ld0, auto ld1, auto drain) {
      const uint8_t* cur = smem + (kt % S) * STAGE + lane * 16;
      const uint8_t* nxt = smem + ((kt + 1) % S) * STAGE + lane * 16;
      if constexpr (decltype(ld0)::value) slice_ld(f0, f1, cur, 1, kt + S - 2, L / 2, L);
      else slice(f0, f1, cur, 1);
      if constexpr (decltype(drain)::value) wait_vmcnt(0);
      else wait_vmcnt((S - 3) * L);
      block_barrier();
      if constexpr (decltype(ld1)::value) slice_ld(f1, f0, nxt, 0, kt + S - 1, 0, L / 2);
      else slice(f1, f0, nxt, 0);
    };
    using T = std::true_type;
    using F = std::false_type;
    unsigned kt = 0;
    if (longk) {
      const unsigned KM = KT - (unsigned)(S - 1);
      for (; kt < KM; ++kt) step(kt, T{}, T{}, F{});
      step(kt, T{}, F{}, F{});
      ++kt;
    }
    for (; kt < KT; ++kt) step(kt, F{}, F{}, T{});
  } else {
    // Register-lean variant for tiles whose accumulators leave no room for a second fragment
    // set: fragments are read right before use (the compiler moves a slice's reads up behind the last MFMAs of
    // the slice before as their registers fall free); with two waves per SIMD the other wave's MFMAs
    // cover the rest of the LDS latency.  One barrier per K step.  Every step issues L loads (real or dummy), so
    // S - 2 steps' worth may always stay in flight.
    Frags f;
    // The step's barrier sits inside slice 1, before its last TAIL MFMAs: by then every fragment of stage kt has
    // been read (the wait on the LDS counter makes sure), so the slot is free for everybody and stage kt + 1 is
    // checked in; the first fragments of stage kt + 1 are read behind those last MFMAs instead of in a gap after
    // the barrier, where all waves of the workgroup would read at the same time with the matrix pipeline idle.
    constexpr int TAIL = NM / 2 > 0 ? NM / 2 : 1;
    constexpr int SPAN = 2 * NM - TAIL;                           // MFMAs before the barrier: all loads go there
    constexpr int EVERY2 = SPAN / L > 0 ? SPAN / L : 1;
    wait_vmcnt((S - 2) * L);
    block_barrier();
#pragma unroll
    for (int r = 0; r < R; ++r) read_one(f, smem + lane * 16, 0, r);
    for (unsigned kt = 0; kt < KT; ++kt) {
      const uint8_t* cur = smem + (kt % S) * STAGE + lane * 16;
      const uint8_t* nxt = smem + ((kt + 1) % S) * STAGE + lane * 16;
      int issued = 0;
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        mfma_one(f, i);
        if (i % EVERY2 == EVERY2 - 1 && issued < L) {
          issue_one(kt + S - 1, issued);
          ++issued;
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) read_one(f, cur, 1, r);
#pragma unroll
      for (int i = 0; i < NM - TAIL; ++i) {
        mfma_one(f, i);
        if ((NM + i) % EVERY2 == EVERY2 - 1 && issued < L) {
          issue_one(kt + S - 1, issued);
          ++issued;
        }
      }
#pragma unroll
      for (; issued < L; ++issued) issue_one(kt + S - 1, issued);
      // stage kt + 1 has landed (the newest (S - 2) L loads are stage kt + 2 .. kt + S - 1) and nobody reads stage kt
      // any more: every read of it has returned
      __builtin_amdgcn_s_waitcnt(0xC07F);                         // lgkmcnt(0)
      wait_vmcnt((S - 2) * L);
      block_barrier();
#pragma unroll
      for (int i = NM - TAIL; i < NM; ++i) mfma_one(f, i);
      // after the last stage this reads a slot nobody writes any more; the result is unused
#pragma unroll
      for (int r = 0; r < R; ++r) read_one(f, nxt, 0, r);
    }
    wait_vmcnt(0);     // dummy loads of the tail must not outlive the stages' reuse in the epilogue
  }

  if constexpr (EPI == kPRequant && BITS == 16) {
    // 16-bit product re-quantized with a multiplier known in advance (the paper's 16-bit scheme, Section 4.2:
    // one fixed multiplier): y = relu?(fma(float(sum), u, bias[n])), q = clamp(rne(y s), +-32767), written as the
    // packed 16-bit activations of the next product -- high-byte plane, low-byte plane, and sum_n q per row
    // (added up over the tile columns with one atomic per row and wave; the caller's launcher zeroes them).
    // Operands were swapped: register r of lane l is (n, m) = (8 (r / 4) + 4 (l / 32) + r % 4, l % 32).
    const int lj = lane % 32, lh = lane / 32;
    const float u = __fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW));
    const float s2 = *p.s_out;
    const bool relu = p.relu != 0;
    const unsigned wm0 = m0 + wm * TM * 32, wn0 = n0 + wn * TN * 32;
    const PackedDims dO(16, p.M, p.N);
    int32_t* rowsum_out = reinterpret_cast<int32_t*>(p.packed_out + dO.plane_bytes());
    __syncthreads();                               // every wave is done reading the last stage
    uint8_t* scratch = smem + wave * 2 * kFragBytes;     // one sub-tile's two planes
    // The usual case -- ReLU on, no row or column of the tile past the end, a positive finite multiplier -- needs less
    // arithmetic per element, and this epilogue is bound by it (33 million elements with the matrix cores idle):
    // after ReLU 0 <= y (NaN became 0), so quant_int is t = min(y s2, 32767) and one rounding addition:
    // t + 1.5 * 2^23 rounds t to the nearest integer, ties to even like rint, and leaves it in the low mantissa bits;
    // byte permutes cut the two planes out of four such words at a time, and the row sums are dot products of the
    // planes' bytes with ones (every value is non-negative, so is its high byte).
    const bool fast = relu && m0 + BM <= p.M && n0 + BN <= p.N && s2 > 0.0f && s2 < __builtin_inff();
    if (fast) {
      unsigned racc[TM];
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) racc[mt] = 0;
#pragma unroll
      for (int nt = 0; nt < TN; ++nt) {
        unsigned ccol[16];
        float bcol[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const unsigned nl = wn0 - n0 + nt * 32 + 8 * (j / 4) + 4 * lh + j % 4;
          ccol[j] = 128u * (unsigned)s_colsum[nl] - 16384u * p.K;
          bcol[j] = s_bias16[nl];
        }
#pragma unroll
        for (int mt = 0; mt < TM; ++mt) {
          const unsigned m = wm0 + mt * 32 + lj;
          const unsigned corr_m = 128u * (unsigned)s_rowsum[m - m0];
          unsigned sum_lo = 0, sum_hi = 0;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint32_t w[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const int r = 4 * q + t;
              const unsigned v = ((unsigned)acc[mt][nt][0][r] << 16) + ((unsigned)acc[mt][nt][NACC - 2][r] << 8) +
                                 (unsigned)acc[mt][nt][NACC - 1][r] + corr_m + ccol[r];
              const float y = fmaxf(fmaf((float)(int)v, u, bcol[r]), 0.0f);
              w[t] = __float_as_uint(__fadd_rn(fminf(__fmul_rn(y, s2), 32767.0f), 12582912.0f));
            }
            const uint32_t lo = __builtin_amdgcn_perm(w[1], w[0], 0x0c0c0400u) | __builtin_amdgcn_perm(w[3], w[2], 0x04000c0cu);
            const uint32_t hi = __builtin_amdgcn_perm(w[1], w[0], 0x0c0c0501u) | __builtin_amdgcn_perm(w[3], w[2], 0x05010c0cu);
            sum_lo = __builtin_amdgcn_udot4(lo, 0x01010101u, sum_lo, false);
            sum_hi = __builtin_amdgcn_udot4(hi, 0x01010101u, sum_hi, false);
            const unsigned at = (lj + 32 * (q / 2)) * 16 + 8 * (q % 2) + 4 * lh;
            *reinterpret_cast<uint32_t*>(scratch + at) = hi;
            *reinterpret_cast<uint32_t*>(scratch + kFragBytes + at) = lo ^ 0x80808080u;
          }
          __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): the wave's own writes
          const u4 vh = *reinterpret_cast<const u4*>(scratch + lane * 16);
          const u4 vl = *reinterpret_cast<const u4*>(scratch + kFragBytes + lane * 16);
          uint8_t* dst = p.packed_out + dO.frag_offset((wm0 + mt * 32) / 32, (wn0 + nt * 32) / 32) + lane * 16;
          *reinterpret_cast<u4*>(dst) = vh;
          *reinterpret_cast<u4*>(dst + kFragBytes) = vl;
          __builtin_amdgcn_s_waitcnt(0xC07F);          // the reads must finish before the next sub-tile overwrites
          racc[mt] += sum_lo + 256u * sum_hi;
        }
      }
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        int rowacc = (int)racc[mt];
        rowacc += __shfl_xor(rowacc, 32, 64);
        if (lh == 0) atomicAdd(&rowsum_out[wm0 + mt * 32 + lj], rowacc);
      }
    } else
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const unsigned m = wm0 + mt * 32 + lj;
      const bool m_ok = m < p.M;
      const unsigned corr_m = 128u * (unsigned)s_rowsum[m - m0] - 16384u * p.K;
      int rowacc = 0;
#pragma unroll
      for (int nt = 0; nt < TN; ++nt) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint32_t hi = 0, lo = 0;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int r = 4 * q + t;
            const unsigned n = wn0 + nt * 32 + 8 * q + 4 * lh + t;
            const unsigned v = ((unsigned)acc[mt][nt][0][r] << 16) + ((unsigned)acc[mt][nt][NACC - 2][r] << 8) +
                               (unsigned)acc[mt][nt][NACC - 1][r] + corr_m + 128u * (unsigned)s_colsum[n - n0];
            float y = fmaf((float)(int)v, u, s_bias16[n - n0]);
            if (relu) y = fmaxf(y, 0.0f);                       // NaN -> 0 like (y > 0) ? y : 0
            const float rr = rintf(__fmul_rn(y, s2));
            int qi;
            asm("v_cvt_i32_f32 %0, %1" : "=v"(qi) : "v"(rr));   // saturates, NaN -> 0
            qi = min(max(qi, -32767), 32767);
            if (!(m_ok && n < p.N)) qi = 0;                     // padding is the value 0, as the quantizer writes it
            rowacc += qi;
            hi |= (uint32_t)((qi >> 8) & 0xFF) << (8 * t);
            lo |= (uint32_t)((qi & 0xFF) ^ 0x80) << (8 * t);
          }
          const unsigned at = (lj + 32 * (q / 2)) * 16 + 8 * (q % 2) + 4 * lh;
          *reinterpret_cast<uint32_t*>(scratch + at) = hi;
          *reinterpret_cast<uint32_t*>(scratch + kFragBytes + at) = lo;
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): the wave's own writes
        const u4 vh = *reinterpret_cast<const u4*>(scratch + lane * 16);
        const u4 vl = *reinterpret_cast<const u4*>(scratch + kFragBytes + lane * 16);
        const unsigned mrow = wm0 + mt * 32, ncol = wn0 + nt * 32;
        if (mrow < dO.Np && ncol < dO.Kp) {
          uint8_t* dst = p.packed_out + dO.frag_offset(mrow / 32, ncol / 32) + lane * 16;
          *reinterpret_cast<u4*>(dst) = vh;
          *reinterpret_cast<u4*>(dst + kFragBytes) = vl;
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);          // the reads must finish before the next sub-tile overwrites
      }
      rowacc += __shfl_xor(rowacc, 32, 64);
      if (lh == 0 && m_ok) atomicAdd(&rowsum_out[m], rowacc);
    }
  } else if constexpr (EPI == kPAmax || EPI == kPRequant || EPI == kPCoop || EPI == kPCoopFast) {
    static_assert(BITS == 8, "fused epilogues are 8 bit");
    constexpr bool COOP = EPI == kPCoop || EPI == kPCoopFast;
    constexpr bool FASTC = EPI == kPCoopFast;
    const bool relu_on = FASTC || p.relu != 0;
    __shared__ float red[NW];
    const int lj = lane % 32, lh = lane / 32;
    const float u = u_early;
    const unsigned wm0 = m0 + wm * TM * 32, wn0 = n0 + wn * TN * 32;
    // a tile with no row or column past the end needs no masking anywhere below
    const bool interior = FASTC || (m0 + BM <= p.M && n0 + BN <= p.N);
    constexpr bool SWAPPED = EPI != kPAmax;
    // bias[n] of this tile (0 without a bias vector or past the last column): in LDS since before the main loop
    auto bias_at = [&](unsigned n) -> float { return sbias[n - n0]; };
    // swapped layout: the 16 registers of a sub-tile are 16 columns n; their biases are fetched once
    float biasv[SWAPPED ? TN : 1][16];
    if constexpr (SWAPPED) {
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
#pragma unroll
        for (int j = 0; j < 16; ++j) biasv[nt][j] = bias_at(wn0 + nt * 32 + 8 * (j / 4) + 4 * lh + j % 4);
    }

    // ---- max|y| of this block, y = relu?(fma((float)acc, u, bias[n])) as in the storing epilogue.
    // For one column n the value y is a monotonic function of the integer sum (both
    // the conversion and the fused multiply-add round monotonically), so max|y| over the rows of a
    // column is reached at the largest or the smallest sum (whatever the sign of u): the rows are reduced as integers and the
    // float expression is evaluated once (with ReLU) or twice per column instead of once per element.
    if constexpr (EPI == kPAmax || COOP) {
      float local = 0.f;
      // with ReLU and u > 0 only the largest sum of a column matters
      const bool max_only = relu_on && u > 0.0f;
      auto column = [&](int imax, int imin, unsigned n, float bias) {
        if (n < p.N && imax >= imin) {                       // imax < imin: no valid row in this lane
          const float hi = fmaf((float)imax, u, bias), lo = fmaf((float)imin, u, bias);
          if (relu_on) local = fmaxf(local, fmaxf(hi, lo));   // max(relu(y)) = max(0, y at an extreme sum)
          else local = fmaxf(local, fmaxf(fabsf(hi), fabsf(lo)));
        }
      };
      auto reduce_rows = [&](auto interior_tag, auto max_only_tag) {
        constexpr bool INTERIOR = decltype(interior_tag)::value;
        constexpr bool MAX_ONLY = decltype(max_only_tag)::value;
        if constexpr (!SWAPPED) {
          // register r of lane l is (m, n) = (8 (r / 4) + 4 (l / 32) + r % 4, l % 32): a lane holds one column
#pragma unroll
          for (int nt = 0; nt < TN; ++nt) {
            int imax = INT_MIN, imin = INT_MAX;
#pragma unroll
            for (int mt = 0; mt < TM; ++mt)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const unsigned m = wm0 + mt * 32 + 8 * (r / 4) + 4 * lh + r % 4;
                const int v = acc[mt][nt][0][r];
                if (INTERIOR || m < p.M) {
                  imax = max(imax, v);
                  if (!MAX_ONLY) imin = min(imin, v);
                }
              }
            if (MAX_ONLY && (INTERIOR || imax != INT_MIN)) imin = imax;
            column(imax, imin, wn0 + nt * 32 + lj, bias_at(wn0 + nt * 32 + lj));
          }
        } else {
          // operands swapped: register j of lane l is (n, m) = (8 (j / 4) + 4 (l / 32) + j % 4, l % 32)
#pragma unroll
          for (int nt = 0; nt < TN; ++nt)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              int imax = INT_MIN, imin = INT_MAX;
#pragma unroll
              for (int mt = 0; mt < TM; ++mt) {
                const unsigned m = wm0 + mt * 32 + lj;
                const int v = acc[mt][nt][0][j];
                if (INTERIOR || m < p.M) {
                  imax = max(imax, v);
                  if (!MAX_ONLY) imin = min(imin, v);
                }
              }
              if (MAX_ONLY && (INTERIOR || imax != INT_MIN)) imin = imax;
              column(imax, imin, wn0 + nt * 32 + 8 * (j / 4) + 4 * lh + j % 4, biasv[nt][j]);
            }
        }
      };
      if constexpr (FASTC) {
        if (max_only) reduce_rows(std::true_type{}, std::true_type{});
        else reduce_rows(std::true_type{}, std::false_type{});
      } else {
        if (interior && max_only) reduce_rows(std::true_type{}, std::true_type{});
        else if (interior) reduce_rows(std::true_type{}, std::false_type{});
        else reduce_rows(std::false_type{}, std::false_type{});
      }
      local = __uint_as_float(wave_max_u32(__float_as_uint(local)));   // local >= 0: bit patterns order like floats
      if (lane == 0) red[wave] = local;
      __syncthreads();
      if constexpr (EPI == kPAmax) {
        if (tid == 0) {
          float m = red[0];
#pragma unroll
          for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);
          p.partial[blockIdx.x] = m;
        }
      } else {
        // ---- grid-wide agreement on max|y|: every workgroup of the launch is resident (the launcher
        // checked), each publishes its maximum and collects everybody's.
        // While the maxima travel, every wave turns its sums into y in place (the float's bits in the
        // accumulator registers): that part of the epilogue does not need the multiplier.
        auto sums_to_y = [&]() {
#pragma unroll
          for (int nt = 0; nt < TN; ++nt)
#pragma unroll
            for (int mt = 0; mt < TM; ++mt)
#pragma unroll
              for (int j = 0; j < 16; ++j) {
                float y = fmaf((float)acc[mt][nt][0][j], u, biasv[SWAPPED ? nt : 0][j]);
                if (relu_on) y = fmaxf(y, 0.0f);
                acc[mt][nt][0][j] = __float_as_int(y);
              }
        };
        if (tid == 0) {
          float m = red[0];
#pragma unroll
          for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);
          grid_max_publish(p.barrier, m);
        }
        sums_to_y();
        if (wave == 0) {
          const float amax = grid_max_collect(p.barrier, p.barrier_ticks);
          if (lane == 0) red[0] = amax;
        }
        __syncthreads();
      }
    }

    if constexpr (EPI != kPAmax) {
      float s2;
      if constexpr (COOP) {
        const float amax = red[0];
        s2 = (amax > 0.0f) ? __fdiv_rn(127.0f, amax) : 1.0f;
      } else if (p.partial != nullptr) {
        // multiplier of the output from the partial maxima of the first pass (every block forms it)
        float amax = 0.f;
        for (unsigned i = tid; i < p.npartial; i += NW * 64) amax = fmaxf(amax, p.partial[i]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        if (lane == 0) red[wave] = amax;
        __syncthreads();
        amax = red[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) amax = fmaxf(amax, red[w]);
        s2 = (amax > 0.0f) ? __fdiv_rn(127.0f, amax) : 1.0f;
        if (blockIdx.x == 0 && tid == 0) *p.s_out = s2;
      } else {
        s2 = *p.s_out;      // fixed multiplier supplied by the caller (the paper's scheme): single pass
      }
      // operands were swapped: register r of lane l is (n, m) = (8 (r / 4) + 4 (l / 32) + r % 4, l % 32),
      // so r = 4 q .. 4 q + 3 are four consecutive n of one row m: one dword of the packed output.
      // Each 32 x 32 sub-tile is exactly one 1 KB fragment of the output; it is assembled in LDS (the
      // pipeline stages are free now) and leaves as one 16-byte store per lane, 1 KB contiguous.
      const PackedDims dO(8, p.M, p.N);
      __syncthreads();                             // every wave is done reading the last stage
      uint8_t* scratch = smem + wave * kFragBytes;
      const bool relu = relu_on;
      auto store_tiles = [&](auto interior_tag) {
        constexpr bool INTERIOR = decltype(interior_tag)::value;
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
#pragma unroll
          for (int mt = 0; mt < TM; ++mt) {
            const unsigned m = wm0 + mt * 32 + lj;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              int qv[4];
#pragma unroll
              for (int t = 0; t < 4; ++t) {
                const unsigned n = wn0 + nt * 32 + 8 * q + 4 * lh + t;
                float y;
                if constexpr (COOP) {
                  y = __int_as_float(acc[mt][nt][0][4 * q + t]);    // converted while waiting for the maximum
                } else {
                  y = fmaf((float)acc[mt][nt][0][4 * q + t], u, biasv[SWAPPED ? nt : 0][4 * q + t]);
                  if (relu) y = fmaxf(y, 0.0f);                     // NaN -> 0 like (y > 0) ? y : 0
                }
                const int v = quant8(y, s2);
                qv[t] = (INTERIOR || (n < p.N && m < p.M)) ? v : 0;   // padding stays zero
              }
              const uint32_t word = (uint32_t)(qv[0] & 0xFF) | ((uint32_t)(qv[1] & 0xFF) << 8) |
                                    ((uint32_t)(qv[2] & 0xFF) << 16) | ((uint32_t)(qv[3] & 0xFF) << 24);
              // slot of row m in the fragment: lj + 32 (K half); the 4 bytes sit at 8 (q % 2) + 4 lh
              *reinterpret_cast<uint32_t*>(scratch + (lj + 32 * (q / 2)) * 16 + 8 * (q % 2) + 4 * lh) = word;
            }
            // the wave reads back what it wrote itself: only its own LDS operations need to be complete
            __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
            const u4 v = *reinterpret_cast<const u4*>(scratch + lane * 16);
            const unsigned mrow = wm0 + mt * 32, ncol = wn0 + nt * 32;
            if (INTERIOR || (mrow < dO.Np && ncol < dO.Kp))
              *reinterpret_cast<u4*>(p.packed_out + dO.frag_offset(mrow / 32, ncol / 32) + lane * 16) = v;
            __builtin_amdgcn_s_waitcnt(0xC07F);      // the read must finish before the next sub-tile overwrites
          }
        }
      };
      // kPCoopFast: after ReLU every y lies in [0, max] (NaN became 0), and the multiplier is 127 / max rounded,
      // so y s2 <= 127 (1 + 2^-23)^2 rounds to at most 127: no clamp can act and no NaN can arrive.  The
      // conversion is then one addition: t + 1.5 * 2^23 rounds t to the nearest integer (ties to even: the
      // adder's own rounding, the same as rint of the same t) and leaves it in the low mantissa bits, whose low
      // byte is the quantized value; byte permutes gather four of them.  An infinite max gives s2 = 0 and
      // products 0 or (inf * 0 =) NaN, whose low byte is 0 like the clamp-and-NaN rule's result.
      auto store_tiles_fast = [&]() {
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
#pragma unroll
          for (int mt = 0; mt < TM; ++mt) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              uint32_t w[4];
#pragma unroll
              for (int t = 0; t < 4; ++t)
                w[t] = __float_as_uint(__fadd_rn(__fmul_rn(__int_as_float(acc[mt][nt][0][4 * q + t]), s2), 12582912.0f));
              const uint32_t word = __builtin_amdgcn_perm(w[1], w[0], 0x0c0c0400u) | __builtin_amdgcn_perm(w[3], w[2], 0x04000c0cu);
              *reinterpret_cast<uint32_t*>(scratch + (lj + 32 * (q / 2)) * 16 + 8 * (q % 2) + 4 * lh) = word;
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): the wave's own writes
            const u4 v = *reinterpret_cast<const u4*>(scratch + lane * 16);
            *reinterpret_cast<u4*>(p.packed_out + dO.frag_offset((wm0 + mt * 32) / 32, (wn0 + nt * 32) / 32) + lane * 16) = v;
            __builtin_amdgcn_s_waitcnt(0xC07F);      // the read must finish before the next sub-tile overwrites
          }
        }
      };
      if constexpr (FASTC) {
        store_tiles_fast();
      } else {
        if (interior) store_tiles(std::true_type{});
        else store_tiles(std::false_type{});
      }
      if constexpr (COOP) {
        if (blockIdx.x == 0 && tid == 0) {
          *p.s_out = grid_max_failed(p.barrier) ? __builtin_nanf("") : s2;
        }
      }
    }
  } else {
    store_epilogue<BITS, TM, TN, NACC, EPI == kPRaw ? kEpiRaw : kEpiDequant, NW>(
        acc, p, m0 + wm * TM * 32, n0 + wn * TN * 32, s_rowsum, s_colsum, EPI == kPDequant ? bias_pre : nullptr, m0, n0);
  }
}

template <int BITS, int BM, int BN, int WM, int WN, int S, int EPI, bool PF = true>
int launch_pp(const GemmArgs& a, hipStream_t s) {
  constexpr int NPL = BITS == 16 ? 2 : 1;
  constexpr size_t smem = (size_t)S * ((BM / 32) + (BN / 32)) * 2 * NPL * kFragBytes + (PF ? 0 : WM * WN * kFragBytes);
  static_assert(smem <= 160 * 1024, "LDS budget");
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  p.amax_slots = a.amax_slots;
  p.partial = a.partial; p.npartial = a.npartial; p.s_out = a.s_out; p.packed_out = static_cast<uint8_t*>(a.packed_out);
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  auto kern = k_gemm_pp<BITS, BM, BN, WM, WN, S, EPI, PF>;
  static bool attr_done = false;
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(WM * WN * 64), smem, s, p);
  return check_hip(hipGetLastError());
}

template <int BITS, int EPI>
int launch_pp_variant(const GemmArgs& a, int variant, hipStream_t s) {
  if constexpr (BITS == 8) {
    switch (variant) {
      case 1: return launch_pp<8, 256, 256, 2, 4, 4, EPI>(a, s);   // 8 waves, 128x64 per wave
      case 2: return launch_pp<8, 256, 256, 2, 2, 4, EPI>(a, s);   // 4 waves, 128x128 per wave
      case 3: return launch_pp<8, 128, 128, 2, 2, 4, EPI>(a, s);   // small tile, 64x64 per wave
      case 4: return launch_pp<8, 256, 128, 4, 2, 4, EPI>(a, s);   // 8 waves, 64x64 per wave
      case 5: return launch_pp<8, 128, 128, 2, 2, 8, EPI>(a, s);   // small tile, deep pipeline (6 stages in flight)
      case 6: return launch_pp<8, 256, 128, 4, 2, 6, EPI>(a, s);   // 8 waves, 64x64 per wave, deep pipeline
      case 7: return launch_pp<8, 128, 64, 2, 2, 8, EPI>(a, s);    // very small tile for narrow results
      case 8: return launch_pp<8, 128, 128, 4, 2, 6, EPI>(a, s);   // small tile, 8 waves (32x64 each): more loads in flight
      case 9: return launch_pp<8, 128, 128, 2, 4, 6, EPI>(a, s);   // small tile, 8 waves (64x32 each)
      default: return MQ_ERR_UNSUPPORTED;
    }
  } else {
    switch (variant) {
      case 1: return launch_pp<16, 128, 128, 4, 2, 4, EPI>(a, s);  // 8 waves, 32x64 per wave
      case 2: return launch_pp<16, 128, 128, 2, 2, 4, EPI>(a, s);  // 4 waves, 64x64 per wave
      case 3: return launch_pp<16, 64, 128, 2, 2, 4, EPI>(a, s);   // small tile, 32x64 per wave
      case 4: return launch_pp<16, 256, 128, 4, 2, 3, EPI, false>(a, s);   // 8 waves, 64x64 per wave, lean registers
      case 5: return launch_pp<16, 128, 128, 4, 2, 4, EPI, false>(a, s);   // as 1 without fragment prefetch
      default: return MQ_ERR_UNSUPPORTED;
    }
  }
}

}  // namespace

namespace {
// Tile configuration of the fused 8-bit passes: the large tile when it fills the chip, else the small one.
int fused_variant(const GemmArgs& a) {
  int v = forced_variant();
  if (v <= 0) v = tuned_variant(8, a.M, a.N, a.K);
  if (v <= 0 || v == 2 || v > 9) v = ((a.M + 255) / 256) * ((a.N + 255) / 256) >= 200 ? 1 : 3;
  return v;
}
size_t tiles_of(int variant, size_t M, size_t N) {
  size_t bm = 256, bn = 256;
  switch (variant) {
    case 3: case 5: case 8: case 9: bm = 128; bn = 128; break;
    case 4: case 6: bm = 256; bn = 128; break;
    case 7: bm = 128; bn = 64; break;
    default: break;
  }
  return ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
}
}  // namespace

int packed_variant_count(int bits) { return bits == 8 ? 14 : 8; }

// Upper bound on the partials the amax pass writes for an [M x N] result (any variant).
size_t gemm_amax_partials(size_t M, size_t N) { return ((M + 127) / 128) * ((N + 63) / 64); }

int launch_gemm_amax_partial(const GemmArgs& a, float* partials, hipStream_t s) {
  GemmArgs b = a;
  b.partial = partials;
  return launch_pp_variant<8, kPAmax>(b, fused_variant(a), s);
}

int launch_gemm_requant(const GemmArgs& a, const float* partials, float* s_out, void* packed_out, hipStream_t s) {
  GemmArgs b = a;
  const int v = fused_variant(a);
  b.partial = const_cast<float*>(partials);
  b.npartial = (unsigned)tiles_of(v, a.M, a.N);     // what the amax pass wrote with the same variant
  b.s_out = s_out;
  b.packed_out = packed_out;
  return launch_pp_variant<8, kPRequant>(b, v, s);
}

static unsigned long long g_barrier_ticks = 50ull * 1000 * 1000;     // 0.5 s of the 100 MHz wall clock
unsigned long long barrier_timeout_ticks() { return g_barrier_ticks; }
void set_barrier_timeout_ticks(unsigned long long ticks) { g_barrier_ticks = ticks; }

template <int BM, int BN, int WM, int WN, int S>
int launch_coop(const GemmArgs& a, hipStream_t s) {
  constexpr size_t smem = (size_t)S * ((BM / 32) + (BN / 32)) * 2 * kFragBytes;
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  const size_t tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu;
  p.s_out = a.s_out;
  p.packed_out = static_cast<uint8_t*>(a.packed_out);
  p.barrier = a.barrier;
  p.barrier_ticks = barrier_timeout_ticks();
  p.clear_words = a.clear_words;
  p.nclear = a.nclear;
  if (a.barrier == nullptr) return MQ_ERR_NULL;
  // ReLU and no partial tile: the kernel whose re-quantization is one addition per element
  const bool fast = a.relu != 0 && a.M % BM == 0 && a.N % BN == 0;
  auto kern = fast ? k_gemm_pp<8, BM, BN, WM, WN, S, kPCoopFast> : k_gemm_pp<8, BM, BN, WM, WN, S, kPCoop>;
  static int max_blocks_of[2] = {-1, -1};       // workgroups the device can hold at once, asked once per kernel
  int& max_blocks = max_blocks_of[fast ? 1 : 0];
  if (max_blocks < 0) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    int per_cu = 0, dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern), WM * WN * 64, smem) != hipSuccess)
      return MQ_ERR_HIP;
    max_blocks = per_cu * cus;
  }
  // the grid-wide barrier needs every workgroup resident at the same time (and has a slot)
  static_assert(BM == 256 && BN == 256 && kBarrierSlots == 256, "single_pass_fits assumes this tile and slot count");
  if (!single_pass_fits(a.M, a.N, (size_t)max_blocks)) return MQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(WM * WN * 64), smem, s, p);
  return check_hip(hipGetLastError());
}

// Product + bias (+ReLU) -> max|y| -> quant_int(y) in ONE launch, for results of at most one tile per
// resident workgroup.  MQ_ERR_UNSUPPORTED otherwise (the caller then runs the two-pass version).
// The kBarrierWords words at barrier must be zero when the kernel starts (an earlier kernel on the stream
// clears them); should the barrier ever time out, *s_out becomes NaN and so does everything computed from it.
int launch_gemm_requant_coop(const GemmArgs& a, float* s_out, void* packed_out, unsigned* barrier,
                             hipStream_t s) {
  GemmArgs b = a;
  b.barrier = barrier;
  b.s_out = s_out;
  b.packed_out = packed_out;
  return launch_coop<256, 256, 2, 4, 4>(b, s);
}

// Single-pass re-quantizing product with a multiplier known in advance (fixed multipliers as in the
// paper): quant_int of the next layer's input happens in the producing epilogue.
int launch_gemm_requant_fixed(const GemmArgs& a, const float* s_fixed, void* packed_out, hipStream_t s) {
  GemmArgs b = a;
  b.partial = nullptr;
  b.npartial = 0;
  b.s_out = const_cast<float*>(s_fixed);
  b.packed_out = packed_out;
  return launch_pp_variant<8, kPRequant>(b, fused_variant(a), s);
}

// 16-bit product re-quantized with a fixed multiplier into packed 16-bit activations (planes + row sums).
// The row sums are accumulated with atomics: they are zeroed here by a small launch first.
int launch_gemm_requant_fixed_i16(const GemmArgs& a, const float* s_fixed, void* packed_out, hipStream_t s) {
  const PackedDims dO(16, a.M, a.N);
  int rc = launch_clear_words(reinterpret_cast<unsigned*>(static_cast<uint8_t*>(packed_out) + dO.plane_bytes()),
                              (unsigned)dO.Np, s);
  if (rc != MQ_OK) return rc;
  GemmArgs b = a;
  b.s_out = const_cast<float*>(s_fixed);
  b.packed_out = packed_out;
  // (measured against the 256 x 128 tile of the fastest plain product on one device in alternation, config 4's first
  // product: 136 us here, 143 us there -- its 192 accumulator registers leave this epilogue too few to work with)
  return launch_pp<16, 128, 128, 4, 2, 4, kPRequant>(b, s);
}

int launch_gemm_packed(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  int v = forced_variant();
  if (v <= 0) v = tuned_variant(a.bits, a.M, a.N, a.K);     // frozen by mq_autotune_gemm for this shape, or 0
  if (v <= 0) {
    // Shape heuristic standing in for a per-shape timing run: the largest tile that still gives
    // every compute unit work, smaller tiles for small problems.
    if (a.bits == 16) {
      const size_t t = ((a.M + 255) / 256) * ((a.N + 127) / 128);
      // enough big tiles to fill the chip: the workgroup per compute unit that walks through them (measured 2 - 7 %
      // ahead of one workgroup per tile, the more the shorter K is)
      v = a.M <= 512 ? 6 : (t >= 200 ? 8 : (((a.M + 127) / 128) * ((a.N + 127) / 128) >= 128 ? 1 : 3));
    } else {
      // small problems (a decode step's 300 sentences) are latency bound: the split-K kernel (variant 10)
      // fetches all operands of a workgroup in one round trip
      const size_t t256 = ((a.M + 255) / 256) * ((a.N + 255) / 256);
      const size_t t128 = ((a.M + 127) / 128) * ((a.N + 127) / 128);
      v = a.M <= 512 ? 10 : (t256 >= 200 ? 1 : (t128 >= 128 ? 3 : 7));
    }
  }
  if ((a.bits == 8 && v == 10) || (a.bits == 16 && v == 6)) return launch_gemm_small(a, epi, s);
  if (a.bits == 16 && v == 7) return launch_gemm_dot2(a, epi, s);                        // vector ALU instead of matrix cores
  if (a.bits == 16 && v == 8) {                                                          // one workgroup per CU, tile after tile
    if (a.K > 64 && a.K < ((size_t)1 << 26)) return launch_gemm_pers16(a, epi, s);
    v = 4;                                                       // a single K step (or an absurdly long K): the tile kernel it derives from
  }
  if (a.bits == 8 && v >= 11 && v <= 13) return launch_gemm_prod(a, epi, v - 11, s);     // loading waves apart
  if (a.bits == 8 && v == 14) return launch_gemm_ks(a, epi, s);                          // K split over two wave groups
  if (a.bits == 8)
    return epi == kEpiRaw ? launch_pp_variant<8, kPRaw>(a, v, s) : launch_pp_variant<8, kPDequant>(a, v, s);
  return epi == kEpiRaw ? launch_pp_variant<16, kPRaw>(a, v, s) : launch_pp_variant<16, kPDequant>(a, v, s);
}

}  // namespace mq
