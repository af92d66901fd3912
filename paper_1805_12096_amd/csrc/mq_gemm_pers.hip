// dot'_int for 16-bit operands (arxiv 1805.12096, Sections 4.2 and 4.3) with one workgroup per compute unit that walks
// through several result tiles (variant 8 of the packed 16-bit products).  The tile kernel it derives from (256 x 128
// tile, eight waves of 64 x 64, three-stage LDS ring, one barrier per 64-element K step, byte planes multiplied as four
// 8-bit matrix products into three accumulators) fills the LDS of a compute unit with one workgroup, so nothing covers a
// tile's start (launch, first operands' round trip to memory) or its end.  Here the K steps of all of a workgroup's
// tiles form one sequence: the loads run S - 1 steps ahead of the matrix instructions across tile boundaries, so the
// next tile's first stages arrive while the current tile's results are being stored.  A tile's row sums, column sums
// and biases come in by direct-to-LDS loads issued before its first K step, into the half of a double buffer the
// previous tile does not use; the accumulators start from zero inside a tile's first matrix instructions instead of
// being cleared between tiles; max|y| (when asked for) is published once per workgroup, after its last tile.  Same
// operands, same results as every other variant.
#include <type_traits>

#include "mq_gemm_common.h"

namespace mq {

namespace {

constexpr int kBM = 256, kBN = 128, kWM = 4, kWN = 2, kS = 3;
constexpr int kNW = kWM * kWN;                    // waves
constexpr int kTM = kBM / kWM / 32, kTN = kBN / kWN / 32;
constexpr int kFPB = 4;                           // fragments per 32-row block and K step: two K slices x two planes
constexpr int kFA = (kBM / 32) * kFPB, kFB = (kBN / 32) * kFPB;
constexpr int kL = (kFA + kFB) / kNW;             // direct-to-LDS loads per wave and stage
constexpr int kStage = (kFA + kFB) * kFragBytes;
constexpr size_t kPersLds = (size_t)kS * kStage + kNW * kFragBytes;   // the ring and one dummy slot per wave
static_assert((kFA + kFB) % kNW == 0, "stage must divide evenly over the waves");
static_assert(kPersLds + 2 * (kBM + 2 * kBN) * 4 + 64 <= 160 * 1024, "LDS budget");

// s_waitcnt with only vmcnt active (split over bits [3:0] and [15:14]): all but the newest kL loads have landed
__device__ __forceinline__ void wait_all_but_one_stage() {
  __builtin_amdgcn_s_waitcnt((kL & 0xF) | ((kL >> 4) << 14) | 0x0F70);
}

__device__ __forceinline__ void fenced_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// tile number (after the XCD remap of the workgroup index) -> tile coordinates, bands of GM tile rows, m fastest
__device__ __forceinline__ void tile_of(unsigned t, unsigned tiles_m, unsigned tiles_n, unsigned GM, unsigned& tile_m,
                                        unsigned& tile_n) {
  const unsigned band = t / (GM * tiles_n), in_band = t % (GM * tiles_n);
  const unsigned first = band * GM;
  const unsigned rows = tiles_m - first < GM ? tiles_m - first : GM;
  tile_m = first + in_band % rows;
  tile_n = in_band / rows;
}

// MULTI: the grid is smaller than the number of tiles, so workgroups take several; without it (at most one tile per
// compute unit) the tile-to-tile code drops out at compile time.
template <int EPI, bool MULTI>
__global__ __launch_bounds__(kNW * 64) void k_gemm_pers16(const Params p) {
  constexpr int NPL = 2, NACC = 3, TM = kTM, TN = kTN, L = kL, S = kS;
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  __shared__ int32_t s_rowsum[2][kBM];
  __shared__ int32_t s_colsum[2][kBN];
  __shared__ float s_bias[2][kBN];

  const int lane = threadIdx.x % 64;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);     // scalar: everything derived from it is too
  const int wm = wave / kWN, wn = wave % kWN;
  const PackedDims dA(16, p.M, p.K), dW(16, p.N, p.K);
  const unsigned KT = (unsigned)(dA.Kp / 64);            // at least S - 1 (the launcher sees to it)
  const unsigned T = p.tiles_m * p.tiles_n, G = gridDim.x;
  const unsigned first = xcd_remap(blockIdx.x, G);
  if (first >= T) return;
  const unsigned nmine = MULTI ? (T - first + G - 1) / G : 1u;        // this workgroup's tiles: first, first + G, ...
  const int32_t* rs = reinterpret_cast<const int32_t*>(p.qA + dA.plane_bytes());
  const int32_t* cs = reinterpret_cast<const int32_t*>(p.packedW + dW.plane_bytes());
  const unsigned lane16 = (unsigned)lane * 16u;
  float amax_run = 0.f;               // max |y| over all of this thread's results, published once at the end
  // the two multipliers are asked for now and divided after the first stages are on their way: the wait for them
  // would otherwise stand between the kernel's start and its first operand loads
  float s_a = 0.f, s_w = 0.f;
  if (EPI == kEpiDequant) { s_a = *p.sA; s_w = *p.sW; }

  // ---- the loading side: K step lk of this workgroup's lo-th tile goes to ring slot lslot ----
  const uint8_t* sbase[L];      // wave-uniform source of this wave's j-th fragment of K step 0 of the tile being loaded
  unsigned koff = 0;            // lk in bytes of one fragment row's run (K below 2^26)
  unsigned lo = 0, lk = 0, lslot = 0;
  unsigned dbase = 0, dstride = kFragBytes;   // LDS offset of this wave's first fragment of the stage, and per fragment
  auto set_loader_tile = [&](unsigned o) {
    unsigned tm, tn;
    tile_of(first + o * G, p.tiles_m, p.tiles_n, 1024u / kBM, tm, tn);
#pragma unroll
    for (int j = 0; j < L; ++j) {
      const int i = wave * L + j;
      const uint8_t* ptr;
      if (i < kFA) {
        size_t blk = (size_t)tm * (kBM / 32) + i / kFPB;
        if (blk >= dA.nblocks) blk = dA.nblocks - 1;     // row blocks past the end: clamped, masked in the epilogue
        ptr = p.qA + dA.frag_offset(blk, 0) + (size_t)(i % kFPB) * kFragBytes;
      } else {
        size_t blk = (size_t)tn * (kBN / 32) + (i - kFA) / kFPB;
        if (blk >= dW.nblocks) blk = dW.nblocks - 1;
        ptr = p.packedW + dW.frag_offset(blk, 0) + (size_t)((i - kFA) % kFPB) * kFragBytes;
      }
      // pinned to scalar registers: as vector registers the addresses would not fit beside the accumulators
      const uint64_t v = reinterpret_cast<uint64_t>(ptr);
      const uint32_t lo32 = __builtin_amdgcn_readfirstlane((uint32_t)v), hi32 = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
      sbase[j] = reinterpret_cast<const uint8_t*>(((uint64_t)hi32 << 32) | lo32);
    }
  };
  auto issue_one = [&](int j) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(sbase[j] + (size_t)koff + lane16),
        (__attribute__((address_space(3))) void*)(smem + dbase + j * dstride), 16, 0, 0);
  };
  // After a stage's L loads: on to the next K step, the next tile after the last one, and past the last tile the
  // same loads re-read the last tile's first K step into a per-wave dummy slot behind the ring, so that every step
  // issues exactly L loads and the wait counts stay the same.
  auto stage_issued = [&]() {
    lslot = lslot + 1 == (unsigned)S ? 0u : lslot + 1;
    koff += kFPB * kFragBytes;
    if (++lk == KT) {
      lk = 0;
      koff = 0;
      ++lo;
      if (lo < nmine) set_loader_tile(lo);
    }
    const bool real = lo < nmine;
    dbase = real ? lslot * kStage + wave * L * kFragBytes : S * kStage + wave * kFragBytes;
    dstride = real ? kFragBytes : 0;
    if (!real) koff = 0;
  };
  // A tile's sums and biases, one direct-to-LDS load of 64 words per wave: waves 0-3 the row sums, 4-5 the column
  // sums, 6-7 the biases.  Rows and columns past the end read a valid word; their results are never stored.  Issued
  // before the tile's first K step, the load is older than that step's loads, so the step's wait and barrier cover it.
  auto stage_sums = [&](unsigned o) {
    unsigned tm, tn;
    tile_of(first + o * G, p.tiles_m, p.tiles_n, 1024u / kBM, tm, tn);
    const unsigned par = o & 1u;
    const void* src;
    void* dst;
    if (wave < 4) {
      size_t i = (size_t)tm * kBM + wave * 64 + lane;
      if (i >= dA.Np) i = dA.Np - 1;
      src = rs + i;
      dst = &s_rowsum[par][wave * 64];
    } else if (wave < 6) {
      size_t i = (size_t)tn * kBN + (wave - 4) * 64 + lane;
      if (i >= dW.Np) i = dW.Np - 1;
      src = cs + i;
      dst = &s_colsum[par][(wave - 4) * 64];
    } else {
      if (p.bias == nullptr) return;
      size_t i = (size_t)tn * kBN + (wave - 6) * 64 + lane;
      if (i >= p.N) i = p.N - 1;
      src = p.bias + i;
      dst = &s_bias[par][(wave - 6) * 64];
    }
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)dst, 4, 0, 0);
  };

  // ---- the multiplying side ----
  v16i acc[TM][TN][NACC];
  struct Frags {
    v4i a[TM][NPL];
    v4i b[TN][NPL];
  };
  constexpr int R = (TM + TN) * NPL;      // fragment reads per 32-element K slice
  constexpr int NM = TM * TN * 4;         // MFMAs per K slice
  auto read_one = [&](Frags& F, const uint8_t* st, int ks, int r) {
    const uint8_t* a_base = st + (wm * TM) * kFPB * kFragBytes;
    const uint8_t* b_base = st + (kFA + (wn * TN) * kFPB) * kFragBytes;
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
  // i-th MFMA of a slice: high x high, high x low, low x high, low x low; the product index is the slowest, so
  // consecutive instructions never accumulate into the same registers
  // fresh: the accumulator's first instruction of a tile takes zero instead of the accumulator (of the three sums per
  // result tile the middle one gets two products per slice: only its first starts from zero)
  auto mfma_one = [&](const Frags& F, int i, bool fresh) {
    const int pr = i / (TM * TN), mt = (i / TN) % TM, nt = i % TN;
    const int pa = (pr == 0 || pr == 1) ? 0 : 1;
    const int pb = (pr == 0 || pr == 2) ? 0 : 1;
    const int ai = pr == 0 ? 0 : (pr == 3 ? 2 : 1);
    const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    acc[mt][nt][ai] =
        __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[mt][pa], F.b[nt][pb], fresh && pr != 2 ? zero : acc[mt][nt][ai], 0, 0, 0);
  };

  set_loader_tile(0);
  dbase = wave * L * kFragBytes;
#pragma unroll
  for (int st = 0; st < S - 1; ++st) {
#pragma unroll
    for (int j = 0; j < L; ++j) issue_one(j);
    stage_issued();
  }
  stage_sums(0);
  // stage 0 has landed once all but the newest L loads have (the sums' load makes that wait for one load more)
  wait_all_but_one_stage();
  fenced_barrier();
  float u = 0.f;
  if (EPI == kEpiDequant) u = __fdiv_rn(1.0f, __fmul_rn(s_a, s_w));

  Frags f;
  constexpr int TAIL = NM / 2;
  constexpr int SPAN = 2 * NM - TAIL;     // MFMAs of a K step before its barrier: the loads sit between them
  constexpr int EVERY = SPAN / L;
#pragma unroll
  for (int r = 0; r < R; ++r) read_one(f, smem + lane16, 0, r);
  unsigned slot = 0;
  // One K step on the stage in `slot`, straight-line code.  FIRST (a tile's first step): the accumulators start from
  // zero inside their first instructions; clearing 192 registers per lane between tiles would be 0.7 us of vector
  // instructions with the matrix cores idle.
  auto step = [&](auto first_c) {
    constexpr bool FIRST = decltype(first_c)::value;
    const unsigned nslot = slot + 1 == (unsigned)S ? 0u : slot + 1;
    const uint8_t* cur = smem + slot * kStage + lane16;
    const uint8_t* nxt = smem + nslot * kStage + lane16;
    int issued = 0;
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      mfma_one(f, i, FIRST);
      if (i % EVERY == EVERY - 1 && issued < L) {
        issue_one(issued);
        ++issued;
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) read_one(f, cur, 1, r);
#pragma unroll
    for (int i = 0; i < NM - TAIL; ++i) {
      mfma_one(f, i, false);
      if ((NM + i) % EVERY == EVERY - 1 && issued < L) {
        issue_one(issued);
        ++issued;
      }
    }
#pragma unroll
    for (; issued < L; ++issued) issue_one(issued);
    // the stage after this one has landed (only the newest L loads may be in flight) and this wave has read all of
    // the current one (every LDS read has returned): past the barrier that holds for everybody
    __builtin_amdgcn_s_waitcnt(0xC07F);                           // lgkmcnt(0)
    wait_all_but_one_stage();
    fenced_barrier();
#pragma unroll
    for (int i = NM - TAIL; i < NM; ++i) mfma_one(f, i, false);
    // the next stage's first fragments, behind the last MFMAs (after the last stage this reads a slot nobody writes
    // any more; the result is unused)
#pragma unroll
    for (int r = 0; r < R; ++r) read_one(f, nxt, 0, r);
    slot = nslot;
    stage_issued();
  };
  for (unsigned o = 0; o < nmine; ++o) {
    step(std::true_type{});
    for (unsigned kt = 1; kt < KT; ++kt) step(std::false_type{});
    // the tile is complete; its successor's first stages are in LDS or on their way
    unsigned tm, tn;
    tile_of(first + o * G, p.tiles_m, p.tiles_n, 1024u / kBM, tm, tn);
    const unsigned m0 = tm * kBM, n0 = tn * kBN, par = o & 1u;
    float bias_pre[TN];
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) bias_pre[nt] = p.bias != nullptr ? s_bias[par][(wn * TN + nt) * 32 + lane % 32] : 0.f;
    store_epilogue<16, TM, TN, NACC, EPI, kNW>(acc, p, m0 + wm * TM * 32, n0 + wn * TN * 32, s_rowsum[par], s_colsum[par],
                                               bias_pre, m0, n0, &u, &amax_run);
    if (o + 1 < nmine) stage_sums(o + 1);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): the dummy loads of the tail must not outlive the workgroup's LDS
  if (EPI == kEpiDequant && p.out_amax != nullptr) publish_block_amax<kNW>(p, amax_run);
}

}  // namespace

int launch_gemm_pers16(const GemmArgs& a, Epilogue epi, hipStream_t s) {
  if (a.bits != 16 || (epi != kEpiRaw && epi != kEpiDequant)) return MQ_ERR_UNSUPPORTED;
  if (PackedDims(16, a.M, a.K).Kp / 64 < (size_t)(kS - 1)) return MQ_ERR_UNSUPPORTED;   // the ring's prologue stays in the first tile
  if (a.K >= ((size_t)1 << 26)) return MQ_ERR_SHAPE;                                      // 32-bit byte offset along K
  const size_t tiles_m = (a.M + kBM - 1) / kBM, tiles_n = (a.N + kBN - 1) / kBN;
  if (tiles_m * tiles_n > 0x7FFFFFFFull) return MQ_ERR_SHAPE;
  Params p{};
  p.qA = static_cast<const uint8_t*>(a.qA);
  p.packedW = static_cast<const uint8_t*>(a.packedW);
  p.M = (unsigned)a.M; p.N = (unsigned)a.N; p.K = (unsigned)a.K;
  p.tiles_m = (unsigned)tiles_m;
  p.tiles_n = (unsigned)tiles_n;
  p.C = a.C; p.sA = a.sA; p.sW = a.sW; p.bias = a.bias; p.relu = a.relu; p.Y = a.Y; p.out_amax = a.out_amax;
  p.amax_slots = a.amax_slots;
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != MQ_OK) return rc;
    rc = check_hip(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    if (rc != MQ_OK) return rc;
    cus = n > 0 ? n : 256;
  }
  const unsigned grid = (unsigned)(tiles_m * tiles_n < (size_t)cus ? tiles_m * tiles_n : (size_t)cus);
  auto launch = [&](auto kern) -> int {
    static bool attr_done = false;
    if (!attr_done) {
      int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPersLds));
      if (rc != MQ_OK) return rc;
      attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kNW * 64), kPersLds, s, p);
    return check_hip(hipGetLastError());
  };
  if (tiles_m * tiles_n > (size_t)grid)
    return epi == kEpiRaw ? launch(k_gemm_pers16<kEpiRaw, true>) : launch(k_gemm_pers16<kEpiDequant, true>);
  return epi == kEpiRaw ? launch(k_gemm_pers16<kEpiRaw, false>) : launch(k_gemm_pers16<kEpiDequant, false>);
}

}  // namespace mq
