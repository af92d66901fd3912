// Greedy output layer of a decode step (arxiv 1805.12096, Section 2.3: with beam
// size 1 no softmax is evaluated, the word with the highest activation wins;
// Section 2.1: the output matrix is the tied 36 000-entry embedding).
//
// Shape of the problem: a few hundred sentences (M) against tens of thousands
// of vocabulary rows (N) at K = model size.  Per step the whole embedding has to
// stream through the chip once (N * K bytes) while the M x N logits never need
// to exist.  So:
//   * work is cut into units of 16 vocabulary rows (all of K), dealt round-robin
//     to one workgroup per compute unit; 36 000 rows give 2250 units, 8.8 per CU;
//   * the matrix instruction is v_mfma_i32_16x16x64_i8 with the embedding as
//     operand `a` and the hidden states as operand `b`: lane l then holds four
//     candidate words for ONE sentence (l % 16), so the running maxima are
//     plain per-lane registers and nothing crosses lanes until the very end;
//   * the quantized hidden states (M x K, a few 100 KB) are loaded once per
//     workgroup into REGISTERS as operand fragments, split over the four waves
//     by 16-sentence tile;
//   * the packed embedding streams through LDS with direct-to-LDS loads: each
//     load instruction gathers, for one 64-element K group, the 16 rows of the
//     unit out of two 32-row fragments, so that LDS receives exactly the
//     operand image (lane l at byte 16 l); many stages are in flight;
//   * sums of 8-bit products over K <= 512 stay below 2^23, so (sum << 8 |
//     255 - stage) is a 32-bit key whose integer maximum is the arg-max with
//     the earliest stage winning ties: two VALU operations per candidate;
//   * every workgroup writes one 64-bit (sum, index) key per sentence, its own
//     run of consecutive keys; a second small kernel reduces them and decodes.
//     No atomics, no initialisation.  (Folding that reduction into this kernel
//     was tried -- 64-bit atomic maxima per sentence with the last workgroup out
//     decoding -- and took three times as long: the 76 800 atomics serialise on
//     the few cache lines that hold the maxima.)
// 64-bit keys order by sum first and by smaller index second:
//   key = (sum ^ 0x80000000) << 32 | (0xFFFFFFFF - n);  0 means "no candidate".
#include <mutex>
#include <type_traits>

#include "mq_gemm_common.h"

namespace mq {

namespace {

constexpr int kWaves = 8;             // two per SIMD: one wave's waits hide behind the other's MFMAs
constexpr int kKG = 8;                // 64-element K groups per unit (K <= 512)
constexpr int kStages = 10;           // 80 KB of LDS, 8 stages in flight
constexpr int kMaxBlocks = 1024;      // upper bound on workgroups (columns of the partials array)

__device__ __forceinline__ void wait_vmcnt_n(int n) {
  switch (n) {
#define MQ_CASE(N) case N: __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | 0x0F70); break;
    MQ_CASE(0) MQ_CASE(1) MQ_CASE(2) MQ_CASE(3) MQ_CASE(4) MQ_CASE(5) MQ_CASE(6) MQ_CASE(7) MQ_CASE(8) MQ_CASE(9)
    MQ_CASE(10) MQ_CASE(11) MQ_CASE(12) MQ_CASE(13) MQ_CASE(14) MQ_CASE(15) MQ_CASE(16)
#undef MQ_CASE
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
  }
}

struct ArgmaxParams {
  const uint8_t* packedA;   // hidden states, packed 8 bit [M x K]
  const uint8_t* packedW;   // embedding, packed 8 bit [N x K]
  unsigned M, N, K;
  unsigned long long* partial;   // BEAM == 1: [gridDim.x][Mpad], Mpad = M rounded up to 16; beam search: [M][gridDim.x][BEAM]
  const int32_t* shortlist;      // optional: vocabulary rows to score, ascending; NULL = all N rows
  unsigned L;                    // candidates: shortlist length, or N
  // beam search (BEAM > 1): partial holds [M][gridDim.x][BEAM] keys, norm [M][gridDim.x] (max, sum) pairs of
  // the softmax normaliser in base 2, u2 = log2(e) / (sA sW) is formed in the kernel
  float2* norm;
  const float* sA;
  const float* sW;
  // beam search with more rows than one workgroup's registers hold: the grid's y index picks a chunk of chunk_rows
  // rows out of Mtotal (M, packedA, partial and norm above then describe the whole problem); 0 = M is the chunk
  unsigned chunk_rows, Mtotal;
};

// What lane l feeds to the 16x16x64 MFMA for rows 16 u .. 16 u + 15 of a packed
// 8-bit operand and K group g (64 elements): K quarter l / 16 of the group lives
// in fragment 2 g + l / 32, half (l / 16) % 2, row slot (u % 2) 16 + l % 16.
// The offset splits into a per-lane constant and a wave-uniform part.
__device__ __forceinline__ unsigned operand16_lane_offset(int lane) {
  return (unsigned)(lane / 32) * kFragBytes + (unsigned)(((lane / 16) % 2) * 32 + lane % 16) * 16;
}
__device__ __forceinline__ size_t operand16_uniform_offset(const PackedDims& d, size_t unit, unsigned g) {
  return d.frag_offset(unit / 2, 2 * g) + (unit % 2) * 256;
}

// TPW: 16-sentence tiles per wave (8 * TPW * 16 >= M).
// GATHER: candidates are the rows listed in p.shortlist (the lexical shortlist of Section 4.1: the
// output product restricted to a subset of the vocabulary).  A unit is then 16 consecutive shortlist
// positions; since every lane of a direct-to-LDS load supplies its own address, gathering the 16
// rows costs nothing extra.  Indices are candidate positions; the reduce kernel maps them back.

// BEAM > 1 (beam search, Table 2's b = 2 and b = 4 rows): every accumulator register keeps its BEAM best
// keys instead of one (sorted insertion: BEAM max / min pairs per candidate), and every sentence tile keeps
// a running (max, sum) of 2^(logit log2 e) so that the k best words come with normalised log-probabilities.
template <int TPW, bool GATHER, int BEAM = 1>
__global__ __launch_bounds__(kWaves * 64) void k_argmax_stream(const ArgmaxParams p_in) {
  ArgmaxParams p = p_in;
  if (BEAM > 1 && p_in.chunk_rows != 0) {
    // this workgroup's chunk of rows: the keys and normalisers are laid out by row, so a chunk's share starts at its
    // first row, and so do its packed hidden states (chunks are whole 32-row blocks)
    const unsigned row0 = blockIdx.y * p_in.chunk_rows;
    p.M = p_in.Mtotal - row0 < p_in.chunk_rows ? p_in.Mtotal - row0 : p_in.chunk_rows;
    p.packedA = p_in.packedA + PackedDims(8, p_in.Mtotal, p_in.K).frag_offset(row0 / 32, 0);
    p.partial = p_in.partial + (size_t)row0 * gridDim.x * BEAM;
    p.norm = p_in.norm + (size_t)row0 * gridDim.x;
  }
  constexpr int KG = kKG, S = kStages;
  constexpr int STAGE = KG * kFragBytes;
  static_assert(KG == kWaves, "one direct-to-LDS load per wave and stage");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const int lane = threadIdx.x % 64;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const PackedDims dA(8, p.M, p.K), dW(8, p.N, p.K);
  const unsigned kgroups = (unsigned)(dW.kfrags / 2);          // real K groups (<= KG)
  const unsigned nunits = GATHER ? (p.L + 15) / 16 : (unsigned)(dW.nblocks * 2);   // 16-candidate units
  const unsigned first = blockIdx.x, stride = gridDim.x;
  const unsigned nlocal = first < nunits ? (nunits - first + stride - 1) / stride : 0;
  const unsigned lane_off = operand16_lane_offset(lane);

  // stage s of the pipeline = this workgroup's s-th unit, all of K; wave w copies K group w
  // (K shorter than 512: a real group is copied again and its products are zeroed through `hid`)
  const unsigned my_group = (unsigned)wave < kgroups ? (unsigned)wave : kgroups - 1;
  const uint8_t* src_lane = p.packedW + lane_off;
  // GATHER: this workgroup's candidate rows, 16 per stage, are fetched into LDS once, before any
  // direct-to-LDS load is in flight (later ordinary loads would have to drain the pipeline)
  int32_t* rows_lds = reinterpret_cast<int32_t*>(smem + S * STAGE + kWaves * kFragBytes);
  if (GATHER) {
    for (unsigned i = threadIdx.x; i < nlocal * 16; i += kWaves * 64) {
      const unsigned pos = (first + (i / 16) * stride) * 16 + i % 16;
      // positions past the end are masked later; an id outside [0, N) reads the nearest row instead of memory
      // outside the embedding (the token reported for it is the id as listed)
      const int id = pos < p.L ? p.shortlist[pos] : p.shortlist[0];
      rows_lds[i] = min(max(id, 0), (int)p.N - 1);
    }
    __syncthreads();
  }
  // One load per wave for stage s.  Past the workgroup's last unit the same instruction fetches unit 0 again into a
  // per-wave slot behind the stages that nobody reads: every stage then issues exactly one load, the number of loads
  // in flight at a given point is a constant, and the waits need neither a branch nor a table.  Needs nlocal > 0.
  auto issue = [&](unsigned s_any) {
    const bool real = s_any < nlocal;
    const unsigned s = real ? s_any : 0;
    uint8_t* dst = real ? smem + (s % S) * STAGE + wave * kFragBytes : smem + S * STAGE + wave * kFragBytes;
    const uint8_t* src;
    if (GATHER) {
      const unsigned r = (unsigned)rows_lds[s * 16 + lane % 16];
      src = p.packedW + dW.frag_offset(r / 32, 2 * my_group + lane / 32) +
            (size_t)((r % 32) + 32 * ((lane / 16) % 2)) * 16;
    } else {
      src = src_lane + operand16_uniform_offset(dW, (size_t)first + (size_t)s * stride, my_group);
    }
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)src, (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
  };
  // The first two stages go out first (their memory latency is the longest wait of the kernel), then the
  // hidden-state operands of this wave's sentence tiles (tile t = wave + 8 i covers sentences 16 t ..
  // 16 t + 15; they come from L2, every workgroup reads the same ones), then the remaining stages.  The
  // memory counter retires loads in order, so waiting for "all but the newest n" later covers stages 0
  // and 1 and the operands while the newer stages are still on their way.  The operand loads are written
  // as instructions so that the waiting is ours: the compiler would wait for ALL outstanding loads, the
  // whole pipeline included, at the first use.
  constexpr int kEarly = 2;
#pragma unroll
  for (int s = 0; s < kEarly; ++s)
    if (nlocal > 0) issue(s);
  v4i hid[TPW][KG];
  const size_t tiles_avail = dA.nblocks * 2;
  // 16-sentence tiles this wave really owns (a slot beyond them would only repeat a tile): TPW or TPW - 1
  const int ntl = (size_t)wave < tiles_avail ? (int)((tiles_avail - 1 - wave) / kWaves) + 1 : 0;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    size_t t = (size_t)wave + kWaves * i;
    if (t >= tiles_avail) t = tiles_avail - 1;   // slot past the end: a copy, never multiplied, never written out
#pragma unroll
    for (int g = 0; g < KG; ++g) {
      const uint8_t* src = p.packedA + lane_off + operand16_uniform_offset(dA, t, (unsigned)g < kgroups ? g : 0);
      asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(hid[i][g]) : "v"(src) : "memory");
    }
  }
#pragma unroll
  for (int s = kEarly; s < S - 1; ++s)
    if (nlocal > 0) issue(s);

  // running maxima, one per accumulator register: (sum << 8) | (255 - stage).  Real sums exceed
  // -2^23, so a key whose sum field is -2^23 means "no candidate yet".
  constexpr int kNone = (int)0x80000000;
  int best[TPW][4];
  int more_best[BEAM > 1 ? TPW : 1][4][BEAM > 1 ? BEAM - 1 : 1];     // places 2 .. BEAM of each register's list
  float run_max[TPW], run_sum[TPW];                                    // softmax normaliser, base 2 (BEAM > 1)
  float u2 = 0.f;
  if constexpr (BEAM > 1) u2 = __fmul_rn(__fdiv_rn(1.0f, __fmul_rn(*p.sA, *p.sW)), 1.44269504088896340736f);
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    run_max[i] = -INFINITY;
    run_sum[i] = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      best[i][r] = kNone;
      if constexpr (BEAM > 1)
#pragma unroll
        for (int j = 0; j < BEAM - 1; ++j) more_best[i][r][j] = kNone;
    }
  }
  // one sentence tile's four new sums (one stage): keys into the sorted lists, logits into the normaliser;
  // valid[r] = false leaves candidate r out (padding past the last candidate)
  auto beam_update = [&](int i, const v4i& sums, int tag, bool v0, bool v1, bool v2, bool v3) {
    const bool valid[4] = {v0, v1, v2, v3};
    float f[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int key = valid[r] ? ((sums[r] << 8) | (tag & 255)) : kNone;
      const int t0 = max(best[i][r], key);
      key = min(best[i][r], key);
      best[i][r] = t0;
#pragma unroll
      for (int j = 0; j < BEAM - 1; ++j) {
        const int t = max(more_best[i][r][j], key);
        key = min(more_best[i][r][j], key);
        more_best[i][r][j] = t;
      }
      f[r] = valid[r] ? __fmul_rn((float)sums[r], u2) : -INFINITY;
    }
    const float mnew = fmaxf(fmaxf(run_max[i], fmaxf(f[0], f[1])), fmaxf(f[2], f[3]));
    if (mnew > -INFINITY) {          // (no valid candidate so far: nothing to add, and inf - inf is avoided)
      run_sum[i] = run_sum[i] * __builtin_amdgcn_exp2f(run_max[i] - mnew) + __builtin_amdgcn_exp2f(f[0] - mnew) +
                   __builtin_amdgcn_exp2f(f[1] - mnew) + __builtin_amdgcn_exp2f(f[2] - mnew) +
                   __builtin_amdgcn_exp2f(f[3] - mnew);
      run_max[i] = mnew;
    }
  };

  // Before stage s is multiplied, stages s and s + 1 must have landed (s + 1 is read from LDS into
  // registers while s is multiplied): of the loads issued so far the oldest s + 2 are needed, `newest` may be
  // outstanding.  With a load in every stage S - 1 + s have been issued (newest = S - 3); without, S - 1
  // (newest = S - 3 - s).
  auto land = [&](int newest) {
    wait_vmcnt_n(newest);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  auto read_stage = [&](unsigned s, v4i (&e)[KG]) {
    const uint8_t* st = smem + (s % S) * STAGE + lane * 16;
#pragma unroll
    for (int g = 0; g < KG; ++g) e[g] = as_v4i(*reinterpret_cast<const u4*>(st + g * kFragBytes));
  };

  // One stage: the unit's K groups (in `e`) against this wave's NT sentence tiles into `cur`, while the
  // maxima are updated from `prev` (the sums of the stage before) and the next unit is read from LDS
  // into `enext`.  The update's VALU work is cut into slices that sit between the MFMA groups, so it
  // runs while the matrix pipeline is busy instead of after it; the scheduling fences keep that order.
  auto stage = [&](auto nt_tag, auto refill_tag, int newest, unsigned s, v4i (&cur)[TPW], const v4i (&prev)[TPW],
                   const v4i (&e)[KG], v4i (&enext)[KG]) {
    constexpr int NT = decltype(nt_tag)::value;
    land(newest);
    // everybody is past stage s - 1 (and has its copy of stage s in registers), so slot s - 1 can be refilled
    if constexpr (decltype(refill_tag)::value) issue(s + S - 1);
    // the next unit's LDS reads are spread between the MFMA groups: eight reads in a row would fill the
    // LDS queue (all eight waves read at the same time) and hold this wave's MFMAs back behind them
    // (after the last unit they read a finished slot again and the result is unused)
    const uint8_t* nx = smem + ((s + 1) % S) * STAGE + lane * 16;
    const int prev_tag = 256 - (int)s;          // 255 - (s - 1); unused garbage for s == 0 (prev holds "none")
    constexpr int ITEMS = NT * 4, PER = (ITEMS + KG - 1) / KG;
    const v4i zero = {0, 0, 0, 0};
#pragma unroll
    for (int g = 0; g < KG; ++g) {
      enext[g] = as_v4i(*reinterpret_cast<const u4*>(nx + g * kFragBytes));
#pragma unroll
      for (int i = 0; i < NT; ++i)
        cur[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(e[g], hid[i][g], g == 0 ? zero : cur[i], 0, 0, 0);
      if constexpr (BEAM == 1) {
#pragma unroll
        for (int j = g * PER; j < (g + 1) * PER && j < ITEMS; ++j)
          best[j / 4][j % 4] = max(best[j / 4][j % 4], (prev[j / 4][j % 4] << 8) | (prev_tag & 255));
      } else {
        // one sentence tile of the stage before per MFMA group (stage 0 has no stage before it)
        if (g < NT && s > 0) beam_update(g < TPW ? g : 0, prev[g < TPW ? g : 0], prev_tag, true, true, true, true);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // two stages per trip so the two accumulator sets and the two unit buffers swap roles without copies
  v4i acc0[TPW], acc1[TPW], e0[KG], e1[KG];
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    acc0[i] = v4i{-8388608, -8388608, -8388608, -8388608};
    acc1[i] = v4i{-8388608, -8388608, -8388608, -8388608};   // "none" for stage 0's update
  }
  if (nlocal > 0) {
    // stage 0 has to be in registers before the loop, and so have the operands: everything but the
    // stages issued after the operands may still be outstanding
    wait_vmcnt_n(S - 1 - kEarly);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    read_stage(0, e0);
  } else {
    wait_vmcnt_n(0);
  }
  // the operands are older than every stage, so they are there now; K groups past the end of K are zeroed
#pragma unroll
  for (int i = 0; i < TPW; ++i)
#pragma unroll
    for (int g = 0; g < KG; ++g) {
      asm volatile("" : "+v"(hid[i][g]));
      if ((unsigned)g >= kgroups) hid[i][g] = v4i{0, 0, 0, 0};
    }
  auto run = [&](auto nt_tag) {
    if (nlocal <= (unsigned)(S - 1)) {
      // The usual case (36 000 rows over 256 workgroups are 9 units each): the prologue has issued everything.
      // Unrolled, so that each stage waits with its own constant and nothing is issued inside the loop.
#pragma unroll
      for (int s = 0; s < S - 1; ++s) {
        if ((unsigned)s >= nlocal) break;
        const int newest = S - 3 - s > 0 ? S - 3 - s : 0;
        if (s % 2 == 0) stage(nt_tag, std::false_type{}, newest, (unsigned)s, acc0, acc1, e0, e1);
        else stage(nt_tag, std::false_type{}, newest, (unsigned)s, acc1, acc0, e1, e0);
      }
    } else {
      for (unsigned s = 0; s < nlocal; s += 2) {
        stage(nt_tag, std::true_type{}, S - 3, s, acc0, acc1, e0, e1);
        if (s + 1 < nlocal) stage(nt_tag, std::true_type{}, S - 3, s + 1, acc1, acc0, e1, e0);
      }
    }
  };
  if (ntl == TPW) run(std::integral_constant<int, TPW>{});
  else run(std::integral_constant<int, TPW - 1>{});
  wait_vmcnt_n(0);      // the refills past the last unit are still landing in their slots
  // the last stage's sums are still pending; only a workgroup's last unit can reach past N, where
  // the rows are padding and must not compete (needs at least two workgroups, which the launcher
  // guarantees whenever there is more than one unit)
  if (nlocal > 0) {
    const unsigned sl = nlocal - 1;
    const unsigned unit0 = (first + sl * stride) * 16 + 4 * (lane / 16);
    const int tag = 255 - (int)sl;
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
      if constexpr (BEAM == 1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int v = (sl % 2 == 0) ? acc0[i][r] : acc1[i][r];
          if (unit0 + r < p.L) best[i][r] = max(best[i][r], (v << 8) | tag);
        }
      } else {
        if (i < ntl)
          beam_update(i, (sl % 2 == 0) ? acc0[i] : acc1[i], tag, unit0 + 0 < p.L, unit0 + 1 < p.L, unit0 + 2 < p.L,
                      unit0 + 3 < p.L);
      }
    }
  }

  if constexpr (BEAM > 1) {
    // Per sentence tile: decode the 4 x BEAM register keys into (sum, lowest index) keys, keep the BEAM best,
    // merge with the three other lane groups that hold candidates of the same sentence, and write the list
    // and the normaliser's (max, sum) pair.
    auto decode = [&](int k32) -> unsigned long long {
      const int sum = k32 >> 8;
      if (sum == -8388608) return 0ull;
      const unsigned st = 255u - (unsigned)(k32 & 255);
      const unsigned n = (first + st * stride) * 16 + 4 * (lane / 16);
      return ((unsigned long long)((unsigned)sum ^ 0x80000000u) << 32) | (unsigned long long)(0xFFFFFFFFu - n);
    };
    auto insert = [&](unsigned long long (&top)[BEAM], unsigned long long k) {
#pragma unroll
      for (int j = 0; j < BEAM; ++j) {
        const unsigned long long hi = top[j] > k ? top[j] : k;
        k = top[j] > k ? k : top[j];
        top[j] = hi;
      }
    };
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
      unsigned long long top[BEAM];
#pragma unroll
      for (int j = 0; j < BEAM; ++j) top[j] = 0ull;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        unsigned long long k = decode(best[i][r]);
        if (k != 0ull) k -= (unsigned)r;                       // candidate index 4 (l / 16) + r: larger index, smaller key
        insert(top, k);
#pragma unroll
        for (int j = 0; j < BEAM - 1; ++j) {
          unsigned long long k2 = decode(more_best[i][r][j]);
          if (k2 != 0ull) k2 -= (unsigned)r;
          insert(top, k2);
        }
      }
      float mx = run_max[i], sm = run_sum[i];
#pragma unroll
      for (int off = 16; off <= 32; off *= 2) {
        unsigned long long other[BEAM];
#pragma unroll
        for (int j = 0; j < BEAM; ++j) other[j] = __shfl_xor(top[j], off, 64);
#pragma unroll
        for (int j = 0; j < BEAM; ++j) insert(top, other[j]);
        const float omx = __shfl_xor(mx, off, 64), osm = __shfl_xor(sm, off, 64);
        const float m2 = fmaxf(mx, omx);
        if (m2 > -INFINITY) {
          sm = sm * __builtin_amdgcn_exp2f(mx - m2) + osm * __builtin_amdgcn_exp2f(omx - m2);
          mx = m2;
        }
      }
      const unsigned m = (wave + kWaves * i) * 16 + lane % 16;
      if (lane < 16 && m < p.M && i < ntl) {
        const size_t at = (size_t)m * gridDim.x + blockIdx.x;
#pragma unroll
        for (int j = 0; j < BEAM; ++j) p.partial[at * BEAM + j] = top[j];
        p.norm[at] = make_float2(mx, sm);
      }
    }
    return;
  }
  // decode the per-register winners, pick the best of the four (smaller word index on ties), merge the
  // four lane groups that share a sentence, and write one key per sentence
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    unsigned long long key = 0ull;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int sum = best[i][r] >> 8;
      if (sum != -8388608) {
        const unsigned s = 255u - (unsigned)(best[i][r] & 255);
        const unsigned n = (first + s * stride) * 16 + 4 * (lane / 16) + r;
        const unsigned long long k =
            ((unsigned long long)((unsigned)sum ^ 0x80000000u) << 32) | (unsigned long long)(0xFFFFFFFFu - n);
        if (k > key) key = k;
      }
    }
    unsigned long long o = __shfl_xor(key, 16, 64);
    if (o > key) key = o;
    o = __shfl_xor(key, 32, 64);
    if (o > key) key = o;
    const unsigned m = (wave + kWaves * i) * 16 + lane % 16;
    // this workgroup's keys are consecutive in memory: the 16 lanes of a sentence tile fill one 128-byte line
    if (lane < 16 && m < p.M) p.partial[(size_t)blockIdx.x * (((size_t)p.M + 15) / 16 * 16) + m] = key;
  }
}

// One workgroup per tile of 16 sentences: 16 groups of 16 lanes each take every 16th workgroup's keys of the tile (one
// 128-byte line per group and load), the groups' maxima meet in LDS, and 16 lanes decode.
__global__ __launch_bounds__(256) void k_argmax_reduce(const unsigned long long* __restrict__ partial, unsigned cols,
                                                       unsigned M, const float* __restrict__ sA,
                                                       const float* __restrict__ sW, int32_t* __restrict__ tok,
                                                       float* __restrict__ maxlogit,
                                                       const int32_t* __restrict__ shortlist) {
  __shared__ unsigned long long red[16][16];
  const unsigned mi = threadIdx.x % 16, gs = threadIdx.x / 16;
  const unsigned m = blockIdx.x * 16 + mi;
  const size_t Mpad = ((size_t)M + 15) / 16 * 16;
  unsigned long long key = 0ull;
  if (m < M) {
    const unsigned long long* col = partial + m;
    unsigned g = gs;
    for (; g + 48 < cols; g += 64) {              // four independent loads in flight per lane
      const unsigned long long k0 = col[(size_t)g * Mpad], k1 = col[(size_t)(g + 16) * Mpad];
      const unsigned long long k2 = col[(size_t)(g + 32) * Mpad], k3 = col[(size_t)(g + 48) * Mpad];
      const unsigned long long a = k0 > k1 ? k0 : k1, b = k2 > k3 ? k2 : k3, c = a > b ? a : b;
      if (c > key) key = c;
    }
    for (; g < cols; g += 16) {
      const unsigned long long k = col[(size_t)g * Mpad];
      if (k > key) key = k;
    }
  }
  red[gs][mi] = key;
  __syncthreads();
  if (gs == 0 && m < M) {
#pragma unroll
    for (int j = 1; j < 16; ++j)
      if (red[j][mi] > key) key = red[j][mi];
    const float u = __fdiv_rn(1.0f, __fmul_rn(*sA, *sW));
    const int best = (int)((unsigned)(key >> 32) ^ 0x80000000u);
    const unsigned pos = 0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull);
    tok[m] = shortlist != nullptr ? shortlist[pos] : (int32_t)pos;
    maxlogit[m] = __fmul_rn((float)best, u);
  }
}

// Beam search: one wave per row.  Merges the per-workgroup lists into the k best (sum, lowest index) keys
// and the per-workgroup (max, sum) pairs into log sum exp; writes tok [M x k] and logprob [M x k].
template <int BEAM>
__global__ __launch_bounds__(256) void k_topk_reduce(const unsigned long long* __restrict__ partial,
                                                     const float2* __restrict__ norm, unsigned cols, unsigned M,
                                                     unsigned k, const float* __restrict__ sA,
                                                     const float* __restrict__ sW, int32_t* __restrict__ tok,
                                                     float* __restrict__ logprob,
                                                     const int32_t* __restrict__ shortlist) {
  const int lane = threadIdx.x % 64;
  const unsigned m = blockIdx.x * 4 + threadIdx.x / 64;
  if (m >= M) return;
  unsigned long long top[BEAM];
#pragma unroll
  for (int j = 0; j < BEAM; ++j) top[j] = 0ull;
  float mx = -INFINITY, sm = 0.f;
  for (unsigned g = lane; g < cols; g += 64) {
    const size_t at = (size_t)m * cols + g;
#pragma unroll
    for (int j = 0; j < BEAM; ++j) {
      unsigned long long key = partial[at * BEAM + j];
#pragma unroll
      for (int q = 0; q < BEAM; ++q) {
        const unsigned long long hi = top[q] > key ? top[q] : key;
        key = top[q] > key ? key : top[q];
        top[q] = hi;
      }
    }
    const float2 nm = norm[at];
    const float m2 = fmaxf(mx, nm.x);
    if (m2 > -INFINITY) {
      sm = sm * __builtin_amdgcn_exp2f(mx - m2) + nm.y * __builtin_amdgcn_exp2f(nm.x - m2);
      mx = m2;
    }
  }
  // normaliser over the wave
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float omx = __shfl_xor(mx, off, 64), osm = __shfl_xor(sm, off, 64);
    const float m2 = fmaxf(mx, omx);
    if (m2 > -INFINITY) {
      sm = sm * __builtin_amdgcn_exp2f(mx - m2) + osm * __builtin_amdgcn_exp2f(omx - m2);
      mx = m2;
    }
  }
  const float u = __fdiv_rn(1.0f, __fmul_rn(*sA, *sW));
  const float lse = (mx + __builtin_amdgcn_logf(sm)) * 0.693147180559945309417f;     // log2 -> natural log
  // k rounds: the wave's best key wins, the lane that held it moves its list up
  for (unsigned j = 0; j < k; ++j) {
    unsigned long long w = top[0];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const unsigned long long o = __shfl_xor(w, off, 64);
      if (o > w) w = o;
    }
    if (top[0] == w && w != 0ull) {      // keys are unique (the index is part of the key)
#pragma unroll
      for (int q = 0; q + 1 < BEAM; ++q) top[q] = top[q + 1];
      top[BEAM - 1] = 0ull;
    }
    if (lane == 0) {
      const int sum = (int)((unsigned)(w >> 32) ^ 0x80000000u);
      const unsigned pos = 0xFFFFFFFFu - (unsigned)(w & 0xFFFFFFFFull);
      tok[(size_t)m * k + j] = shortlist != nullptr ? shortlist[pos] : (int32_t)pos;
      logprob[(size_t)m * k + j] = __fmul_rn((float)sum, u) - lse;
    }
  }
}

template <int TPW, bool GATHER, int BEAM = 1>
int launch_stream(const ArgmaxParams& p, unsigned grid, hipStream_t s, unsigned ny = 1) {
  constexpr size_t smem = (size_t)(kStages + 1) * kKG * kFragBytes + (GATHER ? 255 * 16 * sizeof(int32_t) : 0);
  auto kern = k_argmax_stream<TPW, GATHER, BEAM>;
  static bool attr_done = false;
  if (!attr_done) {
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    if (rc != MQ_OK) return rc;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(grid, ny), dim3(kWaves * 64), smem, s, p);
  return check_hip(hipGetLastError());
}

}  // namespace

// one pass's keys: a run of (rows of the pass, rounded up to 16) keys per workgroup
size_t argmax_stream_ws_bytes(size_t M) {
  const size_t rows = M < (size_t)kWaves * 3 * 16 ? M : (size_t)kWaves * 3 * 16;
  return (size_t)kMaxBlocks * round_up(rows, 16) * sizeof(unsigned long long);
}

// Limits: sums must fit 24 bits (127^2 K < 2^23); at most 255 stages per workgroup.  Any number of rows: 384 per pass.
bool argmax_stream_supported(size_t M, size_t N, size_t K) {
  (void)M;
  return K <= 64 * kKG && N <= (size_t)255 * 256 * 16;
}

int launch_argmax_stream(const void* packedA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                         const float* sW, int32_t* tok, float* maxlogit, void* ws, const int32_t* shortlist,
                         size_t shortlist_len, hipStream_t s, unsigned max_grid) {
  if (!argmax_stream_supported(M, N, K)) return MQ_ERR_UNSUPPORTED;
  const PackedDims dW(8, N, K), dAll(8, M, K);
  static int cus = 0;               // compute units of the device, asked once
  if (cus == 0) {
    int dev = 0, v = 0;
    cus = 256;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
  }
  const size_t units = shortlist != nullptr ? (shortlist_len + 15) / 16 : dW.nblocks * 2;
  unsigned grid = (unsigned)(units < (size_t)cus ? units : (size_t)cus);
  if (grid > (unsigned)kMaxBlocks) grid = kMaxBlocks;
  if (max_grid != 0 && grid > max_grid) grid = max_grid;       // the caller's partials array has that many columns
  if ((units + grid - 1) / grid > 255) return MQ_ERR_UNSUPPORTED;
  // rows beyond what one workgroup's registers hold (3 tiles of 16 sentences per wave) go in further passes
  constexpr size_t kChunk = (size_t)kWaves * 3 * 16;
  for (size_t row0 = 0; row0 < M; row0 += kChunk) {
    const size_t rows = M - row0 < kChunk ? M - row0 : kChunk;
    ArgmaxParams p{};
    p.packedA = static_cast<const uint8_t*>(packedA) + dAll.frag_offset(row0 / 32, 0);
    p.packedW = static_cast<const uint8_t*>(packedW);
    p.M = (unsigned)rows; p.N = (unsigned)N; p.K = (unsigned)K;
    p.partial = static_cast<unsigned long long*>(ws);
    p.shortlist = shortlist;
    p.L = shortlist != nullptr ? (unsigned)shortlist_len : (unsigned)N;
    p.norm = nullptr; p.sA = sA; p.sW = sW;
    const size_t tiles = (rows + 15) / 16;
    const int tpw = (int)((tiles + kWaves - 1) / kWaves);
    int rc;
    if (shortlist != nullptr) {
      switch (tpw) {
        case 1: rc = launch_stream<1, true>(p, grid, s); break;
        case 2: rc = launch_stream<2, true>(p, grid, s); break;
        default: rc = launch_stream<3, true>(p, grid, s); break;
      }
    } else {
      switch (tpw) {
        case 1: rc = launch_stream<1, false>(p, grid, s); break;
        case 2: rc = launch_stream<2, false>(p, grid, s); break;
        default: rc = launch_stream<3, false>(p, grid, s); break;
      }
    }
    if (rc != MQ_OK) return rc;
    hipLaunchKernelGGL(k_argmax_reduce, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, s, p.partial, grid,
                       (unsigned)rows, sA, sW, tok + row0, maxlogit + row0, shortlist);
    rc = check_hip(hipGetLastError());
    if (rc != MQ_OK) return rc;
  }
  return MQ_OK;
}

// ---- the same output layer for callers that cannot allocate: partial winners in a static device array ----
// One pass of kStaticRows sentences against at most kStaticCols workgroups' candidates: 768 KiB per device, held
// until the process ends.  Further passes (more rows) reuse it one after the other on the stream.
namespace {
constexpr size_t kStaticRows = (size_t)kWaves * 3 * 16;     // rows of one pass of the streaming kernel (384)
constexpr unsigned kStaticCols = 256;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned long long scratch[kStaticRows * kStaticCols];
std::mutex g_scratch_mutex;
unsigned long long* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, asked once
}  // namespace

size_t argmax_static_max_rows() { return kStaticRows * 64; }

int launch_argmax_stream_static(const void* packedA, const void* packedW, size_t M, size_t N, size_t K,
                                const float* sA, const float* sW, int32_t* tok, float* maxlogit, hipStream_t s) {
  int dev = -1;
  if (check_hip(hipGetDevice(&dev)) != MQ_OK) return MQ_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return MQ_ERR_UNSUPPORTED;
  unsigned long long* ptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
      // `scratch` itself is only a host-side handle: kernels get the address the runtime reports for this device
      void* addr = nullptr;
      const int rc = check_hip(hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)));
      if (rc != MQ_OK || addr == nullptr) return MQ_ERR_HIP;
      g_scratch_ptr[dev] = static_cast<unsigned long long*>(addr);
    }
    ptr = g_scratch_ptr[dev];
  }
  // every key the reduce kernel reads was written by this call's streaming kernel: nothing has to start at zero
  return launch_argmax_stream(packedA, packedW, M, N, K, sA, sW, tok, maxlogit, ptr, nullptr, 0, s, kStaticCols);
}

size_t topk_stream_ws_bytes(size_t M, int k) {
  // every row's candidates and normalisers from up to 256 workgroups (rows go 256 to a workgroup, all chunks in one launch)
  const int beam = k <= 2 ? 2 : 4;
  return round_up((size_t)256 * M * beam * sizeof(unsigned long long), 256) + (size_t)256 * M * sizeof(float2);
}

bool topk_stream_supported(size_t M, size_t N, size_t K, int k) {
  (void)M;
  return k >= 1 && k <= 4 && (size_t)k <= N && K <= 64 * kKG && N <= (size_t)255 * 256 * 16;
}

// Beam-search output layer: the k <= 4 best words of every row with log-probabilities.  Rows are processed in
// chunks of 256 (two sentence tiles per wave), each chunk streaming the embedding once, all chunks in one launch.
int launch_topk_stream(const void* packedA, const void* packedW, size_t M, size_t N, size_t K, const float* sA,
                       const float* sW, int k, int32_t* tok, float* logprob, void* ws, const int32_t* shortlist,
                       size_t shortlist_len, hipStream_t s) {
  if (!topk_stream_supported(M, N, K, k)) return MQ_ERR_UNSUPPORTED;
  if (shortlist != nullptr && (size_t)k > shortlist_len) return MQ_ERR_SHAPE;
  const PackedDims dW(8, N, K);
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    cus = 256;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
  }
  const size_t units = shortlist != nullptr ? (shortlist_len + 15) / 16 : dW.nblocks * 2;
  unsigned grid = (unsigned)(units < (size_t)cus ? units : (size_t)cus);
  if (grid > 256u) grid = 256u;
  if ((units + grid - 1) / grid > 255) return MQ_ERR_UNSUPPORTED;
  const int beam = k <= 2 ? 2 : 4;
  unsigned long long* keys = static_cast<unsigned long long*>(ws);
  float2* norm = reinterpret_cast<float2*>(static_cast<uint8_t*>(ws) +
                                           round_up((size_t)256 * M * beam * sizeof(unsigned long long), 256));
  // Rows go 256 to a workgroup (two sentence tiles per wave); all chunks run in ONE launch, the grid's y index picking
  // the chunk, and one reduce launch follows for all rows: a launch per chunk (ten for 1200 rows) cost more than the
  // chunks' work.
  constexpr unsigned kChunkRows = 256;
  const unsigned nchunks = (unsigned)((M + kChunkRows - 1) / kChunkRows);
  if (nchunks > 65535u) return MQ_ERR_UNSUPPORTED;
  ArgmaxParams p{};
  p.packedA = static_cast<const uint8_t*>(packedA);
  p.packedW = static_cast<const uint8_t*>(packedW);
  p.M = (unsigned)(M < kChunkRows ? M : kChunkRows); p.N = (unsigned)N; p.K = (unsigned)K;
  p.partial = keys; p.norm = norm; p.sA = sA; p.sW = sW;
  p.shortlist = shortlist;
  p.L = shortlist != nullptr ? (unsigned)shortlist_len : (unsigned)N;
  p.chunk_rows = nchunks > 1 ? kChunkRows : 0u;
  p.Mtotal = (unsigned)M;
  const int tpw = (int)(((size_t)(p.M + 15) / 16 + kWaves - 1) / kWaves);
  int rc;
  if (shortlist != nullptr) {
    if (beam == 2) rc = tpw == 1 ? launch_stream<1, true, 2>(p, grid, s, nchunks) : launch_stream<2, true, 2>(p, grid, s, nchunks);
    else rc = tpw == 1 ? launch_stream<1, true, 4>(p, grid, s, nchunks) : launch_stream<2, true, 4>(p, grid, s, nchunks);
  } else {
    if (beam == 2) rc = tpw == 1 ? launch_stream<1, false, 2>(p, grid, s, nchunks) : launch_stream<2, false, 2>(p, grid, s, nchunks);
    else rc = tpw == 1 ? launch_stream<1, false, 4>(p, grid, s, nchunks) : launch_stream<2, false, 4>(p, grid, s, nchunks);
  }
  if (rc != MQ_OK) return rc;
  if (beam == 2)
    hipLaunchKernelGGL((k_topk_reduce<2>), dim3((unsigned)((M + 3) / 4)), dim3(256), 0, s, keys, norm, grid, (unsigned)M,
                       (unsigned)k, sA, sW, tok, logprob, shortlist);
  else
    hipLaunchKernelGGL((k_topk_reduce<4>), dim3((unsigned)((M + 3) / 4)), dim3(256), 0, s, keys, norm, grid, (unsigned)M,
                       (unsigned)k, sA, sW, tok, logprob, shortlist);
  return check_hip(hipGetLastError());
}

}  // namespace mq
