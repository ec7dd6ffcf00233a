// Weight GEMMs of the fused rows (Algorithm 2's GEMM calls over [buffer + offset, size), Section V-C).
//
// y[m][n] = sum_k x[m][k] W[n][k], fp32 accumulation, M = live rows (small), W streamed once from HBM.
// The work is HBM-bound for M up to a few hundred (M flop per weight byte), so the design goal is to stream W
// at full bandwidth:
//   * W is re-tiled once at init into MFMA operand order: tile (n-tile of 16 columns, k-block of 32) is 1 KiB,
//     lane l holds W[n0 + l%16][k0 + 8*(l/16) .. +8], so every wave load is one contiguous, fully used 1 KiB;
//     tiles are ordered [column group of NT n-tiles][k-block][n-tile in group], so the K slice a wave streams is
//     one contiguous run of memory (NT KiB per k-block).
//   * a column group (NT n-tiles: 64 columns, or 32 for matrices of at most 4096 columns) x one K slice x all rows of
//     a row block is the unit of work; up to 16 rows one wave takes it and reads the rows' operand straight from L2/L1
//     (no LDS, no barriers); above that the rows' operand is staged through LDS once per block of 4 column groups and
//     shared by the block's 4 or 8 waves.
//   * more than 128 rows (context passes, very wide windows): the contraction turns MFMA-bound, so a wave keeps a
//     128 x 64 output tile and a block covers 256 rows x 256 columns; row blocks of one (column block, K slice) get
//     workgroup ids that land on the same XCD, so the weight tiles cross HBM once and are L2 hits for the others.
//   * split-K: for the fused iteration slice count and boundaries depend on (N, K) only -- never on M -- and partial
//     sums are written per slice and added by the consumer in slice order, so a row's result does not depend on which
//     other rows are live (the paper's premise that fused requests undergo identical operations).  A context pass
//     holds rows of one request and is sliced by that request's row count too (context_plan): few slices at hundreds
//     of rows, where the fp32 partial sums would outweigh the weights, more for short prompts.
//   * MFMA v_mfma_f32_16x16x32_{bf16,f16}: A = 16 columns of W, B = 16 rows of x, 32-deep: the accumulator tile is
//     y^T, so a lane holds 4 consecutive output columns of one row and stores them as one 16-byte write.
//   * gate|up of a gated MLP, up to 128 fused rows: no partial sums at all -- the two K halves are the two wave sets of
//     a block and the activation is the kernel's epilogue (gated_lds_kernel), with gate and up columns interleaved in
//     the layout so that a lane holds both; above 128 rows the same halves go through memory as two slices.
// fp32 models (tiny configurations only) use a plain FMA kernel on the untiled matrix.
#include <algorithm>
#include <type_traits>

#include "flover_dev.h"
#include "flover_kernels.h"

namespace flk {

// ---------------------------------------------------------------- re-tiling (init time)

__global__ void retile16_kernel(const uint16_t* __restrict__ W, u32x4_t* __restrict__ wt, int N, int K, int KB,
                                int ntile0, int tstep, int NT, long total) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int lane = (int)(i & 63);
  long t = i >> 6;
  int kb = (int)(t % KB);
  int ntile = (int)(t / KB);
  int n = ntile * 16 + (lane & 15);
  int k = kb * 32 + (lane >> 4) * 8;
  u32x4_t v = {0u, 0u, 0u, 0u};
  if (n < N) v = *(const u32x4_t*)(W + (size_t)n * K + k);
  const int tile = ntile0 + ntile * tstep, g = tile / NT, tt = tile - g * NT;
  wt[(((size_t)g * KB + kb) * NT + tt) * 64 + lane] = v;
}

// ---------------------------------------------------------------- 16-bit MFMA kernel

template <int DT> __device__ __forceinline__ f32x4_t mfma16(const u32x4_t& a, const u32x4_t& b, f32x4_t c) {
  if constexpr (DT == DT_BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// ---- direct variant: 4 independent waves per block, no LDS, no barriers; the rows' operand comes straight from L2/L1.
// grid = (ceil(ngroups/4), S, row blocks), block = 256; a wave owns NT n-tiles (16*NT columns) x one K slice x 16*MT rows.
// W is prefetched PFW k-blocks ahead, x PFA k-blocks ahead (PFW % PFA == 0).
template <int DT, int MT, int NT, int PFW, int PFA>
__global__ __launch_bounds__(256) void gemm16_direct_kernel(const uint16_t* __restrict__ x, const u32x4_t* __restrict__ wt,
                                                            float* __restrict__ part, int M, int N, int K, int ngroups,
                                                            int KB, int kbs, size_t slice_stride, int ldc,
                                                            int xmtt) {
  static_assert(PFW % PFA == 0, "ring shapes");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = blockIdx.x * 4 + wave;
  if (g >= ngroups) return;
  const int s = blockIdx.y;
  const int m0 = blockIdx.z * (16 * MT);
  const int kb0 = s * kbs;
  const int kb1 = min(KB, kb0 + kbs);

  f32x4_t acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[i][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const u32x4_t* wp = wt + ((size_t)g * KB) * NT * 64 + lane;                    // + (kb*NT + t)*64
  // rows' operand: row-major [M][K] (xmtt == 0) or fragment order with xmtt row tiles per k-block
  const size_t tstride = xmtt ? 512 : (size_t)16 * K, kstride = xmtt ? (size_t)xmtt * 512 : 32;
  const uint16_t* xp = xmtt ? x + (size_t)(m0 >> 4) * 512 + lane * 8
                            : x + (size_t)(m0 + (lane & 15)) * K + (lane >> 4) * 8;     // + i*tstride + kb*kstride

  u32x4_t bq[PFW][NT], aq[PFA][MT];
  static_assert(PFW == PFA, "both rings turn together");
#pragma unroll
  for (int j = 0; j < PFW; ++j) {      // same order as the refills in the loop: the wait counts of the first turn match
    const int kk = min(kb0 + j, kb1 - 1);
#pragma unroll
    for (int t = 0; t < NT; ++t) bq[j][t] = __builtin_nontemporal_load(wp + ((size_t)kk * NT + t) * 64);
#pragma unroll
    for (int i = 0; i < MT; ++i) aq[j][i] = *(const u32x4_t*)(xp + i * tstride + kk * kstride);
    __builtin_amdgcn_sched_barrier(0);
  }
  // One turn of the ring.  The steady-state turns (TAIL = false: all PFW k-blocks exist) are free of branches, so the
  // compiler's wait counts for the in-order memory counter stay exact; sched_barrier keeps each refill where it is
  // written, right after the k-block that freed the slot.
  auto turn = [&](auto tail_, int kb) {
    constexpr bool tail = decltype(tail_)::value;
#pragma unroll
    for (int j = 0; j < PFW; ++j) {
      if (!tail || kb + j < kb1) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int t = 0; t < NT; ++t) acc[i][t] = mfma16<DT>(bq[j][t], aq[j % PFA][i], acc[i][t]);
      }
      if (!tail) {
        const int kw = min(kb + j + PFW, kb1 - 1);    // the last turns re-read the last block (in bounds, unused)
#pragma unroll
        for (int t = 0; t < NT; ++t) bq[j][t] = __builtin_nontemporal_load(wp + ((size_t)kw * NT + t) * 64);
        const int ka = min(kb + j + PFA, kb1 - 1);
#pragma unroll
        for (int i = 0; i < MT; ++i) aq[j % PFA][i] = *(const u32x4_t*)(xp + i * tstride + ka * kstride);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  int kb = kb0;
  for (; kb + PFW <= kb1; kb += PFW) turn(std::false_type{}, kb);
  if (kb < kb1) turn(std::true_type{}, kb);
  float* out = part + (size_t)s * slice_stride;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int n = (g * NT + t) * 16 + (lane >> 4) * 4, m = m0 + i * 16 + (lane & 15);
      if (m < M && n < ldc) *(f32x4_t*)(out + (size_t)m * ldc + n) = acc[i][t];
    }
}

// ---- larger M (17..128 rows per block): the rows' operand is staged through LDS once per block and shared by its
// waves; a block covers GPB = 4 column groups (256 columns; 128 for matrices laid out in 32-column groups), each group
// by NT/NTW waves that own NTW of its n-tiles and stream their W tiles from HBM into registers, PF k-blocks ahead.
// From 33 rows up a wave owns 32 columns (8 waves per 256-column block): a single wave issues MFMAs at about 60% of
// the unit's rate, two waves per SIMD interleave and also hide each other's LDS and memory waits.
// LDS holds the x tile in MFMA fragment order ([k-block][m-tile][lane] x 16 B), so every ds_read_b128 of a fragment
// is 1 KiB contiguous and bank-conflict free.  Double-buffered chunks of KC k-blocks, one barrier per chunk.
// The per-(m, n) arithmetic (MFMA sequence over k) is identical to the direct kernel's.
template <int DT, int MT, int NT, int NTW, int KC, int PF, int GPB>
__global__ __launch_bounds__(64 * GPB * (NT / NTW)) void gemm16_lds_kernel(const uint16_t* __restrict__ x,
                                                                         const u32x4_t* __restrict__ wt,
                                                                         float* __restrict__ part, int M, int N, int K,
                                                                         int ngroups, int KB, int kbs,
                                                                         size_t slice_stride, int ldc, int nx,
                                                                         int nslices, int nz, int xmtt) {
  static_assert(PF % KC == 0 && NT % NTW == 0, "ring and tile shapes");
  constexpr int WPG = NT / NTW;                  // waves that share one column group, each taking NTW of its n-tiles
  constexpr int NW = GPB * WPG;                  // waves per block: GPB column groups (256 columns)
  __shared__ u32x4_t lds[2][KC * MT * 64];
  constexpr int FPW = (KC * MT + NW - 1) / NW;   // fragments each wave stages per chunk (surplus ones are skipped)
  constexpr int CPR = PF / KC;                   // chunks per turn of the W ring
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // 1-D grid, XCD-aware: workgroup ids go round-robin over the 8 XCDs (each with its own L2), so the row blocks of one
  // (column block, K slice) task are given ids 8 apart -- same XCD, dispatched back to back -- and the W tiles one of
  // them pulls from HBM are L2 hits for the others.  With a single row block this is the identity mapping.
  const int xcd = blockIdx.x & 7, qq = blockIdx.x >> 3;
  const int zb = qq % nz, task = (qq / nz) * 8 + xcd;
  if (task >= nx * nslices) return;              // padding of the grid (whole block)
  const int bx = task % nx, s = task / nx;
  const int g = bx * GPB + wave / WPG, sub = wave % WPG;
  const int gl = min(g, ngroups - 1);            // surplus waves repeat the last group (they still serve the barriers)
  const int m0 = zb * (16 * MT);
  const int kb0 = s * kbs;
  const int kb1 = min(KB, kb0 + kbs);
  const int nchunks = (kb1 - kb0 + KC - 1) / KC;

  f32x4_t acc[MT][NTW];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NTW; ++t) acc[i][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const u32x4_t* wp = wt + (((size_t)gl * KB) * NT + sub * NTW) * 64 + lane;     // + (kb*NT + t)*64
  // rows' operand: row-major [M][K] (xmtt == 0) or fragment order with xmtt row tiles per k-block
  const size_t tstride = xmtt ? 512 : (size_t)16 * K, kstride = xmtt ? (size_t)xmtt * 512 : 32;
  const uint16_t* xp = xmtt ? x + (size_t)(m0 >> 4) * 512 + lane * 8
                            : x + (size_t)(m0 + (lane & 15)) * K + (lane >> 4) * 8;     // + i*tstride + kb*kstride

  u32x4_t bq[PF][NTW], areg[FPW];
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    const int kk = min(kb0 + j, kb1 - 1);
#pragma unroll
    for (int t = 0; t < NTW; ++t) bq[j][t] = __builtin_nontemporal_load(wp + ((size_t)kk * NT + t) * 64);
  }
  auto load_a = [&](int chunk) {      // one fragment = 16 rows x 64 B per wave load
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
      const int f = min(wave + NW * j, KC * MT - 1), kc = f / MT, i = f - kc * MT;
      const int kk = min(kb0 + chunk * KC + kc, kb1 - 1);
      areg[j] = *(const u32x4_t*)(xp + i * tstride + kk * kstride);
    }
  };
  auto store_a = [&](int buf) {      // surplus waves store the last fragment once more (same data, no branch)
#pragma unroll
    for (int j = 0; j < FPW; ++j) lds[buf][min(wave + NW * j, KC * MT - 1) * 64 + lane] = areg[j];
  };
  load_a(0);
  store_a(0);
  __syncthreads();
  // One chunk: stage the next x tile, multiply this one, refill the W ring.  CC (position in the ring turn) is a
  // compile-time value; TAIL = the chunk may be the last one or short.  The steady-state loop below only runs
  // chunks that are full and have a successor, so its body is free of branches: the compiler's wait counts for the
  // in-order memory counter stay exact there (any branch in the body makes them collapse to "wait for all").
  auto chunk = [&](auto cc_, auto tail_, int c) {
    constexpr int cc = decltype(cc_)::value;
    constexpr bool tail = decltype(tail_)::value;
    const bool more = !tail || c + 1 < nchunks;
    if (more) load_a(c + 1);
    __builtin_amdgcn_sched_barrier(0);        // keep these loads ahead of the chunk's MFMAs (the scheduler sinks them to their use)
    const u32x4_t* la = lds[c & 1];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int kb = kb0 + c * KC + kc;
      if (!tail || kb < kb1) {
        u32x4_t af[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) af[i] = la[(kc * MT + i) * 64 + lane];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int t = 0; t < NTW; ++t) acc[i][t] = mfma16<DT>(bq[cc * KC + kc][t], af[i], acc[i][t]);
      }
      const int kk = min(kb + PF, kb1 - 1);
#pragma unroll
      for (int t = 0; t < NTW; ++t) bq[cc * KC + kc][t] = __builtin_nontemporal_load(wp + ((size_t)kk * NT + t) * 64);
      __builtin_amdgcn_sched_barrier(0);      // refill right after the k-block that freed the slot
    }
    if (more) store_a((c + 1) & 1);
    __syncthreads();
  };
  int c = 0;
  for (; c + CPR < nchunks; c += CPR) {
    if constexpr (CPR >= 1) chunk(std::integral_constant<int, 0>{}, std::false_type{}, c);
    if constexpr (CPR >= 2) chunk(std::integral_constant<int, 1>{}, std::false_type{}, c + 1);
    if constexpr (CPR >= 3) chunk(std::integral_constant<int, 2>{}, std::false_type{}, c + 2);
    if constexpr (CPR >= 4) chunk(std::integral_constant<int, 3>{}, std::false_type{}, c + 3);
  }
  for (; c < nchunks; c += CPR) {               // the last turn of the ring
    if constexpr (CPR >= 1) if (c < nchunks) chunk(std::integral_constant<int, 0>{}, std::true_type{}, c);
    if constexpr (CPR >= 2) if (c + 1 < nchunks) chunk(std::integral_constant<int, 1>{}, std::true_type{}, c + 1);
    if constexpr (CPR >= 3) if (c + 2 < nchunks) chunk(std::integral_constant<int, 2>{}, std::true_type{}, c + 2);
    if constexpr (CPR >= 4) if (c + 3 < nchunks) chunk(std::integral_constant<int, 3>{}, std::true_type{}, c + 3);
  }
  if (g >= ngroups) return;
  float* out = part + (size_t)s * slice_stride;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
      const int n = (g * NT + sub * NTW + t) * 16 + (lane >> 4) * 4, m = m0 + i * 16 + (lane & 15);
      if (m < M && n < ldc) *(f32x4_t*)(out + (size_t)m * ldc + n) = acc[i][t];
    }
}

// ---- gated MLP input (fused iterations of 16-bit gated models): the gate|up contraction with the activation as its
// epilogue, so that neither partial sums nor the two projections reach memory and the activation needs no launch.
// The matrix is laid out in "paired" groups of 32 columns -- group j = [gate columns 16j..16j+15 | up columns
// 16j..16j+15] -- so a lane's accumulators of a group's two n-tiles are gate and up of the same four MLP columns.
// K is split in two halves inside the block: 2 * GPB waves = GPB column groups x 2 halves, each wave the MFMA chain over its
// half's k-blocks in order, each half with its own x tile in LDS (fragment order, double-buffered chunks of KC
// k-blocks, W ring PF k-blocks deep); at the end the second half hands its sums to the first through LDS, which adds
// first half + second half, applies silu(gate) * up and writes the result, rounded to the model dtype, as the next
// GEMM's row operand (row-major or fragment order).  The result of a row is the same for every MT and equal, bit for
// bit, to gemm() with the halves as two K slices followed by the stand-alone activation.
// Every chunk is full and the last ring turn is the only one whose chunks may lack a successor, so the steady state
// is free of branches.  Requires KB % 16 == 0.
template <int DT, int MT, int KC, int PF, int GPB = 4>
__global__ __launch_bounds__(128 * GPB) void gated_lds_kernel(const uint16_t* __restrict__ x, const u32x4_t* __restrict__ wt,
                                                        void* __restrict__ act, int M, int F, int ngroups, int KB,
                                                        int xmtt) {
  static_assert(PF % KC == 0 && KC >= 2, "ring shape; the hand-over below reuses the x tiles' LDS");
  // GPB column groups per block (32 columns each) = waves that stage one half's x tile
  __shared__ u32x4_t lds[2][2][KC * MT * 64];    // [half][buffer]
  constexpr int FPW = (KC * MT + GPB - 1) / GPB;
  constexpr int CPR = PF / KC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = wave / GPB, gw = wave % GPB;
  const int g = blockIdx.x * GPB + gw;
  const int gl = min(g, ngroups - 1);            // surplus waves repeat the last group (they still serve the barriers)
  const int K = KB * 32;
  const int kb0 = half * (KB >> 1), kb1 = kb0 + (KB >> 1);
  const int nchunks = (kb1 - kb0) / KC;

  f32x4_t acc[MT][2];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < 2; ++t) acc[i][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const u32x4_t* wp = wt + ((size_t)gl * KB) * 2 * 64 + lane;                    // + (kb*2 + t)*64
  const size_t tstride = xmtt ? 512 : (size_t)16 * K, kstride = xmtt ? (size_t)xmtt * 512 : 32;
  const uint16_t* xp = xmtt ? x + lane * 8 : x + (size_t)(lane & 15) * K + (lane >> 4) * 8;   // + i*tstride + kb*kstride

  u32x4_t bq[PF][2], areg[FPW];
#pragma unroll
  for (int j = 0; j < PF; ++j)
#pragma unroll
    for (int t = 0; t < 2; ++t) bq[j][t] = __builtin_nontemporal_load(wp + ((size_t)(kb0 + j) * 2 + t) * 64);
  auto load_a = [&](int chunk) {
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
      const int f = min(gw + GPB * j, KC * MT - 1), kc = f / MT, i = f - kc * MT;
      areg[j] = *(const u32x4_t*)(xp + i * tstride + (kb0 + chunk * KC + kc) * kstride);
    }
  };
  auto store_a = [&](int buf) {      // surplus fragments store the last one once more (same data, no branch)
#pragma unroll
    for (int j = 0; j < FPW; ++j) lds[half][buf][min(gw + GPB * j, KC * MT - 1) * 64 + lane] = areg[j];
  };
  load_a(0);
  store_a(0);
  __syncthreads();
  // One chunk: stage the next x tile, multiply this one, refill the W ring.
  auto chunk = [&](auto cc_, auto last_, int c) {
    constexpr int cc = decltype(cc_)::value;
    constexpr bool last = decltype(last_)::value;
    const bool more = !last || c + 1 < nchunks;
    if (more) load_a(c + 1);
    __builtin_amdgcn_sched_barrier(0);
    const u32x4_t* la = lds[half][c & 1];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int kb = kb0 + c * KC + kc;
      u32x4_t af[MT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[i] = la[(kc * MT + i) * 64 + lane];
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[i][t] = mfma16<DT>(bq[cc * KC + kc][t], af[i], acc[i][t]);
      const int kk = min(kb + PF, kb1 - 1);      // the last turn re-reads the last block (in bounds, unused)
#pragma unroll
      for (int t = 0; t < 2; ++t) bq[cc * KC + kc][t] = __builtin_nontemporal_load(wp + ((size_t)kk * 2 + t) * 64);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) store_a((c + 1) & 1);
    __syncthreads();
  };
  auto ring_turn = [&](auto last_, int c) {
    static_assert(CPR <= 4, "chunks per ring turn");
    if constexpr (CPR >= 1) chunk(std::integral_constant<int, 0>{}, last_, c);
    if constexpr (CPR >= 2) chunk(std::integral_constant<int, 1>{}, last_, c + 1);
    if constexpr (CPR >= 3) chunk(std::integral_constant<int, 2>{}, last_, c + 2);
    if constexpr (CPR >= 4) chunk(std::integral_constant<int, 3>{}, last_, c + 3);
  };
  int c = 0;
  for (; c + CPR < nchunks; c += CPR) ring_turn(std::false_type{}, c);
  ring_turn(std::true_type{}, c);
  // second half -> first half through LDS (the x tiles are no longer read: every wave is past the last barrier)
  f32x4_t* red = (f32x4_t*)&lds[0][0][0];
  static_assert(sizeof(lds) >= (size_t)GPB * MT * 2 * 64 * sizeof(f32x4_t), "hand-over space");
  if (half == 1) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int t = 0; t < 2; ++t) red[((gw * MT + i) * 2 + t) * 64 + lane] = acc[i][t];
  }
  __syncthreads();
  if (half == 1 || g >= ngroups) return;
  const int j = g * 16 + (lane >> 4) * 4;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const f32x4_t gate = acc[i][0] + red[((gw * MT + i) * 2 + 0) * 64 + lane];
    const f32x4_t up = acc[i][1] + red[((gw * MT + i) * 2 + 1) * 64 + lane];
    const int m = i * 16 + (lane & 15);
    if (m < M) stv4<DT>(act, xrow_index(m, j, F, xmtt), act_swiglu(gate, up));
  }
}

// ---- context passes (hundreds of rows): the contraction is MFMA-bound there, so each wave keeps a 128 x 64 output
// tile (MTW = 8 row tiles x NT = 4 n-tiles, 128 accumulator registers): per k-block 32 MFMAs for 8 KiB of LDS reads and
// 4 KiB of W loads, which halves the operand traffic per flop of the 128-row kernel above (whose waves own 128 x 32).
// A block is 4 column units x 2 row halves = 8 waves over 256 rows x 256 columns; a unit is 64 columns = one group of
// the matrix layout or (NTL = 2) two consecutive ones; x tile and W ring as above.
// The per-(m, n) arithmetic is again the same MFMA sequence over k.
// GATED (a paired gate|up matrix taken in one slice): instead of partial sums the wave writes silu(gate) * up of its
// two column groups, rounded to the model dtype, as the next GEMM's row operand (`part` is then that buffer, N = 2F).
template <int DT, int MTW, int NT, int NTL, int KC, int PF, bool GATED = false>
__global__ __launch_bounds__(512) void gemm16_rows_kernel(const uint16_t* __restrict__ x, const u32x4_t* __restrict__ wt,
                                                          float* __restrict__ part, int M, int N, int K, int ngroups,
                                                          int KB, int kbs, size_t slice_stride, int ldc, int nx,
                                                          int nslices, int nz, int xmtt) {
  static_assert(!GATED || NTL == 2, "gate and up tiles alternate in groups of two");
  static_assert(PF % KC == 0 && NT % NTL == 0, "ring and tile shapes");
  constexpr int MTB = 2 * MTW;                   // row tiles per block
  constexpr int NW = 8;
  __shared__ u32x4_t lds[2][KC * MTB * 64];
  constexpr int FPW = (KC * MTB + NW - 1) / NW;
  constexpr int CPR = PF / KC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int xcd = blockIdx.x & 7, qq = blockIdx.x >> 3;     // row blocks of one task share an XCD (see above)
  const int zb = qq % nz, task = (qq / nz) * 8 + xcd;
  if (task >= nx * nslices) return;
  const int bx = task % nx, s = task / nx;
  const int g = bx * 4 + (wave >> 1), half = wave & 1;
  const int gl = min(g, ngroups - 1);
  const int m0 = zb * (16 * MTB);
  const int kb0 = s * kbs;
  const int kb1 = min(KB, kb0 + kbs);
  const int nchunks = (kb1 - kb0 + KC - 1) / KC;
  const int live_tiles = min(MTW, max(0, (M - m0 - half * (16 * MTW) + 15) / 16));   // of this wave's MTW row tiles

  f32x4_t acc[MTW][NT];
#pragma unroll
  for (int i = 0; i < MTW; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[i][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // the wave's NT n-tiles are NT / NTL consecutive column groups of the matrix layout (NTL tiles per group)
  const u32x4_t* wp = wt + ((size_t)gl * (NT / NTL) * KB) * NTL * 64 + lane;     // + woff(kb, t)
  auto woff = [&](int kb, int t) { return (((size_t)(t / NTL) * KB + kb) * NTL + (t % NTL)) * 64; };
  // rows' operand: row-major [M][K] (xmtt == 0) or fragment order with xmtt row tiles per k-block
  const size_t tstride = xmtt ? 512 : (size_t)16 * K, kstride = xmtt ? (size_t)xmtt * 512 : 32;
  const uint16_t* xp = xmtt ? x + (size_t)(m0 >> 4) * 512 + lane * 8
                            : x + (size_t)(m0 + (lane & 15)) * K + (lane >> 4) * 8;     // + i*tstride + kb*kstride

  u32x4_t bq[PF][NT], areg[FPW];
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    const int kk = min(kb0 + j, kb1 - 1);
#pragma unroll
    for (int t = 0; t < NT; ++t) bq[j][t] = wp[woff(kk, t)];
  }
  auto load_a = [&](int chunk) {
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
      const int f = min(wave + NW * j, KC * MTB - 1), kc = f / MTB, i = f - kc * MTB;
      const int kk = min(kb0 + chunk * KC + kc, kb1 - 1);
      areg[j] = *(const u32x4_t*)(xp + i * tstride + kk * kstride);
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int j = 0; j < FPW; ++j) lds[buf][min(wave + NW * j, KC * MTB - 1) * 64 + lane] = areg[j];
  };
  load_a(0);
  store_a(0);
  __syncthreads();
  // Chunks as in the kernel above: branch-free steady state, refills pinned where they are written.
  auto chunk = [&](auto cc_, auto tail_, auto full_, int c) {
    constexpr int cc = decltype(cc_)::value;
    constexpr bool tail = decltype(tail_)::value;
    constexpr bool full = decltype(full_)::value;
    const bool more = !tail || c + 1 < nchunks;
    if (more) load_a(c + 1);
    __builtin_amdgcn_sched_barrier(0);
    const u32x4_t* la = lds[c & 1];
    if constexpr (full && !tail) {
      // Every row tile live and every k-block of the chunk inside the slice (all but a ragged last row block and a
      // slice's last chunk): no branches, and a row tile's fragment is read from LDS two tiles ahead of its MFMAs.
      const u32x4_t* lw = la + (half * MTW) * 64 + lane;
      constexpr int T = KC * MTW;
      auto frag = [&](int q) { return lw[((q / MTW) * MTB + (q % MTW)) * 64]; };
      u32x4_t af[3];
      af[0] = frag(0);
      af[1] = frag(1);
#pragma unroll
      for (int q = 0; q < T; ++q) {
        const int kc = q / MTW, i = q % MTW;
        if (q + 2 < T) af[(q + 2) % 3] = frag(q + 2);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[i][t] = mfma16<DT>(bq[cc * KC + kc][t], af[q % 3], acc[i][t]);
        if (i == MTW - 1) {
          const int kk = min(kb0 + c * KC + kc + PF, kb1 - 1);
#pragma unroll
          for (int t = 0; t < NT; ++t) bq[cc * KC + kc][t] = wp[woff(kk, t)];
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    } else
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int kb = kb0 + c * KC + kc;
      if (!tail || kb < kb1) {
#pragma unroll
        for (int i = 0; i < MTW; ++i)
          if (i < live_tiles) {               // wave-uniform: row tiles past M are skipped
            const u32x4_t af = la[(kc * MTB + half * MTW + i) * 64 + lane];
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[i][t] = mfma16<DT>(bq[cc * KC + kc][t], af, acc[i][t]);
          }
      }
      const int kk = min(kb + PF, kb1 - 1);
#pragma unroll
      for (int t = 0; t < NT; ++t) bq[cc * KC + kc][t] = wp[woff(kk, t)];
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) store_a((c + 1) & 1);
    __syncthreads();
  };
  static_assert(CPR <= 2, "ring turns of one or two chunks");
  // Two copies of the loop, chosen per wave (the accumulators stay in place in each; both pass the same barriers).
  auto loops = [&](auto full_) {
    int c = 0;
    for (; c + CPR < nchunks; c += CPR) {
      chunk(std::integral_constant<int, 0>{}, std::false_type{}, full_, c);
      if constexpr (CPR >= 2) chunk(std::integral_constant<int, 1>{}, std::false_type{}, full_, c + 1);
    }
    for (; c < nchunks; c += CPR) {
      chunk(std::integral_constant<int, 0>{}, std::true_type{}, full_, c);
      if constexpr (CPR >= 2) if (c + 1 < nchunks) chunk(std::integral_constant<int, 1>{}, std::true_type{}, full_, c + 1);
    }
  };
  if (live_tiles == MTW) loops(std::true_type{});
  else loops(std::false_type{});
  if (g >= ngroups) return;
  if constexpr (GATED) {
    const int F = N >> 1;
#pragma unroll
    for (int i = 0; i < MTW; ++i)
#pragma unroll
      for (int pr = 0; pr < NT / 2; ++pr) {
        const int j = (g * (NT / 2) + pr) * 16 + (lane >> 4) * 4, m = m0 + (half * MTW + i) * 16 + (lane & 15);
        if (m < M && j < F) stv4<DT>(part, xrow_index(m, j, F, xmtt), act_swiglu(acc[i][2 * pr], acc[i][2 * pr + 1]));
      }
    return;
  }
  float* out = part + (size_t)s * slice_stride;
#pragma unroll
  for (int i = 0; i < MTW; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int n = (g * NT + t) * 16 + (lane >> 4) * 4, m = m0 + (half * MTW + i) * 16 + (lane & 15);
      if (m < M && n < ldc) *(f32x4_t*)(out + (size_t)m * ldc + n) = acc[i][t];
    }
}

// ---------------------------------------------------------------- fp32 FMA kernel (tiny models)

// one wave per output column, 8 rows at a time; lanes stride K, fixed butterfly reduction.
__global__ __launch_bounds__(256) void gemm32_kernel(const float* __restrict__ x, const float* __restrict__ W,
                                                     float* __restrict__ out, int M, int N, int K, int ldc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave;
  if (n >= N) return;
  const int m0 = blockIdx.y * 8;
  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;
  const float* wr = W + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float w = wr[k];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int m = min(m0 + r, M - 1);
      acc[r] = fmaf(x[(size_t)m * K + k], w, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const float v = group_sum<64>(acc[r]);
    if (lane == 0 && m0 + r < M) out[(size_t)(m0 + r) * ldc + n] = v;
  }
}

// ---------------------------------------------------------------- host side

GemmPlan gemm_plan(int dtype, int N, int K) {
  GemmPlan p{};
  p.N = N;
  p.K = K;
  p.ldc = part_ld(N);
  if (dtype == DT_F32) {
    p.Npad = N;
    p.NT = 0;
    p.KB = 0;
    p.S = 1;
    p.kbs = 0;
    return p;
  }
  p.Npad = (N + 63) / 64 * 64;
  p.KB = K / 32;
  // Everything below is a function of (N, K) only, never of the number of live rows.  A wave owns 64 columns -- 32 for
  // matrices of at most 4096 columns, which would otherwise need 13 K slices to fill the chip -- and K is split just
  // enough for about 800 waves (3 per CU, each streaming a contiguous run of W with a deep prefetch ring): more slices
  // only add partial-sum traffic, for this kernel's stores and for the row-wise kernel that adds the slices up
  // (measured on the 7B stream: 32-column waves for out-proj and FFN-down + 2 % tokens/s, for the wider matrices - 2 %).
  p.NT = p.Npad / 64 <= 64 ? 2 : 4;
  const int ngroups = p.Npad / (16 * p.NT);
  const int target = 800;
  int S = (target + ngroups / 2) / ngroups;
  int maxS = std::min(16, p.KB / 8);
  if (maxS < 1) maxS = 1;
  if (S > maxS) S = maxS;
  if (S < 1) S = 1;
  p.kbs = (p.KB + S - 1) / S;
  p.S = (p.KB + p.kbs - 1) / p.kbs;
  return p;
}

// gate|up of a gated MLP (N = 2F): paired 32-column groups, no K slices (the fused kernels split K in two inside),
// when the shape allows it; otherwise the plain plan of a 2F-column matrix with gate and up side by side.
GemmPlan gemm_plan_gated(int dtype, int F, int K) {
  GemmPlan p = gemm_plan(dtype, 2 * F, K);
  if (dtype == DT_F32 || F % 32 != 0 || (K / 32) % 16 != 0) return p;
  p.NT = 2;
  p.S = 2;               // the two halves of K: partial sums of gemm(), the two in-kernel chains of the fused kernels
  p.kbs = p.KB / 2;
  p.paired = 1;
  return p;
}

size_t gemm_tiled_bytes(int dtype, int N, int K) {
  if (dtype == DT_F32) return (size_t)N * K * 4;
  const size_t Npad = (size_t)(N + 63) / 64 * 64;
  return Npad * K * 2;
}

// Context passes: the slice count that minimises a simple cost model of the 256 x 256 blocks on 256 compute units:
// rounds of blocks x k-blocks per slice (about 1 us per k-block step of a block, measured), plus the fp32 partial sums
// written by this kernel and re-read by the next one (about 2 TB/s in effect: the stores are a burst at the kernel's
// end that nothing overlaps; the divisor is the one that minimises the context passes' time on a stream of prompts of
// 32 to 1024 rows, flat between 1.7 and 2.5) -- at hundreds of rows those outweigh the weights
// when the iteration's slicing is kept, while a single slice leaves most of the chip idle for the 4096-column matrices.
GemmPlan context_plan(const GemmPlan& p, int dtype, int M, int max_slices) {
  GemmPlan q = p;
  if (dtype == DT_F32 || M <= 128) return q;
  const long units = (long)((p.Npad / 64 + 3) / 4) * ((M + 255) / 256);
  const int smax = std::max(1, std::min(max_slices, 16));   // what the caller's partial-sum buffer holds; the row-wise
                                                             // kernels load up to 16 slices at once
  double best = 0.0;
  int bestS = 1;
  for (int S = 1; S <= smax; ++S) {
    const int kbs = (p.KB + S - 1) / S;
    if ((p.KB + kbs - 1) / kbs != S) continue;                       // slice counts that leave an empty last slice
    const double rounds = (double)((units * S + 255) / 256);
    // a paired gate|up matrix in one slice writes the activation instead of partial sums (gemm_gated)
    const double sums = (p.paired && S == 1) ? (double)M * p.N / 2.0e6 : (double)S * M * p.N * 8.0 / 2.0e6;
    const double cost = rounds * kbs * 1.0 + sums;   // microseconds
    if (S == 1 || cost < best) {
      best = cost;
      bestS = S;
    }
  }
  q.S = bestS;
  q.kbs = (p.KB + q.S - 1) / q.S;
  return q;
}

hipError_t retile(int dtype, const void* W, int N, int K, void* tiled, int n_off, int NT, hipStream_t st, int tile_step) {
  if (dtype == DT_F32) {
    if (tile_step != 1) return hipErrorInvalidValue;
    return hipMemcpyAsync((char*)tiled + (size_t)n_off * K * 4, W, (size_t)N * K * 4, hipMemcpyDeviceToDevice, st);
  }
  const int KB = K / 32;
  const int ntiles = (N + 15) / 16;
  const long total = (long)ntiles * KB * 64;
  retile16_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>((const uint16_t*)W, (u32x4_t*)tiled, N, K, KB,
                                                                         n_off / 16, tile_step, NT, total);
  return hipGetLastError();
}

hipError_t zero_fill(void* p, size_t bytes, hipStream_t st) { return hipMemsetAsync(p, 0, bytes, st); }

template <int DT, int MT, int NT, int PFW, int PFA>
static void launch_direct(const void* x, const void* wt, float* part, int M, const GemmPlan& p, size_t ss, int xmtt,
                          hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const int ngroups = p.Npad / (16 * NT);
  dim3 grid((ngroups + 3) / 4, p.S, (M + 16 * MT - 1) / (16 * MT));
  launch_timed(gemm16_direct_kernel<DT, MT, NT, PFW, PFA>, grid, dim3(256), st, ev0, ev1, (const uint16_t*)x,
               (const u32x4_t*)wt, part, M, p.N, p.K, ngroups, p.KB, p.kbs, ss, p.ldc, xmtt);
}
template <int DT, int MT, int NT, int NTW, int PF, int GPB = 4, int KC = 2>
static void launch_lds(const void* x, const void* wt, float* part, int M, const GemmPlan& p, size_t ss, int xmtt,
                       hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
                                                // GPB column groups per block: 256 columns, or 128 for the 32-column groups
                                                // (8 groups per block measured 3 % slower on the 7B stream)
  const int ngroups = p.Npad / (16 * NT);
  const int nx = (ngroups + GPB - 1) / GPB, nz = (M + 16 * MT - 1) / (16 * MT);
  const int tasks8 = (nx * p.S + 7) / 8 * 8;
  launch_timed(gemm16_lds_kernel<DT, MT, NT, NTW, KC, PF, GPB>, dim3(tasks8 * nz), dim3(64 * GPB * (NT / NTW)), st, ev0, ev1,
               (const uint16_t*)x, (const u32x4_t*)wt, part, M, p.N, p.K, ngroups, p.KB, p.kbs, ss, p.ldc, nx, p.S, nz, xmtt);
}

template <int DT, int NTL, bool GATED = false>
static void launch_rows(const void* x, const void* wt, float* part, int M, const GemmPlan& p, size_t ss, int xmtt,
                        hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const int ngroups = p.Npad / 64;            // units of 64 columns, whatever the layout's group width
  const int nx = (ngroups + 3) / 4, nz = (M + 255) / 256;
  const int tasks8 = (nx * p.S + 7) / 8 * 8;
  launch_timed(gemm16_rows_kernel<DT, 8, 4, NTL, 2, 2, GATED>, dim3(tasks8 * nz), dim3(512), st, ev0, ev1, (const uint16_t*)x,
               (const u32x4_t*)wt, part, M, p.N, p.K, ngroups, p.KB, p.kbs, ss, p.ldc, nx, p.S, nz, xmtt);
}

template <int DT, int NT>
static void dispatch16(const void* x, const void* wt, float* part, int M, const GemmPlan& p, size_t ss, int xmtt,
                       hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (M <= 16) launch_direct<DT, 1, NT, 8, 8>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);
  else if (M <= 32) launch_lds<DT, 2, NT, NT, 4, 4, (NT == 2 ? 4 : 2)>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);     // 4 waves, one per column group
  else if (NT == 2 && !p.paired && M <= 128) {
    // 32-column groups above 32 rows: two waves per group, one n-tile each (8 waves per 128-column block); measured
    // 0.6 us (33-64 rows) and 1.5 us (65-128 rows) faster per launch than one wave per group.  For these groups chunks
    // of 4 k-blocks (half the barriers) are 0.2-1.5 us faster per launch at every row count; for the 64-column ones not.
    // one variant per count of 16-row tiles: a block stages and multiplies exactly the live tiles
    switch ((M + 15) / 16) {
      case 3: launch_lds<DT, 3, NT, 1, 4, 4, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 4: launch_lds<DT, 4, NT, 1, 4, 4, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 5: launch_lds<DT, 5, NT, 1, 4, 4, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 6: launch_lds<DT, 6, NT, 1, 4, 4, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 7: launch_lds<DT, 7, NT, 1, 4, 4, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      default: launch_lds<DT, 8, NT, 1, 4, 4, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);
    }
  }
  else if (M <= 128 && !(NT == 2 && p.paired)) {
    switch ((M + 15) / 16) {                                                                  // 8 waves, two per column group
      case 3: launch_lds<DT, 3, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 4: launch_lds<DT, 4, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 5: launch_lds<DT, 5, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 6: launch_lds<DT, 6, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      case 7: launch_lds<DT, 7, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1); break;
      default: launch_lds<DT, 8, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);
    }
  }
  else if (M <= 64) launch_lds<DT, 4, NT, 2, 4>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);
  else if (M <= 128) launch_lds<DT, 8, NT, 2, 4, 8>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);   // paired: 8 groups, 256 columns
  else launch_rows<DT, NT>(x, wt, part, M, p, ss, xmtt, st, ev0, ev1);             // row blocks of 256
}

template <int DT>
static void dispatch_gated(const void* x, const void* wt, void* act, int M, const GemmPlan& p, int xmtt, hipStream_t st,
                           hipEvent_t ev0, hipEvent_t ev1) {
  const int F = p.N / 2, ngroups = F / 16, nx = (ngroups + 3) / 4;
  const uint16_t* xx = (const uint16_t*)x;
  const u32x4_t* ww = (const u32x4_t*)wt;
  // chunks of 4 k-blocks at one row tile (half the barriers), of 2 above.  A matrix whose 128-column blocks outnumber
  // the compute units (F > 16384; measured at the 30B shape, 280 blocks: 97 / 101 / 109 us at <= 16 / 17-32 / 33-64 rows
  // against 86 / 87 / 101 for the wider blocks) takes 256-column blocks of 16 waves, half as many; at the 7B shape (172
  // against 86 blocks) the 128-column blocks are 1.5x faster.
  if (nx > 256) {
    const dim3 g8((ngroups + 7) / 8), b16(1024);
    if (M <= 16) launch_timed(gated_lds_kernel<DT, 1, 4, 8, 8>, g8, b16, st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt);
    else if (M <= 32) launch_timed(gated_lds_kernel<DT, 2, 4, 8, 8>, g8, b16, st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt);
    else launch_timed(gated_lds_kernel<DT, 4, 4, 4, 8>, g8, b16, st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt);   // M <= 64
  }
  else if (M <= 16) launch_timed(gated_lds_kernel<DT, 1, 4, 8>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt);
  else if (M <= 32) launch_timed(gated_lds_kernel<DT, 2, 2, 8>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt);
  else switch ((M + 15) / 16) {     // M <= 128: one variant per count of 16-row tiles
    case 3: launch_timed(gated_lds_kernel<DT, 3, 2, 8>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt); break;
    case 4: launch_timed(gated_lds_kernel<DT, 4, 2, 8>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt); break;
    case 5: launch_timed(gated_lds_kernel<DT, 5, 2, 4>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt); break;
    case 6: launch_timed(gated_lds_kernel<DT, 6, 2, 4>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt); break;
    case 7: launch_timed(gated_lds_kernel<DT, 7, 2, 4>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt); break;
    default: launch_timed(gated_lds_kernel<DT, 8, 2, 4>, dim3(nx), dim3(512), st, ev0, ev1, xx, ww, act, M, F, ngroups, p.KB, xmtt);
  }
}

// The iteration's plan (two K halves): up to gated_fused_rows(p) rows one launch; above that gemm() with the two K
// halves as partial sums and the activation as its own launch -- the same two chains, added in the same order, rounded
// once: bit-identical results.  (At 65-128 rows the x tile of a 128-column block weighs as much as its weights; the one
// launch still measures 1.3 % faster per step there than the two: no partial sums, no second launch.)  A context
// pass's plan: one slice -> the 256-row-block kernel with the activation as its epilogue; any other slice count ->
// gemm() and the activation launch.
hipError_t gemm_gated(int dtype, const void* x, const void* wt, int M, const GemmPlan& p, void* act, float* part,
                      size_t slice_stride, int xmtt, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (M <= 0) return hipSuccess;
  if (!p.paired || dtype == DT_F32) return hipErrorInvalidValue;
  if (p.S == 1 && M > 128) {
    if (dtype == DT_BF16) launch_rows<DT_BF16, 2, true>(x, wt, (float*)act, M, p, 0, xmtt, st, ev0, ev1);
    else launch_rows<DT_F16, 2, true>(x, wt, (float*)act, M, p, 0, xmtt, st, ev0, ev1);
    return hipGetLastError();
  }
  if (M > gated_fused_rows(p) || p.S != 2) {
    hipError_t e = gemm(dtype, x, wt, M, p, part, slice_stride, xmtt, st, ev0, nullptr);   // timed from the first launch's
    if (e != hipSuccess) return e;                                                       // start to the second's end
    return activation(dtype, true, part, p.S, slice_stride, p.ldc, nullptr, act, M, p.N / 2, xmtt, st, true, ev1);
  }
  if (dtype == DT_BF16) dispatch_gated<DT_BF16>(x, wt, act, M, p, xmtt, st, ev0, ev1);
  else dispatch_gated<DT_F16>(x, wt, act, M, p, xmtt, st, ev0, ev1);
  return hipGetLastError();
}

hipError_t gemm(int dtype, const void* x, const void* wt, int M, const GemmPlan& p, float* part, size_t slice_stride,
                int xmtt, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (M <= 0) return hipSuccess;
  if (dtype == DT_F32) {
    if (xmtt) return hipErrorInvalidValue;   // fp32 rows are always row-major
    dim3 grid((p.N + 3) / 4, (M + 7) / 8);
    launch_timed(gemm32_kernel, grid, dim3(256), st, ev0, ev1, (const float*)x, (const float*)wt, part, M, p.N, p.K, p.ldc);
  } else if (dtype == DT_BF16) {
    if (p.NT == 4) dispatch16<DT_BF16, 4>(x, wt, part, M, p, slice_stride, xmtt, st, ev0, ev1);
    else dispatch16<DT_BF16, 2>(x, wt, part, M, p, slice_stride, xmtt, st, ev0, ev1);
  } else {
    if (p.NT == 4) dispatch16<DT_F16, 4>(x, wt, part, M, p, slice_stride, xmtt, st, ev0, ev1);
    else dispatch16<DT_F16, 2>(x, wt, part, M, p, slice_stride, xmtt, st, ev0, ev1);
  }
  return hipGetLastError();
}

}  // namespace flk
