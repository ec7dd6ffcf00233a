// Ragged masked self-attention of one fused decode iteration: every live row attends over its own request's
// cached K/V rows [0, len) -- requests arrived at different times, so every row has its own length
// (temporal fusion, Section V-C; the attention itself sits in Algorithm 2's "...").
//
// HBM-bound (about 1 flop per byte, every K/V byte read once), so the kernel is a streamer:
//   * the cache is [slot][head][pos][d]: one head's rows are contiguous, a wave load instruction fetches
//     64 lanes x 16 B = 1 KiB of consecutive rows, each row spread over LPR = d*elem/16 adjacent lanes;
//   * the lane group that holds a row reduces q.k over its LPR lanes with DPP, keeps its own online softmax
//     state (m, l, o) over the rows it sees (rows r with r % (64/LPR) == group), and the groups are merged
//     once at the end -- no LDS, no barriers, registers only, occupancy hides latency;
//   * work is flattened to (row, chunk) x head so a launch has thousands of similar wave tasks however ragged the
//     lengths are: a row of len positions has ceil(len / CHUNK) chunks of equal length (no short remainder task, which
//     would leave the memory system under-used while the full-length tasks finish); chunking depends on the
//     request's own length only, and a second tiny kernel merges a row's chunks in chunk order (results never depend
//     on other rows).
#include "flover_dev.h"
#include "flover_kernels.h"

namespace flk {

// grid = (n_items, n_head / 4), block = 256: wave w handles head blockIdx.y * 4 + w of item blockIdx.x.
// items[i] = (row, chunk, slot, len).  Writes the unnormalised partial (m, l, o[D]) of (row, chunk, head) at index
// (row * maxch + chunk) * n_head + head: the place depends on the row and the chunk alone, so the merge kernel finds a
// row's partials without looking anything up.
template <int DT, int D, int U>
__global__ __launch_bounds__(256) void attn_partial_kernel(const void* __restrict__ q, const void* __restrict__ kc,
                                                           const void* __restrict__ vc, const int4* __restrict__ items, int nh,
                                                           int Smax, int chunk, int maxch,
                                                           float scale, float* __restrict__ pml, float* __restrict__ po) {
  constexpr int EB = (DT == DT_F32) ? 4 : 2;
  constexpr int EPL = 16 / EB;          // elements per lane
  constexpr int LPR = D / EPL;          // lanes per row
  constexpr int RPW = 64 / LPR;         // rows per wave load
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int item = blockIdx.x;
  const int hd = blockIdx.y * 4 + wave;
  const int4 it = items[item];          // one load: the cache addresses below depend on nothing else
  const int row = it.x, ch = it.y, slot = it.z, len = it.w;
  // the row's ceil(len / chunk) chunks are made equally long, so that no wave task of a row is a short remainder
  const int nch = (len + chunk - 1) / chunk, cr = (len + nch - 1) / nch;
  const int j0 = ch * cr, j1 = min(len, j0 + cr);
  const int grp = lane / LPR, li = lane % LPR;

  float qf[EPL];
  {
    const u32x4_t qr = *(const u32x4_t*)((const char*)q + ((size_t)(row * nh + hd) * D + li * EPL) * EB);
    unpack16<DT>(qr, qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] *= scale;
  }
  const size_t head_off = ((size_t)slot * nh + hd) * Smax * D * EB + (size_t)li * 16;
  const char* kb = (const char*)kc + head_off;
  const char* vb = (const char*)vc + head_off;

  float m = -INFINITY, l = 0.f, o[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) o[e] = 0.f;

  // Two register buffers: the loads of the next RPW*U rows are in flight while the current ones are consumed.
  u32x4_t krA[U], vrA[U], krB[U], vrB[U];
  auto load = [&](u32x4_t* kr, u32x4_t* vr, int jb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = min(jb + u * RPW + grp, j1 - 1);      // clamp: stays inside the request's valid rows
      kr[u] = __builtin_nontemporal_load((const u32x4_t*)(kb + (size_t)r * D * EB));
      vr[u] = __builtin_nontemporal_load((const u32x4_t*)(vb + (size_t)r * D * EB));
    }
  };
  auto consume = [&](const u32x4_t* kr, const u32x4_t* vr, int jb) {
    float s[U];
    float tmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      unpack16<DT>(kr[u], kf);
      float d0 = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d0 = fmaf(qf[e], kf[e], d0);
      d0 = group_sum<LPR>(d0);
      s[u] = (jb + u * RPW + grp < j1) ? d0 : -INFINITY;
      tmax = fmaxf(tmax, s[u]);
    }
    const float mn = fmaxf(m, tmax);
    const float ms = (mn == -INFINITY) ? 0.f : mn;       // a group that has seen no valid row yet
    const float alpha = __expf(m - ms);                  // m = -inf -> 0
    l *= alpha;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] *= alpha;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float p = __expf(s[u] - ms);
      l += p;
      float vf[EPL];
      unpack16<DT>(vr[u], vf);
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] = fmaf(p, vf[e], o[e]);
    }
    m = mn;
  };
  constexpr int STEP = RPW * U;
  load(krA, vrA, j0);
  int jb = j0;
  // Steady state without branches (the compiler's wait counts for the in-order memory counter collapse to "wait for
  // everything" around a branch, which would make consuming one buffer wait for the other's loads too); the loads
  // past the chunk re-read its last row.
  for (; jb + 2 * STEP <= j1; jb += 2 * STEP) {
    load(krB, vrB, jb + STEP);
    __builtin_amdgcn_sched_barrier(0);
    consume(krA, vrA, jb);
    load(krA, vrA, jb + 2 * STEP);
    __builtin_amdgcn_sched_barrier(0);
    consume(krB, vrB, jb + STEP);
  }
  if (jb < j1) {                                           // one or two steps left (wave-uniform)
    const bool two = jb + STEP < j1;
    if (two) load(krB, vrB, jb + STEP);
    consume(krA, vrA, jb);
    if (two) consume(krB, vrB, jb + STEP);
  }
  // merge the RPW lane groups (lanes with equal li): butterfly over the group index bits
  if constexpr (RPW > 1) {
    float mt = m;
#pragma unroll
    for (int dlt = LPR; dlt < 64; dlt <<= 1) mt = fmaxf(mt, __shfl_xor(mt, dlt, 64));
    const float w = (m == -INFINITY) ? 0.f : __expf(m - mt);
    l *= w;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] *= w;
#pragma unroll
    for (int dlt = LPR; dlt < 64; dlt <<= 1) {
      l += __shfl_xor(l, dlt, 64);
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] += __shfl_xor(o[e], dlt, 64);
    }
    m = mt;
  }
  if (grp == 0) {
    const size_t pi = ((size_t)row * maxch + ch) * nh + hd;
    float* op = po + pi * D + li * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) op[e] = o[e];
    if (li == 0) {
      pml[pi * 2] = m;
      pml[pi * 2 + 1] = l;
    }
  }
}

// grid = (M, ceil(n_head / HPB)), block = 256: merges a row's chunks in chunk order, normalises, rounds to dtype.  A
// thread owns 4 consecutive elements of one head's output (D / 4 threads per head, HPB = 1024 / D heads per block).
// out is [M][nh * D] row-major (mtt == 0) or in the GEMM's fragment order with mtt row tiles.
// The partials of a row sit at a place known from the row index alone, so the loads of the first four chunks go out
// together with the load of the row's length (one memory round trip for rows of up to 4 chunks; slots of chunks the row
// does not have are read and never used); longer rows fetch the rest in a second round.
template <int DT, int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ pml, const float* __restrict__ po,
                                                         const int* __restrict__ row_len, int chunk, int maxch, int nh,
                                                         void* __restrict__ out, int mtt) {
  constexpr int FIRST = 4;
  constexpr int TPH = D / 4, HPB = 256 / TPH;
  const int row = blockIdx.x, hd = blockIdx.y * HPB + threadIdx.x / TPH, i = (threadIdx.x % TPH) * 4;
  if (hd >= nh) return;
  const size_t base = ((size_t)row * maxch) * nh + hd;       // + ch * nh
  float mc[FIRST], lc[FIRST];
  f32x4_t oc[FIRST];
#pragma unroll
  for (int j = 0; j < FIRST; ++j) {
    const size_t pi = base + (size_t)min(j, maxch - 1) * nh;
    const float2 ml = *(const float2*)(pml + pi * 2);
    mc[j] = ml.x;
    lc[j] = ml.y;
    oc[j] = ld4(po + pi * D + i);
  }
  const int nc = (row_len[row] + chunk - 1) / chunk;
  float red_m = -INFINITY;                                    // the global maximum needs the m of every chunk
#pragma unroll
  for (int j = 0; j < FIRST; ++j)
    if (j < nc) red_m = fmaxf(red_m, mc[j]);
  for (int c = FIRST; c < nc; ++c) red_m = fmaxf(red_m, pml[(base + (size_t)c * nh) * 2]);
  float l = 0.f;
  f32x4_t o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < FIRST; ++j)
    if (j < nc) {
      const float w = __expf(mc[j] - red_m);
      l += w * lc[j];
      o += w * oc[j];
    }
  for (int c0 = FIRST; c0 < nc; c0 += 4) {      // longer rows: 4 chunks at a time, loads first, arithmetic in chunk order
    float m2[4], l2[4];
    f32x4_t o2[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const size_t pi = base + (size_t)min(c0 + j, nc - 1) * nh;
      const float2 ml = *(const float2*)(pml + pi * 2);
      m2[j] = ml.x;
      l2[j] = ml.y;
      o2[j] = ld4(po + pi * D + i);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (c0 + j < nc) {
        const float w = __expf(m2[j] - red_m);
        l += w * l2[j];
        o += w * o2[j];
      }
  }
  stv4<DT>(out, xrow_index(row, hd * D + i, nh * D, mtt), o / l);
}

// ---------------------------------------------------------------- pre-processing variant (context decoder)
// Rows of one pre-processing pass are consecutive positions of ONE slot, so neighbouring rows read almost the same
// K/V rows.  Here a wave serves QB consecutive query rows at once: every K/V row it loads is used by all of them
// (causal mask per query), which divides the cache traffic of the context pass by up to QB.  Same chunking, same
// partial layout and the same merge kernel as above.
// grid = (n_blocks, n_head / 4), block = 256.  blocks[b] = (first row, rows in block (<= QB), chunk, -).
template <int DT, int D, int QB>
__global__ __launch_bounds__(256) void attn_prefill_kernel(const void* __restrict__ q, const void* __restrict__ kc,
                                                           const void* __restrict__ vc, const int4* __restrict__ blocks,
                                                           const int* __restrict__ row_slot,
                                                           const int* __restrict__ row_len, int nh, int Smax, int chunk,
                                                           int maxch, float scale, float* __restrict__ pml,
                                                           float* __restrict__ po) {
  constexpr int EB = (DT == DT_F32) ? 4 : 2;
  constexpr int EPL = 16 / EB;
  constexpr int LPR = D / EPL;
  constexpr int RPW = 64 / LPR;
  constexpr int U = 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int4 bk = blocks[blockIdx.x];
  const int first = bk.x, nr = bk.y, ch = bk.z;
  const int hd = blockIdx.y * 4 + wave;
  const int slot = row_slot[first];
  const int len0 = row_len[first];                          // rows are consecutive positions: len_i = len0 + i
  const int j0 = ch * chunk, j1 = min(len0 + nr - 1, j0 + chunk);
  const int grp = lane / LPR, li = lane % LPR;

  float qf[QB][EPL];
#pragma unroll
  for (int i = 0; i < QB; ++i) {
    const int r = first + min(i, nr - 1);
    const u32x4_t qr = *(const u32x4_t*)((const char*)q + ((size_t)(r * nh + hd) * D + li * EPL) * EB);
    unpack16<DT>(qr, qf[i]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[i][e] *= scale;
  }
  const size_t head_off = ((size_t)slot * nh + hd) * Smax * D * EB + (size_t)li * 16;
  const char* kb = (const char*)kc + head_off;
  const char* vb = (const char*)vc + head_off;

  float m[QB], l[QB], o[QB][EPL];
#pragma unroll
  for (int i = 0; i < QB; ++i) {
    m[i] = -INFINITY;
    l[i] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[i][e] = 0.f;
  }
  for (int jb = j0; jb < j1; jb += RPW * U) {
    u32x4_t kr[U], vr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = min(jb + u * RPW + grp, j1 - 1);
      kr[u] = *(const u32x4_t*)(kb + (size_t)r * D * EB);
      vr[u] = *(const u32x4_t*)(vb + (size_t)r * D * EB);
    }
    float kf[U][EPL], vf[U][EPL];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      unpack16<DT>(kr[u], kf[u]);
      unpack16<DT>(vr[u], vf[u]);
    }
#pragma unroll
    for (int i = 0; i < QB; ++i) {
      float sc[U];
      float tmax = -INFINITY;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float d0 = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d0 = fmaf(qf[i][e], kf[u][e], d0);
        d0 = group_sum<LPR>(d0);
        sc[u] = (jb + u * RPW + grp < min(len0 + i, j1) && i < nr) ? d0 : -INFINITY;   // causal: key < len_i
        tmax = fmaxf(tmax, sc[u]);
      }
      const float mn = fmaxf(m[i], tmax);
      const float ms = (mn == -INFINITY) ? 0.f : mn;
      const float alpha = __expf(m[i] - ms);
      l[i] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[i][e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = __expf(sc[u] - ms);
        l[i] += p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[i][e] = fmaf(p, vf[u][e], o[i][e]);
      }
      m[i] = mn;
    }
  }
#pragma unroll
  for (int i = 0; i < QB; ++i) {
    float mi = m[i], lv = l[i];
    if constexpr (RPW > 1) {
      float mt = mi;
#pragma unroll
      for (int dlt = LPR; dlt < 64; dlt <<= 1) mt = fmaxf(mt, __shfl_xor(mt, dlt, 64));
      const float w = (mi == -INFINITY) ? 0.f : __expf(mi - mt);
      lv *= w;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[i][e] *= w;
#pragma unroll
      for (int dlt = LPR; dlt < 64; dlt <<= 1) {
        lv += __shfl_xor(lv, dlt, 64);
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[i][e] += __shfl_xor(o[i][e], dlt, 64);
      }
      mi = mt;
    }
    const int r = first + i;
    if (i < nr && ch * chunk < len0 + i && grp == 0) {       // this chunk holds keys this query may see
      const size_t pi = ((size_t)r * maxch + ch) * nh + hd;
      float* op = po + pi * D + li * EPL;
#pragma unroll
      for (int e = 0; e < EPL; ++e) op[e] = o[i][e];
      if (li == 0) {
        pml[pi * 2] = mi;
        pml[pi * 2 + 1] = lv;
      }
    }
  }
}

// ---------------------------------------------------------------- pre-processing variant on the matrix cores
// 16-bit models: a wave serves 32 consecutive query rows (two tiles of 16) and walks its chunk 32 keys at a time.
//   scores   S^T[key][query] = K . Q^T   : A = K rows (a lane's 16 bytes of a cache row are 8 consecutive d of one
//                                          key), B = Q^T (8 consecutive d of one query) -- both straight from memory;
//   softmax  per query = per output column: 8 values in the lane, then the 4 lane groups (2 shuffles);
//   output   O^T[d][query] += V^T . P^T  : B = P^T is what the lane already holds from S^T (keys 4g..4g+3 of both
//            16-key tiles = its 8 k-slots), A = V^T needs 8 keys of one d per lane: the V rows are staged in LDS
//            (wave-private, row stride D + 8 elements: 16-byte aligned and conflict-free) and read back transposed.
// P enters the second product as two 16-bit terms (value + rounding remainder), i.e. with 16 or more significant bits;
// m, l and the accumulators stay fp32.  Same chunking, partial layout and merge kernel as the other variants.     grid = (n_blocks, n_head / 4), block = 256 (a wave per head).
constexpr int kPrefillMfmaQB = 32;
template <int DT> __device__ __forceinline__ uint32_t pack2(float a, float b) {
  if constexpr (DT == DT_BF16) return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
  else return (uint32_t)f32_to_f16(a) | ((uint32_t)f32_to_f16(b) << 16);
}
template <int DT> __device__ __forceinline__ f32x4_t mfma_kq(const u32x4_t& a, const u32x4_t& b, f32x4_t c) {
  if constexpr (DT == DT_BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

template <int DT, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_prefill_mfma_kernel(const void* __restrict__ q, const void* __restrict__ kc,
                                                                const void* __restrict__ vc,
                                                                const int4* __restrict__ blocks,
                                                                const int* __restrict__ row_slot,
                                                                const int* __restrict__ row_len, int nh, int Smax,
                                                                int chunk, int maxch, float scale,
                                                                float* __restrict__ pml, float* __restrict__ po) {
  static_assert(DT != DT_F32, "16-bit models only");
  constexpr int QT = kPrefillMfmaQB / 16;   // query tiles per wave
  constexpr int KS = D / 32;                // MFMA steps over the head dimension
  constexpr int DTL = D / 16;               // output tiles over the head dimension
  constexpr int VSTR = D + 8;               // LDS row stride (elements)
  constexpr int LPRV = D / 8;               // lanes per V row when staging (16 bytes each)
  constexpr int RPL = 64 / LPRV;            // V rows per wave load
  __shared__ __attribute__((aligned(16))) uint16_t vlds[4][32 * VSTR];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, n = lane & 15;
  const int4 bk = blocks[blockIdx.x];
  const int first = bk.x, nr = bk.y, ch = bk.z;
  const int hd = blockIdx.y * 4 + wave;
  const int slot = row_slot[first];
  const int len0 = row_len[first];                          // rows are consecutive positions: len_i = len0 + i
  const int j0 = ch * chunk, j1 = min(len0 + nr - 1, j0 + chunk);
  uint16_t* vl = vlds[wave];

  u32x4_t qf[QT][KS];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int r = first + min(t * 16 + n, nr - 1);
    const uint16_t* qr = (const uint16_t*)q + (size_t)(r * nh + hd) * D + g * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[t][ks] = *(const u32x4_t*)(qr + ks * 32);
  }
  const size_t head_off = ((size_t)slot * nh + hd) * Smax * D;
  const uint16_t* kb = (const uint16_t*)kc + head_off;
  const uint16_t* vb = (const uint16_t*)vc + head_off;

  f32x4_t oacc[DTL][QT];
  float m[QT], l[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m[t] = -INFINITY;
    l[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DTL; ++dt) oacc[dt][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }

  for (int jb = j0; jb < j1; jb += 32) {
    // K rows as the A operand, V rows to LDS (rows past the chunk repeat its last row; they are masked below)
    u32x4_t kf[2][KS], vr[32 / RPL];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const uint16_t* kr = kb + (size_t)min(jb + kt * 16 + n, j1 - 1) * D + g * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[kt][ks] = *(const u32x4_t*)(kr + ks * 32);
    }
#pragma unroll
    for (int i = 0; i < 32 / RPL; ++i) {
      const int row = i * RPL + lane / LPRV;
      vr[i] = *(const u32x4_t*)(vb + (size_t)min(jb + row, j1 - 1) * D + (lane % LPRV) * 8);
    }
    __builtin_amdgcn_wave_barrier();          // the previous block's transposed reads come before these writes
#pragma unroll
    for (int i = 0; i < 32 / RPL; ++i) {
      const int row = i * RPL + lane / LPRV;
      *(u32x4_t*)(vl + row * VSTR + (lane % LPRV) * 8) = vr[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // scores: rows = keys kt*16 + 4g + r, column = query n of tile t
    u32x4_t pb[QT], pl[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      f32x4_t sacc[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        sacc[kt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) sacc[kt] = mfma_kq<DT>(kf[kt][ks], qf[t][ks], sacc[kt]);
      }
      const int qi = t * 16 + n;
      const int lim = (qi < nr) ? min(len0 + qi, j1) : 0;        // causal: key < len_i, and inside the chunk
      float sc[8];
      float tmax = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = jb + kt * 16 + 4 * g + r;
          const float v = (key < lim) ? sacc[kt][r] * scale : -INFINITY;
          sc[kt * 4 + r] = v;
          tmax = fmaxf(tmax, v);
        }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float mn = fmaxf(m[t], tmax);
      const float ms = (mn == -INFINITY) ? 0.f : mn;
      const float alpha = __expf(m[t] - ms);
      float p[8], ps = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        p[j] = __expf(sc[j] - ms);
        ps += p[j];
      }
      l[t] = l[t] * alpha + ps;                                   // per-lane share; the lane groups are added at the end
      m[t] = mn;
#pragma unroll
      for (int dt = 0; dt < DTL; ++dt) oacc[dt][t] *= alpha;
      // The probabilities enter the second product as two 16-bit terms, p = hi + lo with hi = p rounded to the model
      // dtype and lo = (p - hi) rounded: 16 significant bits for bf16 (more for fp16), so that this kernel weighs the V
      // rows as accurately as the decode kernel's fp32 probabilities do (one term alone would add a rounding point
      // that the decode path does not have).
      float q_[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) q_[j] = p[j] - rdt<DT>(p[j]);
      pb[t] = u32x4_t{pack2<DT>(p[0], p[1]), pack2<DT>(p[2], p[3]), pack2<DT>(p[4], p[5]), pack2<DT>(p[6], p[7])};
      pl[t] = u32x4_t{pack2<DT>(q_[0], q_[1]), pack2<DT>(q_[2], q_[3]), pack2<DT>(q_[4], q_[5]), pack2<DT>(q_[6], q_[7])};
    }
    // output: A = V^T, k-slot j of lane group g <-> key 4g + j (j < 4) or 16 + 4g + (j - 4), as in pb
#pragma unroll
    for (int dt = 0; dt < DTL; ++dt) {
      const uint16_t* vcol = vl + dt * 16 + n;
      uint32_t w[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int ka = (jj < 2) ? 4 * g + 2 * jj : 16 + 4 * g + 2 * (jj - 2);
        w[jj] = (uint32_t)vcol[ka * VSTR] | ((uint32_t)vcol[(ka + 1) * VSTR] << 16);
      }
      const u32x4_t va = u32x4_t{w[0], w[1], w[2], w[3]};
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        oacc[dt][t] = mfma_kq<DT>(va, pl[t], oacc[dt][t]);
        oacc[dt][t] = mfma_kq<DT>(va, pb[t], oacc[dt][t]);
      }
    }
  }
  // partial results: lane (n, g) owns O[query n][d = dt*16 + 4g .. +3]
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float lv = l[t];
    lv += __shfl_xor(lv, 16, 64);
    lv += __shfl_xor(lv, 32, 64);
    const int qi = t * 16 + n;
    const int r = first + min(qi, nr - 1);
    if (qi < nr && ch * chunk < len0 + qi) {                     // this chunk holds keys this query may see
      const size_t pi = ((size_t)r * maxch + ch) * nh + hd;
#pragma unroll
      for (int dt = 0; dt < DTL; ++dt) *(f32x4_t*)(po + pi * D + dt * 16 + 4 * g) = oacc[dt][t];
      if (g == 0) {
        pml[pi * 2] = m[t];
        pml[pi * 2 + 1] = lv;
      }
    }
  }
}

// ---------------------------------------------------------------- host side

int attn_chunk() { return 256; }
int prefill_rows_per_block(int dtype) { return dtype == DT_F32 ? kPrefillQB : kPrefillMfmaQB; }

template <int DT, int D>
static void launch_attn(const void* q, const void* kc, const void* vc, const AttnWork& w, int M, int nh, int Smax,
                        void* out, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const float scale = 1.0f / sqrtf((float)D);
  launch_timed(attn_partial_kernel<DT, D, 4>, dim3(w.n_items, nh / 4), dim3(256), st, ev0, ev1, q, kc, vc, w.items, nh, Smax,
               w.chunk, w.maxch, scale, w.pml, w.po);
  attn_merge_kernel<DT, D><<<dim3(M, (nh * D + 1023) / 1024), 256, 0, st>>>(w.pml, w.po, w.row_len, w.chunk, w.maxch, nh, out, w.out_mtt);
}

hipError_t decode_attention(int dtype, int d, const void* q, const void* kc, const void* vc, const AttnWork& w, int M,
                            int nh, int Smax, void* out, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (M <= 0 || w.n_items <= 0) return hipSuccess;
  if (d == 128) {
    if (dtype == DT_F32) launch_attn<DT_F32, 128>(q, kc, vc, w, M, nh, Smax, out, st, ev0, ev1);
    else if (dtype == DT_F16) launch_attn<DT_F16, 128>(q, kc, vc, w, M, nh, Smax, out, st, ev0, ev1);
    else launch_attn<DT_BF16, 128>(q, kc, vc, w, M, nh, Smax, out, st, ev0, ev1);
  } else {
    if (dtype == DT_F32) launch_attn<DT_F32, 64>(q, kc, vc, w, M, nh, Smax, out, st, ev0, ev1);
    else if (dtype == DT_F16) launch_attn<DT_F16, 64>(q, kc, vc, w, M, nh, Smax, out, st, ev0, ev1);
    else launch_attn<DT_BF16, 64>(q, kc, vc, w, M, nh, Smax, out, st, ev0, ev1);
  }
  return hipGetLastError();
}

template <int DT, int D>
static void launch_prefill(const void* q, const void* kc, const void* vc, const AttnWork& w, int M, int nh, int Smax,
                           void* out, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)D);
  if constexpr (DT == DT_F32)
    attn_prefill_kernel<DT, D, kPrefillQB><<<dim3(w.n_blocks, nh / 4), 256, 0, st>>>(
        q, kc, vc, w.blocks, w.row_slot, w.row_len, nh, Smax, w.chunk, w.maxch, scale, w.pml, w.po);
  else
    attn_prefill_mfma_kernel<DT, D><<<dim3(w.n_blocks, nh / 4), 256, 0, st>>>(
        q, kc, vc, w.blocks, w.row_slot, w.row_len, nh, Smax, w.chunk, w.maxch, scale, w.pml, w.po);
  attn_merge_kernel<DT, D><<<dim3(M, (nh * D + 1023) / 1024), 256, 0, st>>>(w.pml, w.po, w.row_len, w.chunk, w.maxch, nh, out, w.out_mtt);
}

hipError_t prefill_attention(int dtype, int d, const void* q, const void* kc, const void* vc, const AttnWork& w, int M,
                             int nh, int Smax, void* out, hipStream_t st) {
  if (M <= 0 || w.n_blocks <= 0) return hipSuccess;
  if (d == 128) {
    if (dtype == DT_F32) launch_prefill<DT_F32, 128>(q, kc, vc, w, M, nh, Smax, out, st);
    else if (dtype == DT_F16) launch_prefill<DT_F16, 128>(q, kc, vc, w, M, nh, Smax, out, st);
    else launch_prefill<DT_BF16, 128>(q, kc, vc, w, M, nh, Smax, out, st);
  } else {
    if (dtype == DT_F32) launch_prefill<DT_F32, 64>(q, kc, vc, w, M, nh, Smax, out, st);
    else if (dtype == DT_F16) launch_prefill<DT_F16, 64>(q, kc, vc, w, M, nh, Smax, out, st);
    else launch_prefill<DT_BF16, 64>(q, kc, vc, w, M, nh, Smax, out, st);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------- memory shuffle copy (Section V-D)
// One launch moves every listed slot: block b -> (move, segment = (layer, K|V, head), piece of PIECE bytes).
// moves[i] = (src slot, dst slot, bytes per segment = len * d * elem, first block index).
// Sources lie outside the chosen window and destinations are holes inside it, so the two sets are disjoint and
// the copies can run in any order.
__global__ __launch_bounds__(256) void compact_kernel(char* __restrict__ cache, const int4* __restrict__ moves, int n_moves,
                                                      int nseg_per_slot, int C, size_t slot_bytes, int piece) {
  // binary search: last move whose first block <= blockIdx.x
  int lo = 0, hi = n_moves - 1;
  const int b = blockIdx.x;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (moves[mid].w <= b) lo = mid; else hi = mid - 1;
  }
  const int4 mv = moves[lo];
  const int bytes = mv.z;
  const int ppseg = (bytes + piece - 1) / piece;
  const int rel = b - mv.w;
  const int seg = rel / ppseg, pc = rel - seg * ppseg;
  // segment `seg` = (layer*2 + kv) * nh + head; cache is [(layer*2+kv)][C][nh][S][d]
  const int nh = nseg_per_slot;             // heads per (layer,kv) plane, passed by the host
  const int plane = seg / nh, head = seg - plane * nh;
  const size_t base = ((size_t)plane * C) * slot_bytes;
  const size_t head_bytes = slot_bytes / nh;
  const char* src = cache + base + (size_t)mv.x * slot_bytes + (size_t)head * head_bytes + (size_t)pc * piece;
  char* dst = cache + base + (size_t)mv.y * slot_bytes + (size_t)head * head_bytes + (size_t)pc * piece;
  const int n = min(piece, bytes - pc * piece);       // multiple of 16
  for (int off = threadIdx.x * 16; off < n; off += 256 * 16) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)(src + off));
    __builtin_nontemporal_store(v, (u32x4_t*)(dst + off));
  }
}

hipError_t compact(void* cache, int planes, int C, int nh, size_t slot_bytes, const void* moves_dev, int n_moves,
                   int total_blocks, int piece, hipStream_t st) {
  if (n_moves <= 0 || total_blocks <= 0) return hipSuccess;
  (void)planes;
  compact_kernel<<<total_blocks, 256, 0, st>>>((char*)cache, (const int4*)moves_dev, n_moves, nh, C, slot_bytes, piece);
  return hipGetLastError();
}

}  // namespace flk
