// Weight GEMMs of the fused rows (Algorithm 2's GEMM calls over [buffer + offset, size), Section V-C).
//
// y[m][n] = sum_k x[m][k] W[n][k], fp32 accumulation, M = live rows (small), W streamed once from HBM.
// The work is HBM-bound for M up to a few hundred (M flop per weight byte), so the design goal is to stream W
// at full bandwidth:
//   * W is re-tiled once at init into MFMA operand order: tile (n-tile of 16 columns, k-block of 32) is 1 KiB,
//     lane l holds W[n0 + l%16][k0 + 8*(l/16) .. +8], so every wave load is one contiguous, fully used 1 KiB.
//   * a wave owns 64 output columns (4 n-tiles) x one K slice x up to 128 rows; no LDS, no barriers: the rows'
//     operand comes straight from L2/L1 (the 4 waves of a block share the K slice, so they hit the same lines).
//   * split-K: slice count and boundaries depend on (N, K) only -- never on M -- and partial sums are written per
//     slice and added by the consumer in slice order, so a row's result does not depend on which other rows
//     are live (the paper's premise that fused requests undergo identical operations).
//   * MFMA v_mfma_f32_16x16x32_{bf16,f16}: A = 16 rows of x, B = 16 columns of W, 32-deep.
// fp32 models (tiny configurations only) use a plain FMA kernel on the untiled matrix.
#include "flover_dev.h"
#include "flover_kernels.h"

namespace flk {

// ---------------------------------------------------------------- re-tiling (init time)

__global__ void retile16_kernel(const uint16_t* __restrict__ W, u32x4_t* __restrict__ wt, int N, int K, int KB,
                                int ntile0, long total) {
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
  wt[((size_t)(ntile0 + ntile) * KB + kb) * 64 + lane] = v;
}

// ---------------------------------------------------------------- 16-bit MFMA kernel

template <int DT> __device__ __forceinline__ f32x4_t mfma16(const u32x4_t& a, const u32x4_t& b, f32x4_t c) {
  if constexpr (DT == DT_BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// grid = (ceil(ngroups/4), S, ceil(M/(16*MT))), block = 256 (4 independent waves)
template <int DT, int MT, int PF>
__global__ __launch_bounds__(256) void gemm16_kernel(const uint16_t* __restrict__ x, const u32x4_t* __restrict__ wt,
                                                     float* __restrict__ part, int M, int N, int K, int ngroups, int KB,
                                                     int kbs, size_t slice_stride, int ldc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = blockIdx.x * 4 + wave;
  if (g >= ngroups) return;
  const int s = blockIdx.y;
  const int m0 = blockIdx.z * (16 * MT);
  const int kb0 = s * kbs;
  const int kb1 = min(KB, kb0 + kbs);

  f32x4_t acc[MT][4];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[i][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const u32x4_t* wp = wt + ((size_t)(g * 4) * KB) * 64 + lane;                     // + t*KB*64 + kb*64
  const uint16_t* xp = x + (size_t)(m0 + (lane & 15)) * K + (lane >> 4) * 8;     // + i*16*K + kb*32
  const size_t wtile = (size_t)KB * 64;

  u32x4_t bq[PF][4], aq[PF][MT];
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    const int kk = min(kb0 + j, kb1 - 1);
#pragma unroll
    for (int t = 0; t < 4; ++t) bq[j][t] = __builtin_nontemporal_load(wp + t * wtile + (size_t)kk * 64);
#pragma unroll
    for (int i = 0; i < MT; ++i) aq[j][i] = *(const u32x4_t*)(xp + (size_t)i * 16 * K + kk * 32);
  }
  for (int kb = kb0; kb < kb1; kb += PF) {
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      if (kb + j < kb1) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int t = 0; t < 4; ++t) acc[i][t] = mfma16<DT>(aq[j][i], bq[j][t], acc[i][t]);
      }
      const int kk = min(kb + j + PF, kb1 - 1);      // tail re-reads the last block (in bounds, unused)
#pragma unroll
      for (int t = 0; t < 4; ++t) bq[j][t] = __builtin_nontemporal_load(wp + t * wtile + (size_t)kk * 64);
#pragma unroll
      for (int i = 0; i < MT; ++i) aq[j][i] = *(const u32x4_t*)(xp + (size_t)i * 16 * K + kk * 32);
    }
  }
  float* out = part + (size_t)s * slice_stride;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int n = (g * 4 + t) * 16 + (lane & 15);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + i * 16 + (lane >> 4) * 4 + r;
        if (m < M && n < N) out[(size_t)m * ldc + n] = acc[i][t][r];
      }
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
  if (dtype == DT_F32) {
    p.Npad = N;
    p.KB = 0;
    p.S = 1;
    p.kbs = 0;
    return p;
  }
  p.Npad = (N + 63) / 64 * 64;
  p.KB = K / 32;
  const int ngroups = p.Npad / 64;
  // enough waves to fill 256 CUs a few times over, each with at least 8 k-blocks to stream; a function of (N,K) only
  int S = (2048 + ngroups - 1) / ngroups;
  int maxS = p.KB / 8;
  if (maxS < 1) maxS = 1;
  if (S > maxS) S = maxS;
  if (S > 16) S = 16;
  if (S < 1) S = 1;
  p.kbs = (p.KB + S - 1) / S;
  p.S = (p.KB + p.kbs - 1) / p.kbs;
  return p;
}

size_t gemm_tiled_bytes(int dtype, int N, int K) {
  if (dtype == DT_F32) return (size_t)N * K * 4;
  const size_t Npad = (size_t)(N + 63) / 64 * 64;
  return Npad * K * 2;
}

hipError_t retile(int dtype, const void* W, int N, int K, void* tiled, int n_off, hipStream_t st) {
  if (dtype == DT_F32)
    return hipMemcpyAsync((char*)tiled + (size_t)n_off * K * 4, W, (size_t)N * K * 4, hipMemcpyDeviceToDevice, st);
  const int KB = K / 32;
  const int ntiles = (N + 15) / 16;
  const long total = (long)ntiles * KB * 64;
  retile16_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>((const uint16_t*)W, (u32x4_t*)tiled, N, K, KB,
                                                                         n_off / 16, total);
  return hipGetLastError();
}

hipError_t zero_fill(void* p, size_t bytes, hipStream_t st) { return hipMemsetAsync(p, 0, bytes, st); }

template <int DT, int MT, int PF>
static void launch16(const void* x, const void* wt, float* part, int M, const GemmPlan& p, size_t slice_stride, int ldc,
                     hipStream_t st) {
  const int ngroups = p.Npad / 64;
  dim3 grid((ngroups + 3) / 4, p.S, (M + 16 * MT - 1) / (16 * MT));
  gemm16_kernel<DT, MT, PF><<<grid, 256, 0, st>>>((const uint16_t*)x, (const u32x4_t*)wt, part, M, p.N, p.K, ngroups, p.KB,
                                                  p.kbs, slice_stride, ldc);
}

template <int DT>
static void dispatch16(const void* x, const void* wt, float* part, int M, const GemmPlan& p, size_t ss, int ldc,
                       hipStream_t st) {
  if (M <= 16) launch16<DT, 1, 8>(x, wt, part, M, p, ss, ldc, st);
  else if (M <= 32) launch16<DT, 2, 6>(x, wt, part, M, p, ss, ldc, st);
  else if (M <= 64) launch16<DT, 4, 4>(x, wt, part, M, p, ss, ldc, st);
  else launch16<DT, 8, 2>(x, wt, part, M, p, ss, ldc, st);
}

hipError_t gemm(int dtype, const void* x, const void* wt, int M, const GemmPlan& p, float* part, size_t slice_stride,
                int ldc, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  if (dtype == DT_F32) {
    dim3 grid((p.N + 3) / 4, (M + 7) / 8);
    gemm32_kernel<<<grid, 256, 0, st>>>((const float*)x, (const float*)wt, part, M, p.N, p.K, ldc);
  } else if (dtype == DT_BF16) {
    dispatch16<DT_BF16>(x, wt, part, M, p, slice_stride, ldc, st);
  } else {
    dispatch16<DT_F16>(x, wt, part, M, p, slice_stride, ldc, st);
  }
  return hipGetLastError();
}

}  // namespace flk
