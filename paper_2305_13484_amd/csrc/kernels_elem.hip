// Row-wise kernels of the fused decoder step (Algorithm 2's LayerNorm / GenericActivation calls over
// [buffer + offset, size), plus embedding, rotary + KV append and the greedy choice).
//
// Each consumes the split-K partial sums of the GEMM before it (added in slice order, then bias), so a GEMM's
// epilogue lives in the next launch and nothing depends on how many rows are live.  All are HBM/L2 streaming
// kernels: one block (or wave) per row, coalesced 4-byte-per-lane accesses, fixed reduction trees.
#include "flover_dev.h"
#include "flover_kernels.h"

namespace flk {

// sum of S partial slices at element idx, slice order
__device__ __forceinline__ float psum(const float* __restrict__ part, int S, size_t stride, size_t idx) {
  float v = part[idx];
  for (int s = 1; s < S; ++s) v += part[(size_t)s * stride + idx];
  return v;
}

// ---------------------------------------------------------------- embedding
// x[m][i] = wte[tok[m]][i] (+ wpe[pos[m]][i])            grid = M, block = 256
template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const void* __restrict__ wte, const void* __restrict__ wpe,
                                                    const int* __restrict__ tok, const int* __restrict__ pos,
                                                    float* __restrict__ x, int H) {
  const int m = blockIdx.x;
  const size_t t = (size_t)tok[m] * H;
  const size_t p = wpe ? (size_t)pos[m] * H : 0;
  for (int i = threadIdx.x; i < H; i += 256) {
    float v = ld<DT>(wte, t + i);
    if (wpe) v += ld<DT>(wpe, p + i);
    x[(size_t)m * H + i] = v;
  }
}

// ---------------------------------------------------------------- residual add + norm
// x[m] += sum_s part[s][m] + bias   (skipped when part == nullptr), then
// h[m] = LayerNorm(x[m]) * g + b   (RMS == 0)   or   x[m] / rms(x[m]) * g   (RMS == 1), rounded to dtype.
// grid = M, block = 256; H <= 256 * 32.
template <int DT, int RMS>
__global__ __launch_bounds__(256) void add_norm_kernel(float* __restrict__ x, const float* __restrict__ part, int S,
                                                       size_t stride, const void* __restrict__ bias,
                                                       const void* __restrict__ g, const void* __restrict__ b,
                                                       void* __restrict__ h, int H, float eps) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  constexpr int PER = 32;
  float v[PER];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < PER; ++c) {
    const int i = threadIdx.x + c * 256;
    v[c] = 0.f;
    if (i < H) {
      float t = x[(size_t)m * H + i];
      if (part) {
        float a = psum(part, S, stride, (size_t)m * H + i);
        if (bias) a += ld<DT>(bias, i);
        t += a;
        x[(size_t)m * H + i] = t;
      }
      v[c] = t;
      sum += RMS ? t * t : t;
    }
  }
  sum = block_sum<4>(sum, red);
  float mean = 0.f, inv;
  if (RMS) {
    inv = 1.0f / sqrtf(sum / (float)H + eps);
  } else {
    mean = sum / (float)H;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < PER; ++c)
      if (threadIdx.x + c * 256 < H) sq += (v[c] - mean) * (v[c] - mean);
    sq = block_sum<4>(sq, red);
    inv = 1.0f / sqrtf(sq / (float)H + eps);
  }
#pragma unroll
  for (int c = 0; c < PER; ++c) {
    const int i = threadIdx.x + c * 256;
    if (i < H) {
      float o = (v[c] - mean) * inv * ld<DT>(g, i);
      if (!RMS) o += ld<DT>(b, i);
      st<DT>(h, (size_t)m * H + i, o);
    }
  }
}

// ---------------------------------------------------------------- QKV epilogue: bias, rotary, KV append
// part: [S][M][3H] (q | k | v).  For row m (slot, pos) and head hd: q -> qout[m][hd][:] (dtype),
// k, v -> cache[slot][hd][pos][:] (dtype).  Rotary (LLaMA): pairs (i, i + d/2), cos/sin from a table [max_seq][d/2].
// grid = (M, n_head), block = d/2.
template <int DT>
__global__ void qkv_post_kernel(const float* __restrict__ part, int S, size_t stride, const void* __restrict__ bias,
                                const float* __restrict__ rope_cs, const int* __restrict__ slot,
                                const int* __restrict__ pos, void* __restrict__ qout, void* __restrict__ kcache,
                                void* __restrict__ vcache, int H, int nh, int d, int Smax) {
  const int m = blockIdx.x, hd = blockIdx.y, i = threadIdx.x, half = d >> 1;
  const size_t row = (size_t)m * 3 * H;
  const int c0 = hd * d + i, c1 = c0 + half;
  float q0 = psum(part, S, stride, row + c0), q1 = psum(part, S, stride, row + c1);
  float k0 = psum(part, S, stride, row + H + c0), k1 = psum(part, S, stride, row + H + c1);
  float v0 = psum(part, S, stride, row + 2 * H + c0), v1 = psum(part, S, stride, row + 2 * H + c1);
  if (bias) {
    q0 += ld<DT>(bias, c0); q1 += ld<DT>(bias, c1);
    k0 += ld<DT>(bias, H + c0); k1 += ld<DT>(bias, H + c1);
    v0 += ld<DT>(bias, 2 * H + c0); v1 += ld<DT>(bias, 2 * H + c1);
  }
  const int p = pos[m];
  if (rope_cs) {
    const float cs = rope_cs[((size_t)p * half + i) * 2], sn = rope_cs[((size_t)p * half + i) * 2 + 1];
    const float a = q0 * cs - q1 * sn, b = q1 * cs + q0 * sn;
    q0 = a; q1 = b;
    const float c = k0 * cs - k1 * sn, e = k1 * cs + k0 * sn;
    k0 = c; k1 = e;
  }
  st<DT>(qout, (size_t)m * H + c0, q0);
  st<DT>(qout, (size_t)m * H + c1, q1);
  const size_t kv = (((size_t)slot[m] * nh + hd) * Smax + p) * d;
  st<DT>(kcache, kv + i, k0);
  st<DT>(kcache, kv + i + half, k1);
  st<DT>(vcache, kv + i, v0);
  st<DT>(vcache, kv + i + half, v1);
}

// ---------------------------------------------------------------- MLP activation
// GPT:   a[m][j] = gelu_tanh(sum_s part[s][m][j] + b1[j])                      part row length F
// LLaMA: a[m][j] = silu(gate) * up, gate = part[..][m][j], up = part[..][m][F + j]   part row length 2F
template <int DT, int SWIGLU>
__global__ __launch_bounds__(256) void act_kernel(const float* __restrict__ part, int S, size_t stride,
                                                  const void* __restrict__ bias, void* __restrict__ a, int F, long total) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const long m = idx / F;
  const int j = (int)(idx - m * F);
  float o;
  if (SWIGLU) {
    const float g = psum(part, S, stride, (size_t)m * 2 * F + j);
    const float u = psum(part, S, stride, (size_t)m * 2 * F + F + j);
    o = g / (1.0f + expf(-g)) * u;
  } else {
    const float t = psum(part, S, stride, (size_t)m * F + j) + ld<DT>(bias, j);
    o = 0.5f * t * (1.0f + tanhf(0.7978845608028654f * (t + 0.044715f * t * t * t)));
  }
  st<DT>(a, idx, o);
}

// ---------------------------------------------------------------- logits + greedy token
// logits[m][j] = sum_s part[s][m][j] (fp32, optionally stored); tok[m] = argmax_j, lowest j on ties.
// grid = M, block = 256.
__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ part, int S, size_t stride,
                                                     float* __restrict__ logits, int* __restrict__ tok, int V) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  const int m = blockIdx.x;
  float best = -INFINITY;
  int arg = 0x7fffffff;
  for (int j = threadIdx.x; j < V; j += 256) {
    const float v = psum(part, S, stride, (size_t)m * V + j);
    if (logits) logits[(size_t)m * V + j] = v;
    if (v > best || (v == best && j < arg)) { best = v; arg = j; }
  }
  if (arg == 0x7fffffff) { best = -INFINITY; }
#pragma unroll
  for (int dlt = 1; dlt < 64; dlt <<= 1) {
    const float ov = __shfl_xor(best, dlt, 64);
    const int oi = __shfl_xor(arg, dlt, 64);
    if (ov > best || (ov == best && oi < arg)) { best = ov; arg = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = arg; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < arg)) { best = bv[w]; arg = bi[w]; }
    tok[m] = arg;
  }
}

// ---------------------------------------------------------------- host launchers

#define FLK_DT_SWITCH(dtype, CALL)                        \
  switch (dtype) {                                        \
    case DT_F32: { constexpr int DT = DT_F32; CALL; } break;  \
    case DT_F16: { constexpr int DT = DT_F16; CALL; } break;  \
    default: { constexpr int DT = DT_BF16; CALL; } break;     \
  }

hipError_t embed(int dtype, const void* wte, const void* wpe, const int* tok, const int* pos, float* x, int M, int H,
                 hipStream_t st) {
  if (M <= 0) return hipSuccess;
  FLK_DT_SWITCH(dtype, (embed_kernel<DT><<<M, 256, 0, st>>>(wte, wpe, tok, pos, x, H)));
  return hipGetLastError();
}

hipError_t add_norm(int dtype, bool rms, float* x, const float* part, int S, size_t stride, const void* bias,
                    const void* g, const void* b, void* h, int M, int H, float eps, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  if (rms) {
    FLK_DT_SWITCH(dtype, (add_norm_kernel<DT, 1><<<M, 256, 0, st>>>(x, part, S, stride, bias, g, b, h, H, eps)));
  } else {
    FLK_DT_SWITCH(dtype, (add_norm_kernel<DT, 0><<<M, 256, 0, st>>>(x, part, S, stride, bias, g, b, h, H, eps)));
  }
  return hipGetLastError();
}

hipError_t qkv_post(int dtype, const float* part, int S, size_t stride, const void* bias, const float* rope_cs,
                    const int* slot, const int* pos, void* q, void* kcache, void* vcache, int M, int H, int nh, int d,
                    int Smax, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  FLK_DT_SWITCH(dtype, (qkv_post_kernel<DT><<<dim3(M, nh), d / 2, 0, st>>>(part, S, stride, bias, rope_cs, slot, pos, q,
                                                                           kcache, vcache, H, nh, d, Smax)));
  return hipGetLastError();
}

hipError_t activation(int dtype, bool swiglu, const float* part, int S, size_t stride, const void* bias, void* a, int M,
                      int F, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  const long total = (long)M * F;
  const unsigned grid = (unsigned)((total + 255) / 256);
  if (swiglu) {
    FLK_DT_SWITCH(dtype, (act_kernel<DT, 1><<<grid, 256, 0, st>>>(part, S, stride, bias, a, F, total)));
  } else {
    FLK_DT_SWITCH(dtype, (act_kernel<DT, 0><<<grid, 256, 0, st>>>(part, S, stride, bias, a, F, total)));
  }
  return hipGetLastError();
}

hipError_t logits_argmax(const float* part, int S, size_t stride, float* logits, int* tok, int M, int V, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  argmax_kernel<<<M, 256, 0, st>>>(part, S, stride, logits, tok, V);
  return hipGetLastError();
}

}  // namespace flk
