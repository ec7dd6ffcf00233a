// Row-wise kernels of the fused decoder step (Algorithm 2's LayerNorm / GenericActivation calls over
// [buffer + offset, size), plus embedding, rotary + KV append and the greedy choice).
//
// Each consumes the split-K partial sums of the GEMM before it (added in slice order, then bias), so a GEMM's
// epilogue lives in the next launch and nothing depends on how many rows are live.  All are HBM/L2 streaming
// kernels: one block (or wave) per row, coalesced 4-byte-per-lane accesses, fixed reduction trees.
#include "flover_dev.h"
#include "flover_kernels.h"

namespace flk {

// Sum of S split-K slices at 4 consecutive elements, added in slice order (s = 0, 1, 2, ...).  Up to 8 slices (every
// plan of the fused iteration) the code is straight-line for the given count -- one scalar jump on S, which is uniform
// over the grid, then all loads issued before the first addition, so a thread pays the memory latency once; beyond
// that (context passes of short prompts) the loads are predicated one by one.
template <int S>
__device__ __forceinline__ f32x4_t psum4_fixed(const float* __restrict__ p, size_t stride) {
  f32x4_t pv[S];
#pragma unroll
  for (int j = 0; j < S; ++j) pv[j] = ld4(p + (size_t)j * stride);
  f32x4_t v = pv[0];
#pragma unroll
  for (int j = 1; j < S; ++j) v += pv[j];
  return v;
}
__device__ __forceinline__ f32x4_t psum4(const float* __restrict__ part, int S, size_t stride, size_t idx) {
  const float* p = part + idx;
  switch (S) {
    case 1: return psum4_fixed<1>(p, stride);
    case 2: return psum4_fixed<2>(p, stride);
    case 3: return psum4_fixed<3>(p, stride);
    case 4: return psum4_fixed<4>(p, stride);
    case 5: return psum4_fixed<5>(p, stride);
    case 6: return psum4_fixed<6>(p, stride);
    case 7: return psum4_fixed<7>(p, stride);
    case 8: return psum4_fixed<8>(p, stride);
    default: break;
  }
  f32x4_t pv[16];
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if (j < S) pv[j] = ld4(p + (size_t)j * stride);
  f32x4_t v = pv[0];
#pragma unroll
  for (int j = 1; j < 16; ++j)
    if (j < S) v += pv[j];
  for (int s = 16; s < S; ++s) v += ld4(p + (size_t)s * stride);
  return v;
}
// ---------------------------------------------------------------- embedding
// x[m][i] = wte[tok[m]][i] (+ wpe[pos[m]][i])            grid = M, block = 256
// tok[m] < 0 feeds the token the previous iteration chose for its row -1 - tok[m] (still on the device).
template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const void* __restrict__ wte, const void* __restrict__ wpe,
                                                    const int* __restrict__ tok, const int* __restrict__ pos,
                                                    const int* __restrict__ tok_prev, float* __restrict__ x, int H) {
  const int m = blockIdx.x;
  int tk = tok[m];
  if (tk < 0) tk = tok_prev[-1 - tk];
  const size_t t = (size_t)tk * H;
  const size_t p = wpe ? (size_t)pos[m] * H : 0;
  for (int i = threadIdx.x * 4; i < H; i += 1024) {
    f32x4_t v = ldv4<DT>(wte, t + i);
    if (wpe) v += ldv4<DT>(wpe, p + i);
    *(f32x4_t*)(x + (size_t)m * H + i) = v;
  }
}

// ---------------------------------------------------------------- residual add + norm
// x[m] += sum_s part[s][m] + bias   (skipped when part == nullptr), then
// h[m] = LayerNorm(x[m]) * g + b   (RMS == 0)   or   x[m] / rms(x[m]) * g   (RMS == 1), rounded to dtype.
// grid = M, block = 1024, 4 consecutive elements per thread and pass (2 passes cover H <= 8192); H % 4 == 0.
// part rows have length ldp.  All slice loads of a pass are issued before the first addition.
template <int DT, int RMS>
__global__ __launch_bounds__(1024) void add_norm_kernel(float* __restrict__ x, const float* __restrict__ part, int S,
                                                        size_t stride, int ldp, const void* __restrict__ bias,
                                                        const void* __restrict__ g, const void* __restrict__ b,
                                                        void* __restrict__ h, int H, float eps, int mtt) {
  __shared__ float red[16];
  const int m = blockIdx.x;
  constexpr int PER = 2;
  f32x4_t v[PER], gv[PER], bv[PER];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < PER; ++c) {
    const int i = (threadIdx.x + c * 1024) * 4;
    v[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    gv[c] = v[c];
    bv[c] = v[c];
    if (i < H) {
      gv[c] = ldv4<DT>(g, i);                     // issued early: needed only after the reductions
      if (!RMS) bv[c] = ldv4<DT>(b, i);
      f32x4_t t = *(const f32x4_t*)(x + (size_t)m * H + i);
      if (part) {
        f32x4_t a = psum4(part, S, stride, (size_t)m * ldp + i);
        if (bias) a += ldv4<DT>(bias, i);
        t += a;
        *(f32x4_t*)(x + (size_t)m * H + i) = t;
      }
      v[c] = t;
      sum += RMS ? (t[0] * t[0] + t[1] * t[1]) + (t[2] * t[2] + t[3] * t[3]) : (t[0] + t[1]) + (t[2] + t[3]);
    }
  }
  sum = block_sum<16>(sum, red);
  float mean = 0.f, inv;
  if (RMS) {
    inv = 1.0f / sqrtf(sum / (float)H + eps);
  } else {
    mean = sum / (float)H;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < PER; ++c)
      if ((threadIdx.x + c * 1024) * 4 < H) {
        const f32x4_t dlt = v[c] - mean;
        sq += (dlt[0] * dlt[0] + dlt[1] * dlt[1]) + (dlt[2] * dlt[2] + dlt[3] * dlt[3]);
      }
    sq = block_sum<16>(sq, red);
    inv = 1.0f / sqrtf(sq / (float)H + eps);
  }
#pragma unroll
  for (int c = 0; c < PER; ++c) {
    const int i = (threadIdx.x + c * 1024) * 4;
    if (i < H) {
      f32x4_t o = (v[c] - mean) * inv * gv[c];
      if (!RMS) o += bv[c];
      stv4<DT>(h, xrow_index(m, i, H, mtt), o);
    }
  }
}

// ---------------------------------------------------------------- QKV epilogue: bias, rotary, KV append
// part: [S][M][ldp] rows (q | k | v).  For row m (slot, pos) and head hd: q -> qout[m][hd][:] (dtype),
// k, v -> cache[slot][hd][pos][:] (dtype).  Rotary (LLaMA): pairs (i, i + d/2), cos/sin from a table [max_seq][d/2][2].
// grid = (M, 3): blockIdx.y picks q, k or v; block = n_head * d / 8: thread (hd, j) owns elements 4j..4j+3 and their
// partners 4j + d/2 .. of its vector.
template <int DT>
__global__ void qkv_post_kernel(const float* __restrict__ part, int S, size_t stride, int ldp,
                                const void* __restrict__ bias, const float* __restrict__ rope_cs,
                                const int* __restrict__ slot, const int* __restrict__ pos, void* __restrict__ qout,
                                void* __restrict__ kcache, void* __restrict__ vcache, int H, int nh, int d, int Smax) {
  const int m = blockIdx.x, which = blockIdx.y, half = d >> 1, tph = d >> 3;
  const int hd = threadIdx.x / tph, i = (threadIdx.x - hd * tph) * 4;
  const int c0 = which * H + hd * d + i, c1 = c0 + half;
  const float* p0 = part + (size_t)m * ldp + c0;
  const float* p1 = part + (size_t)m * ldp + c1;
  // Load order: the row's position first, then every split-K slice (their addresses need nothing else), and only then
  // the rotary table row, whose address waits for the position -- so that wait overlaps the slices' flight.
  const int p = pos[m];
  const bool rot = rope_cs && which < 2;
  f32x4_t a0 = ld4(p0), a1 = ld4(p1);
  f32x4_t u0[8], u1[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)                             // slices 1..8; S is uniform over the grid: scalar branches
    if (1 + j < S) {
      u0[j] = ld4(p0 + (size_t)(1 + j) * stride);
      u1[j] = ld4(p1 + (size_t)(1 + j) * stride);
    }
  __builtin_amdgcn_sched_barrier(0);
  f32x4_t t0 = {1.f, 0.f, 1.f, 0.f}, t1 = t0;          // (cos, sin) of 4 consecutive pairs
  if (rot) {
    const float* t = rope_cs + ((size_t)p * half + i) * 2;
    t0 = ld4(t);
    t1 = ld4(t + 4);
  }
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (1 + j < S) { a0 += u0[j]; a1 += u1[j]; }
  for (int s0 = 9; s0 < S; s0 += 8) {                     // more than 9 slices: context passes of short prompts only
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const size_t o = (size_t)min(s0 + j, S - 1) * stride;
      u0[j] = ld4(p0 + o);
      u1[j] = ld4(p1 + o);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < S) { a0 += u0[j]; a1 += u1[j]; }
  }
  if (bias) { a0 += ldv4<DT>(bias, c0); a1 += ldv4<DT>(bias, c1); }
  if (rot) {
    const f32x4_t cs = {t0[0], t0[2], t1[0], t1[2]}, sn = {t0[1], t0[3], t1[1], t1[3]};
    rope_rotate(a0, a1, cs, sn);
  }
  if (which == 0) {
    stv4<DT>(qout, (size_t)m * H + hd * d + i, a0);
    stv4<DT>(qout, (size_t)m * H + hd * d + i + half, a1);
  } else {
    void* cache = which == 1 ? kcache : vcache;
    const size_t kv = (((size_t)slot[m] * nh + hd) * Smax + p) * d;
    stv4<DT>(cache, kv + i, a0);
    stv4<DT>(cache, kv + i + half, a1);
  }
}

// ---------------------------------------------------------------- MLP activation
// GPT:   a[m][j] = gelu_tanh(sum_s part[s][m][j] + b1[j])                            part row length ldp >= F
// LLaMA: a[m][j] = silu(gate) * up, gate = part[..][m][j], up = part[..][m][F + j]   part row length ldp >= 2F
// 4 consecutive j per thread; F % 4 == 0.
template <int DT, int SWIGLU>
__global__ __launch_bounds__(256) void act_kernel(const float* __restrict__ part, int S, size_t stride, int ldp,
                                                  const void* __restrict__ bias, void* __restrict__ a, int F, long total4,
                                                  int mtt, int paired) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total4) return;
  const int F4 = F >> 2;
  const long m = idx / F4;
  const int j = (int)(idx - m * F4) * 4;
  f32x4_t o;
  if (SWIGLU) {
    // gate column j and up column j: side by side halves of the row, or (paired) tiles of 16 interleaved
    const size_t gj = paired ? (size_t)(j >> 4) * 32 + (j & 15) : (size_t)j, uj = paired ? gj + 16 : (size_t)F + j;
    const f32x4_t g = psum4(part, S, stride, (size_t)m * ldp + gj);
    const f32x4_t u = psum4(part, S, stride, (size_t)m * ldp + uj);
    o = act_swiglu(g, u);
  } else {
    const f32x4_t t = psum4(part, S, stride, (size_t)m * ldp + j) + ldv4<DT>(bias, j);
    o = act_gelu(t);
  }
  stv4<DT>(a, xrow_index((int)m, j, F, mtt), o);
}

// ---------------------------------------------------------------- logits + greedy token
// logits[m][j] = sum_s part[s][m][j] (fp32, optionally stored, row length V); tok[m] = argmax_j, lowest j on ties.
// grid = M, block = 1024; part rows have length ldp (multiple of 4, >= V).
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ part, int S, size_t stride, int ldp,
                                                      float* __restrict__ logits, int* __restrict__ tok, int V) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const int m = blockIdx.x;
  float best = -INFINITY;
  int arg = 0x7fffffff;
  for (int j0 = threadIdx.x * 4; j0 < V; j0 += 4 * 4096) {      // four strides at a time: their loads go out together
    f32x4_t v[4];
    if (S == 2) {          // the output projection's usual slicing: straight-line, all eight loads in flight at once
      f32x4_t w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float* p = part + (size_t)m * ldp + min(j0 + u * 4096, ldp - 4);
        v[u] = ld4(p);
        w[u] = ld4(p + stride);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] += w[u];
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = psum4(part, S, stride, (size_t)m * ldp + min(j0 + u * 4096, ldp - 4));
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 4096;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < V) {
          if (logits) logits[(size_t)m * V + j + e] = v[u][e];
          if (v[u][e] > best) { best = v[u][e]; arg = j + e; }      // ascending j: the first maximum stays
        }
    }
  }
#pragma unroll
  for (int dlt = 1; dlt < 64; dlt <<= 1) {
    const float ov = __shfl_xor(best, dlt, 64);
    const int oi = __shfl_xor(arg, dlt, 64);
    if (ov > best || (ov == best && oi < arg)) { best = ov; arg = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = arg; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < arg)) { best = bv[w]; arg = bi[w]; }
    tok[m] = (arg == 0x7fffffff) ? 0 : arg;       // a row of NaNs has no maximum
  }
}

// ---------------------------------------------------------------- host launchers

#define FLK_DT_SWITCH(dtype, CALL)                        \
  switch (dtype) {                                        \
    case DT_F32: { constexpr int DT = DT_F32; CALL; } break;  \
    case DT_F16: { constexpr int DT = DT_F16; CALL; } break;  \
    default: { constexpr int DT = DT_BF16; CALL; } break;     \
  }

hipError_t embed(int dtype, const void* wte, const void* wpe, const int* tok, const int* pos, const int* tok_prev,
                 float* x, int M, int H, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  FLK_DT_SWITCH(dtype, (embed_kernel<DT><<<M, 256, 0, st>>>(wte, wpe, tok, pos, tok_prev, x, H)));
  return hipGetLastError();
}

hipError_t add_norm(int dtype, bool rms, float* x, const float* part, int S, size_t stride, int ldp, const void* bias,
                    const void* g, const void* b, void* h, int M, int H, float eps, int mtt, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  if (rms) {
    FLK_DT_SWITCH(dtype, (add_norm_kernel<DT, 1><<<M, 1024, 0, st>>>(x, part, S, stride, ldp, bias, g, b, h, H, eps, mtt)));
  } else {
    FLK_DT_SWITCH(dtype, (add_norm_kernel<DT, 0><<<M, 1024, 0, st>>>(x, part, S, stride, ldp, bias, g, b, h, H, eps, mtt)));
  }
  return hipGetLastError();
}

hipError_t qkv_post(int dtype, const float* part, int S, size_t stride, int ldp, const void* bias, const float* rope_cs,
                    const int* slot, const int* pos, void* q, void* kcache, void* vcache, int M, int H, int nh, int d,
                    int Smax, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  FLK_DT_SWITCH(dtype, (qkv_post_kernel<DT><<<dim3(M, 3), nh * d / 8, 0, st>>>(part, S, stride, ldp, bias, rope_cs, slot, pos, q,
                                                                           kcache, vcache, H, nh, d, Smax)));
  return hipGetLastError();
}

hipError_t activation(int dtype, bool swiglu, const float* part, int S, size_t stride, int ldp, const void* bias, void* a,
                      int M, int F, int mtt, hipStream_t st, bool paired, hipEvent_t ev1) {
  if (M <= 0) return hipSuccess;
  if (paired && !swiglu) return hipErrorInvalidValue;
  const long total = (long)M * (F / 4);
  const unsigned grid = (unsigned)((total + 255) / 256);
  if (swiglu) {
    FLK_DT_SWITCH(dtype, (launch_timed(act_kernel<DT, 1>, dim3(grid), dim3(256), st, nullptr, ev1, part, S, stride, ldp, bias, a, F,
                                       total, mtt, paired ? 1 : 0)));
  } else {
    FLK_DT_SWITCH(dtype, (act_kernel<DT, 0><<<grid, 256, 0, st>>>(part, S, stride, ldp, bias, a, F, total, mtt, 0)));
  }
  return hipGetLastError();
}

hipError_t logits_argmax(const float* part, int S, size_t stride, int ldp, float* logits, int* tok, int M, int V,
                         hipStream_t st) {
  if (M <= 0) return hipSuccess;
  argmax_kernel<<<M, 1024, 0, st>>>(part, S, stride, ldp, logits, tok, V);
  return hipGetLastError();
}

}  // namespace flk
