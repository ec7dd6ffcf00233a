// Host-side launchers of the HIP kernels (internal to the library; the public boundary is include/flover.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace flk {

// ---- weight GEMM
struct GemmPlan {
  int N, K;
  int Npad;   // N rounded up to 64 columns (16-bit dtypes)
  int NT;     // n-tiles (of 16 columns) per wave
  int KB;     // K / 32
  int S;      // split-K slices, a function of (N, K) only
  int kbs;    // k-blocks per slice
  int ldc;    // row length of the partial-sum slices (N rounded up to 4)
  int paired = 0;   // gate|up of a gated MLP in paired 32-column groups (see gemm_plan_gated)
};
inline int part_ld(int N) { return (N + 3) / 4 * 4; }
GemmPlan gemm_plan(int dtype, int N, int K);
// gate|up of a gated MLP with F columns each.  paired = 1: group j of the layout holds gate columns 16j..16j+15 then up
// columns 16j..16j+15 (re-tile gate with n_off = 0 and up with n_off = 16, both with tile_step = 2), K is cut in two
// halves, gemm_gated() serves the fused iterations, and gemm() writes its partial sums in that column order (gate column
// j at (j/16)*32 + j%16, up column j 16 further).  paired = 0 (fp32, or a shape the fused kernels do not take): gemm_plan(2F, K), up after gate.
GemmPlan gemm_plan_gated(int dtype, int F, int K);
size_t gemm_tiled_bytes(int dtype, int N, int K);
// Slicing for a context pass of M rows of one request (a function of the matrix shape and of that request's own row
// count only): same tiling, its own number of K slices, at most max_slices (what the partial-sum buffer holds) and 16.
GemmPlan context_plan(const GemmPlan& p, int dtype, int M, int max_slices);
// Re-tile W [N][K] into `tiled` starting at output column n_off (multiple of 16) of a possibly larger matrix whose
// plan uses NT n-tiles per column group.
// Tile t of W lands at tile position n_off/16 + t * tile_step of the layout.
hipError_t retile(int dtype, const void* W, int N, int K, void* tiled, int n_off, int NT, hipStream_t st,
                  int tile_step = 1);
hipError_t zero_fill(void* p, size_t bytes, hipStream_t st);
// part[s][m][p.ldc] (slice stride in floats) = x[M][K] . W^T over slice s of K.
// xmtt == 0: x is row-major [gemm_rows_read(M)][K]; xmtt = ceil(M/16) (16-bit dtypes only): x is in fragment order
// (tiles of 16 rows x 32 k, [k-block][row tile], see xrow_index) and the buffer holds K/32 * gemm_rows_read(M)/16 tiles.
// ev0 / ev1 (optional, here and below): take the start / end time stamps of the call's first / last dispatch.
hipError_t gemm(int dtype, const void* x, const void* w_tiled, int M, const GemmPlan& p, float* part,
                size_t slice_stride, int xmtt, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// act[M][F] = silu(x . Wgate^T) * (x . Wup^T) rounded to the model dtype, for a paired plan (16-bit dtypes); x and act
// are both row-major (xmtt == 0) or both in fragment order with xmtt row tiles per k-block; reads the rows gemm() reads.
// part / slice_stride as for gemm(): used above gated_fused_rows(p) rows, where the contraction and the activation are
// two launches (same result, bit for bit).
// rows up to which gemm_gated() is one launch for this plan: 128, or 64 for a matrix whose 128-column blocks outnumber the
// compute units (it takes 16-wave blocks, whose hand-over space in LDS ends at four row tiles)
inline int gated_fused_rows(const GemmPlan& p) { return (p.N / 2 / 16 + 3) / 4 > 256 ? 64 : 128; }
hipError_t gemm_gated(int dtype, const void* x, const void* w_tiled, int M, const GemmPlan& p, void* act, float* part,
                      size_t slice_stride, int xmtt, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// rows of x that gemm() may read for M live rows
inline int gemm_rows_read(int M) {
  return M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : M <= 128 ? 128 : (M + 255) / 256 * 256;
}

// ---- row-wise kernels
// tok[m] < 0: the token is tok_prev[-1 - tok[m]] (device-resident choice of the previous iteration).
hipError_t embed(int dtype, const void* wte, const void* wpe, const int* tok, const int* pos, const int* tok_prev,
                 float* x, int M, int H, hipStream_t st);
// `part` is the preceding GEMM's split-K output: S slices, `stride` floats apart, rows of `ldp` floats (ldp % 4 == 0).
// h (and the outputs of activation and of the attention calls below) feed a GEMM: with mtt = ceil(M/16) they are
// written in fragment order (16-bit dtypes; see gemm), with mtt == 0 row-major.
hipError_t add_norm(int dtype, bool rms, float* x, const float* part, int S, size_t stride, int ldp, const void* bias,
                    const void* g, const void* b, void* h, int M, int H, float eps, int mtt, hipStream_t st);
hipError_t qkv_post(int dtype, const float* part, int S, size_t stride, int ldp, const void* bias, const float* rope_cs,
                    const int* slot, const int* pos, void* q, void* kcache, void* vcache, int M, int H, int nh, int d,
                    int Smax, hipStream_t st);
// paired: gate and up columns of `part` interleaved in tiles of 16 (see gemm_plan_gated); gated activation only.
hipError_t activation(int dtype, bool swiglu, const float* part, int S, size_t stride, int ldp, const void* bias, void* a,
                      int M, int F, int mtt, hipStream_t st, bool paired = false, hipEvent_t ev1 = nullptr);
hipError_t logits_argmax(const float* part, int S, size_t stride, int ldp, float* logits, int* tok, int M, int V,
                         hipStream_t st);

// ---- ragged decode attention
struct AttnWork {          // all device pointers
  const int4* items;       // [n_items] (row, chunk, slot of the row, cache rows of the row)
  const int* row_slot;     // [M]
  const int* row_len;      // [M] rows of cache attended to (>= 1)
  float* pml;              // [M][maxch][nh][2]: (m, l) of chunk ch of row r at ((r * maxch + ch) * nh + head)
  float* po;               // [M][maxch][nh][d]
  int n_items;
  int chunk;
  int maxch;               // chunk slots per row in pml / po: at least ceil(longest row / chunk)
  const int4* blocks = nullptr;   // pre-processing passes: (first row, rows <= prefill_rows_per_block, chunk, -)
  int n_blocks = 0;
  int out_mtt = 0;                // layout of the attention output: 0 row-major, else fragment order (see add_norm)
};
constexpr int kPrefillQB = 8;     // query rows one wave serves in a pre-processing pass (fp32 models)
int prefill_rows_per_block(int dtype);   // rows per entry of AttnWork::blocks: 8 for fp32, 32 for the 16-bit (MFMA) kernel
int attn_chunk();   // positions per wave task; fixed for the process, so chunking depends on a request's own length only
// ev0 / ev1 (optional) take the start / end time stamps of the streaming kernel's dispatch (the merge kernel follows).
hipError_t decode_attention(int dtype, int d, const void* q, const void* kc, const void* vc, const AttnWork& w, int M,
                            int nh, int Smax, void* out, hipStream_t st, hipEvent_t ev0 = nullptr,
                            hipEvent_t ev1 = nullptr);

// Attention of a pre-processing pass: rows listed in w.blocks are runs of consecutive positions of one slot.
hipError_t prefill_attention(int dtype, int d, const void* q, const void* kc, const void* vc, const AttnWork& w, int M,
                             int nh, int Smax, void* out, hipStream_t st);

// ---- memory shuffle copy
constexpr int kCompactPiece = 16384;   // bytes per block
hipError_t compact(void* cache, int planes, int C, int nh, size_t slot_bytes, const void* moves_dev, int n_moves,
                   int total_blocks, int piece, hipStream_t st);

}  // namespace flk
