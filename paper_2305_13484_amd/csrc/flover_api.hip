// C ABI of the fused decoder step: Buffer Manager (arena layout), Inference Scheduler (queues, slot window,
// Algorithm 3) and the per-iteration launch sequence.  See include/flover.h for the contract of every call.
//
// Paper mapping: flover_init = Launcher + Buffer Manager + scheduler start (Section V-A); flover_add_request =
// body of Algorithm 1 (Section V-B); flover_step = Algorithm 2 up to FindAndEvict's detection (Section V-C);
// flover_reorder_evict = eviction, Algorithm 3 and the memory shuffle (Section V-D).
#include "../../include/flover.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <deque>
#include <mutex>
#include <string>
#include <vector>

#include "flover_kernels.h"

namespace {

thread_local std::string g_err;   // last error of calls that have no context, per calling thread

struct Slot {
  int state = FLOVER_SLOT_EMPTY;
  uint64_t req_id = 0;
  int len = 0;          // cached KV rows = position of the next token fed
  int next_token = 0;
  int generated = 0;
  int max_new = 0;
  bool pending = false;   // context cache still being written on the pre-processing stream (event prep_ev[ev])
  int ev = -1;
  int dev_row = -1;       // >= 0: the next token is row dev_row of submitted iteration dev_step, not yet on the host
  int64_t dev_step = -1;
};
struct Waiting {
  uint64_t req_id;
  std::vector<int32_t> prompt;
  int max_new;
};
struct LayerW {
  void *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
};
struct Row {
  int slot, tok, pos;
};

// One execution lane: a stream with the row buffers and staging a pass of the decoder needs.  The fused iteration
// owns one; with asynchronous pre-processing the context decoder owns a second one (Section V-B: pre-processing runs
// beside the inference stream), otherwise both names refer to the same lane.
constexpr int kStageRing = 4;
struct Lane {
  hipStream_t st = nullptr;
  float* x = nullptr;
  void *h = nullptr, *q = nullptr, *att = nullptr, *act = nullptr;
  float* part = nullptr;
  int* tok_out = nullptr;
  int* d_stage = nullptr;   // tok | pos | slot | len | (2 host-only arrays) | items(4x) | context-pass blocks(4x)
  float *pml = nullptr, *po = nullptr;
  // pinned host staging; a ring so that passes can be queued without waiting for the previous copy
  int* h_stage[kStageRing] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t staged[kStageRing] = {nullptr, nullptr, nullptr, nullptr};   // copy of h_stage[i] has been consumed
  bool staged_busy[kStageRing] = {false, false, false, false};
  int ring = 1, next = 0;
  int tok_next = 0;         // ring of token buffers: advanced only by passes that return tokens
  int* h_tok = nullptr;     // [kStageRing][rows_cap]
  hipEvent_t done[kStageRing] = {nullptr, nullptr, nullptr, nullptr};     // submitted iteration's tokens are in h_tok
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
int esize(int dtype) { return dtype == FLOVER_F32 ? 4 : 2; }

// Bump allocator over the arena; with base == nullptr it only measures.
struct Bump {
  char* base;
  size_t off = 0;
  void* take(size_t bytes) {
    off = align_up(off, 256);
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

}  // namespace

struct flover_ctx {
  flover_config cfg;
  hipStream_t st;
  std::string err;
  std::mutex err_mu;                 // the two lanes may fail at the same time (see fail())
  // weights in the arena
  std::vector<LayerW> lw;
  std::vector<bool> layer_loaded;
  int layers_loaded = 0;
  void *wte, *wpe, *lnf_g, *lnf_b, *wlm;
  float* rope_cs;
  flk::GemmPlan p_qkv, p_o, p_1, p_2, p_lm;
  // KV cache [L][2][C][nh][S][d]
  char* kv;
  size_t kv_bytes, slot_bytes, plane_bytes;
  // per-pass buffers
  int rows_cap, max_items;
  Lane step_lane;
  // asynchronous pre-processing: two lanes (stream + row buffers each), taken in turn by arriving requests, so that the
  // context passes of two requests run side by side -- a pass's GEMM launches leave a quarter to a third of the compute
  // units idle (172-192 blocks on 256), which the other request's launches fill
  static constexpr int kPrepLanes = 2;   // three lanes: 1.4 % less pre-processing time on the 7B stream, four: more
  Lane prep_lanes[kPrepLanes];
  int prep_next = 0;
  int4* d_moves;
  size_t stage_ints;
  size_t part_floats = 0;      // capacity of a lane's split-K partial-sum buffer
  size_t act_off = 0;          // arena offset where the row buffers start
  struct InFlight {                  // an iteration submitted with flover_step_submit and not collected yet
    int64_t id;
    int ring, n;
    size_t ev_end;                   // profiling pairs recorded up to here belong to this or earlier iterations
    std::vector<uint64_t> req_id;
    std::vector<int32_t> slot;
    std::vector<uint8_t> fin;
  };
  std::deque<InFlight> inflight;
  int64_t next_step_id = 0;
  int4* h_moves_ring[kStageRing] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t moves_ev[kStageRing] = {nullptr, nullptr, nullptr, nullptr};
  bool moves_busy[kStageRing] = {false, false, false, false};
  int moves_next = 0;
  hipEvent_t compact_ev = nullptr;   // end of the most recent shuffle copy on the iteration's stream
  bool compact_pending = false;      // ... recorded and not yet known to be complete
  std::vector<hipEvent_t> prep_ev;   // one per slot: the slot's context cache is complete
  mutable std::mutex mu;             // scheduler state; see flover.h for which calls may run concurrently
  // scheduler
  std::vector<Slot> slots;
  std::deque<Waiting> reque;   // Q_R
  int lo = 0, hi = 0;          // window [lo,hi): buffer offset and size in slots
  int last_launches = 0;
  int launches = 0;
  // optional timing of the kernels with HIP events on the library's stream
  int profile = 0;                         // 0 off, 1 sampled launches (see flover_set_profile), 2 every launch of every kind
  int64_t prof_iter = 0;                   // fused iterations enqueued since the level was set (level 1 samples by it)
  bool in_step = false;                    // only the fused iteration is timed, not pre-processing
  bool prof_now = false;                   // the pass being enqueued on the iteration's lane is a timed one
  std::vector<hipEvent_t> ev;              // pool of pairs
  std::deque<int> ev_kind;                 // kind of each recorded pair not yet added up
  std::deque<int64_t> ev_bytes;            // its algorithmic bytes
  size_t ev_base = 0;                      // number of the pair at the front
  double prof_ms[FLOVER_PROF_KINDS] = {0};
  int64_t prof_launches[FLOVER_PROF_KINDS] = {0};
  int64_t prof_bytes[FLOVER_PROF_KINDS] = {0};
};

namespace {

// Records the message of a failing call.  A context's message has its own lock: with asynchronous pre-processing the
// thread in flover_add_request and the thread in flover_step can both fail while the scheduler lock is released.
int fail(flover_ctx* c, int code, const std::string& msg) {
  if (c) {
    std::lock_guard<std::mutex> lock(c->err_mu);
    c->err = msg;
  } else {
    g_err = msg;
  }
  return code;
}
#define HIPCHK(ctx, expr)                                                                        \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess)                                                                        \
      return fail(ctx, FLOVER_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));          \
  } while (0)

int check_shape(const flover_config* c, std::string* why) {
  auto bad = [&](const char* m) { *why = m; return FLOVER_E_INVAL; };
  if (!c) return bad("null config");
  if (c->arch != FLOVER_ARCH_GPT && c->arch != FLOVER_ARCH_LLAMA) return bad("arch");
  if (c->dtype < FLOVER_F32 || c->dtype > FLOVER_BF16) return bad("dtype");
  if (c->n_layer < 1 || c->hidden < 32 || c->n_head < 4 || c->ffn < 32 || c->vocab < 2) return bad("shape");
  if (c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 64 or 128");
  if (c->hidden != c->n_head * c->head_dim) return bad("hidden != n_head * head_dim");
  if (c->n_head % 4) return bad("n_head must be a multiple of 4");
  if (c->hidden % 32 || c->ffn % 32) return bad("hidden and ffn must be multiples of 32");
  if (c->hidden > 8192) return bad("hidden > 8192");
  if (c->max_seq < 2 || c->max_concurrency < 1) return bad("max_seq / max_concurrency");
  return FLOVER_OK;
}

// Lays the arena out; fills ctx pointers when base != nullptr.  Returns bytes used.
size_t layout(flover_ctx* c, char* base) {
  const flover_config& f = c->cfg;
  const int e = esize(f.dtype), L = f.n_layer, H = f.hidden, F = f.ffn, V = f.vocab, C = f.max_concurrency, S = f.max_seq;
  const bool gpt = f.arch == FLOVER_ARCH_GPT;
  Bump b{base};
  c->p_qkv = flk::gemm_plan(f.dtype, 3 * H, H);
  c->p_o = flk::gemm_plan(f.dtype, H, H);
  c->p_1 = gpt ? flk::gemm_plan(f.dtype, F, H) : flk::gemm_plan_gated(f.dtype, F, H);
  c->p_2 = flk::gemm_plan(f.dtype, H, F);
  c->p_lm = flk::gemm_plan(f.dtype, V, H);
  c->lw.resize(L);
  for (int l = 0; l < L; ++l) {
    LayerW& w = c->lw[l];
    w.ln1_g = b.take((size_t)H * e);
    w.ln1_b = gpt ? b.take((size_t)H * e) : nullptr;
    w.wqkv = b.take(flk::gemm_tiled_bytes(f.dtype, 3 * H, H));
    w.bqkv = gpt ? b.take((size_t)3 * H * e) : nullptr;
    w.wo = b.take(flk::gemm_tiled_bytes(f.dtype, H, H));
    w.bo = gpt ? b.take((size_t)H * e) : nullptr;
    w.ln2_g = b.take((size_t)H * e);
    w.ln2_b = gpt ? b.take((size_t)H * e) : nullptr;
    w.w1 = b.take(flk::gemm_tiled_bytes(f.dtype, gpt ? F : 2 * F, H));
    w.b1 = gpt ? b.take((size_t)F * e) : nullptr;
    w.w2 = b.take(flk::gemm_tiled_bytes(f.dtype, H, F));
    w.b2 = gpt ? b.take((size_t)H * e) : nullptr;
  }
  c->wte = b.take((size_t)V * H * e);
  c->wpe = gpt ? b.take((size_t)S * H * e) : nullptr;
  c->lnf_g = b.take((size_t)H * e);
  c->lnf_b = gpt ? b.take((size_t)H * e) : nullptr;
  c->wlm = b.take(flk::gemm_tiled_bytes(f.dtype, V, H));
  c->rope_cs = gpt ? nullptr : (float*)b.take((size_t)S * (f.head_dim / 2) * 2 * sizeof(float));
  c->slot_bytes = (size_t)f.n_head * S * f.head_dim * e;
  c->plane_bytes = c->slot_bytes * C;
  c->kv_bytes = c->plane_bytes * 2 * L;
  c->kv = (char*)b.take(c->kv_bytes);
  const int R = (std::max(C, 1024) + 255) / 256 * 256;   // rows per pass: live rows of an iteration, or a chunk of a prompt
  c->rows_cap = R;
  const int chunks = (S + flk::attn_chunk() - 1) / flk::attn_chunk();
  c->max_items = R * chunks;
  size_t pw = 0;
  for (const flk::GemmPlan* p : {&c->p_qkv, &c->p_o, &c->p_1, &c->p_2, &c->p_lm}) pw = std::max(pw, (size_t)p->S * p->ldc);
  c->stage_ints = (size_t)6 * R + (size_t)8 * c->max_items;   // row arrays, (row, chunk, slot, len) items, context-pass blocks
  c->act_off = align_up(b.off, 256);
  std::vector<Lane*> lanes{&c->step_lane};
  for (Lane& pl : c->prep_lanes) lanes.push_back(&pl);
  for (Lane* ln : lanes) {
    if (ln != &c->step_lane && !f.async_preprocess) break;
    ln->x = (float*)b.take((size_t)R * H * 4);
    ln->h = b.take((size_t)R * H * e);
    ln->q = b.take((size_t)R * H * e);
    ln->att = b.take((size_t)R * H * e);
    ln->act = b.take((size_t)R * F * e);
    ln->part = (float*)b.take(pw * R * 4);
    c->part_floats = pw * R;
    ln->tok_out = (int*)b.take((size_t)R * 4);
    ln->d_stage = (int*)b.take(c->stage_ints * 4);
    ln->pml = (float*)b.take((size_t)c->max_items * f.n_head * 2 * 4);
    ln->po = (float*)b.take((size_t)c->max_items * f.n_head * f.head_dim * 4);
  }
  c->d_moves = (int4*)b.take((size_t)C * sizeof(int4));
  return align_up(b.off, 256);
}

// AssignMemId: the slot adjacent to the live region, or -1 if none is free.
int place(flover_ctx* c) {
  if (c->lo == c->hi) {
    c->lo = 0;
    c->hi = 1;
    return 0;
  }
  if (c->hi < c->cfg.max_concurrency) return c->hi++;
  if (c->lo > 0) return --c->lo;
  return -1;
}

// Event pair for a profiled launch; returns its index in the event pool or -1 when profiling of `kind` is off.
// Pairs are numbered in recording order; pair g lives in pool entry g % kEvPool until it has been added up.
constexpr size_t kEvPool = 4096;
int prof_begin(flover_ctx* c, int kind, int64_t bytes) {
  if (c->profile == 0) return -1;
  if (!c->in_step && kind != FLOVER_PROF_COMPACT) return -1;
  if (c->ev_kind.size() >= kEvPool) return -1;            // every pool entry is waiting to be added up
  const size_t p = (c->ev_base + c->ev_kind.size()) % kEvPool;
  while (c->ev.size() < 2 * (p + 1)) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return -1;
    c->ev.push_back(e);
  }
  c->ev_kind.push_back(kind);
  c->ev_bytes.push_back(bytes);
  return (int)p;
}
// Adds up the recorded pairs numbered below `upto` -- all of them when the stream has been synchronised, those of
// the oldest submitted iteration when that one is collected.
void prof_collect(flover_ctx* c, size_t upto = (size_t)-1) {
  while (c->ev_base < upto && !c->ev_kind.empty()) {
    const size_t p = c->ev_base % kEvPool;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev[2 * p], c->ev[2 * p + 1]) == hipSuccess) {
      c->prof_ms[c->ev_kind.front()] += ms;
      c->prof_launches[c->ev_kind.front()] += 1;
      c->prof_bytes[c->ev_kind.front()] += c->ev_bytes.front();
    }
    c->ev_kind.pop_front();
    c->ev_bytes.pop_front();
    c->ev_base += 1;
  }
}
// `sampled`: this launch is one of those level 1 times (level 2 times every launch).
// gated_out: the plan is a paired gate|up plan and the launch is the fused one that writes the activation there.
hipError_t timed_gemm(flover_ctx* c, Lane& ln, int kind, const void* x, const void* w, int n, const flk::GemmPlan& p,
                      size_t ss, int mtt, bool sampled, void* gated_out = nullptr) {
  const int64_t bytes = (int64_t)flk::gemm_tiled_bytes(c->cfg.dtype, p.N, p.K);
  const int pi = (&ln == &c->step_lane && c->prof_now && (sampled || c->profile >= 2)) ? prof_begin(c, kind, bytes) : -1;
  hipEvent_t ev0 = pi >= 0 ? c->ev[2 * pi] : nullptr, ev1 = pi >= 0 ? c->ev[2 * pi + 1] : nullptr;
  return gated_out ? flk::gemm_gated(c->cfg.dtype, x, w, n, p, gated_out, ln.part, ss, mtt, ln.st, ev0, ev1)
                   : flk::gemm(c->cfg.dtype, x, w, n, p, ln.part, ss, mtt, ln.st, ev0, ev1);
}

// One pass of the decoder over n rows on lane `ln`: a single launch per operation covers all of them.
// With want_tokens the final norm, output projection and argmax run and ln.h_tok (host) holds the choices.
// With wait the call returns after the lane's stream has drained; otherwise the pass is only enqueued.
int run_rows(flover_ctx* c, Lane& ln, const Row* rows, int n, bool want_tokens, float* logits_out, bool context_pass,
             bool wait, int* ring_used = nullptr) {
  const flover_config& f = c->cfg;
  const int H = f.hidden, F = f.ffn, V = f.vocab, nh = f.n_head, d = f.head_dim, L = f.n_layer, R = c->rows_cap;
  const bool gpt = f.arch == FLOVER_ARCH_GPT;
  hipStream_t st = ln.st;
  if (n <= 0) return FLOVER_OK;
  // row descriptors and the attention work list, one host-to-device copy from the next staging buffer of the ring
  const int ri = ln.next;
  ln.next = (ln.next + 1) % ln.ring;
  if (ln.staged_busy[ri]) {
    HIPCHK(c, hipEventSynchronize(ln.staged[ri]));
    ln.staged_busy[ri] = false;
  }
  int* hs = ln.h_stage[ri];
  int *tok = hs, *pos = hs + R, *slot = hs + 2 * R, *len = hs + 3 * R, *nchunk = hs + 5 * R;   // nchunk: host use only
  int* items = hs + 6 * R;
  int n_items = 0;
  int64_t attn_bytes = 0;   // K and V rows [0,len) of every row, all heads: what one attention launch has to read
  for (int i = 0; i < n; ++i) {
    attn_bytes += (int64_t)(rows[i].pos + 1) * 2 * H * esize(f.dtype);
    tok[i] = rows[i].tok;
    pos[i] = rows[i].pos;
    slot[i] = rows[i].slot;
    len[i] = rows[i].pos + 1;
    const int nc = (len[i] + flk::attn_chunk() - 1) / flk::attn_chunk();
    nchunk[i] = nc;
    for (int ch = 0; ch < nc; ++ch) {
      items[4 * n_items] = i;
      items[4 * n_items + 1] = ch;
      items[4 * n_items + 2] = rows[i].slot;
      items[4 * n_items + 3] = len[i];
      ++n_items;
    }
  }
  // context pass: runs of consecutive positions of one slot are served several query rows per wave
  const int qb = flk::prefill_rows_per_block(f.dtype);
  int n_blocks = 0;
  int* blk = items + 4 * n_items;
  if (context_pass) {
    for (int i = 0; i < n;) {
      int nr = 1;
      while (nr < qb && i + nr < n && rows[i + nr].slot == rows[i].slot && rows[i + nr].pos == rows[i].pos + nr)
        ++nr;
      for (int ch = 0; ch < nchunk[i + nr - 1]; ++ch) {
        blk[4 * n_blocks] = i;
        blk[4 * n_blocks + 1] = nr;
        blk[4 * n_blocks + 2] = ch;
        blk[4 * n_blocks + 3] = 0;
        ++n_blocks;
      }
      i += nr;
    }
  }
  HIPCHK(c, hipMemcpyAsync(ln.d_stage, hs, ((size_t)6 * R + (size_t)4 * n_items + (size_t)4 * n_blocks) * 4,
                           hipMemcpyHostToDevice, st));
  if (!wait) {
    HIPCHK(c, hipEventRecord(ln.staged[ri], st));
    ln.staged_busy[ri] = true;
  }
  int* ds = ln.d_stage;
  const int *d_tok = ds, *d_pos = ds + R, *d_slot = ds + 2 * R, *d_len = ds + 3 * R;
  flk::AttnWork aw{(const int4*)(ds + 6 * R), d_slot, d_len, ln.pml, ln.po, n_items, flk::attn_chunk(),
                   (f.max_seq + flk::attn_chunk() - 1) / flk::attn_chunk()};
  aw.blocks = (const int4*)(ds + 6 * R + 4 * n_items);
  aw.n_blocks = n_blocks;
  // what feeds a GEMM (norm output, attention output, MLP activation) is written in the order the GEMM's MFMA reads
  // it: 16-bit models only, tiles of 16 rows, mtt of them per k-block
  const int mtt = f.dtype == FLOVER_F32 ? 0 : (n + 15) / 16;
  aw.out_mtt = mtt;
  const bool prof = &ln == &c->step_lane && (wait || want_tokens);
  if (&ln == &c->step_lane) c->prof_now = prof;
  // level 1 keeps the timed launches few: the attention launch of one layer in eight, and on every fourth iteration the
  // four GEMMs of the middle layer and the output projection (a timed dispatch costs about as much as a small kernel)
  const bool gemm_iter = prof && !context_pass && (c->prof_iter++ & 3) == 0;

  int launches = 0;
  // K slicing: the iteration's is fixed by the matrix shape; a context pass holds rows of one request only and may
  // slice by that request's row count as well (still independent of what else is in flight)
  auto ctx_plan = [&](const flk::GemmPlan& p) {
    return flk::context_plan(p, f.dtype, n, (int)std::min<size_t>(16, c->part_floats / ((size_t)n * p.ldc)));
  };
  const flk::GemmPlan p_qkv = context_pass ? ctx_plan(c->p_qkv) : c->p_qkv;
  const flk::GemmPlan p_o = context_pass ? ctx_plan(c->p_o) : c->p_o;
  const flk::GemmPlan p_1 = context_pass ? ctx_plan(c->p_1) : c->p_1;
  const flk::GemmPlan p_2 = context_pass ? ctx_plan(c->p_2) : c->p_2;
  const size_t ss_qkv = (size_t)n * p_qkv.ldc, ss_h = (size_t)n * p_o.ldc, ss_1 = (size_t)n * p_1.ldc,
               ss_v = (size_t)n * c->p_lm.ldc;
  HIPCHK(c, flk::embed(f.dtype, c->wte, c->wpe, d_tok, d_pos, ln.tok_out, ln.x, n, H, st));
  ++launches;
  for (int l = 0; l < L; ++l) {
    const LayerW& w = c->lw[l];
    const bool first = l == 0;
    HIPCHK(c, flk::add_norm(f.dtype, !gpt, ln.x, first ? nullptr : ln.part, p_2.S, ss_h, p_2.ldc,
                            first ? nullptr : c->lw[l - 1].b2,
                            w.ln1_g, w.ln1_b, ln.h, n, H, f.norm_eps, mtt, st));
    char* kl = c->kv + (size_t)(2 * l) * c->plane_bytes;
    char* vl = kl + c->plane_bytes;
    const bool gs = gemm_iter && l == L / 2;
    HIPCHK(c, timed_gemm(c, ln, FLOVER_PROF_GEMM_QKV, ln.h, w.wqkv, n, p_qkv, ss_qkv, mtt, gs));
    HIPCHK(c, flk::qkv_post(f.dtype, ln.part, p_qkv.S, ss_qkv, p_qkv.ldc, w.bqkv, c->rope_cs, d_slot, d_pos, ln.q, kl, vl, n, H, nh,
                            d, f.max_seq, st));
    if (context_pass && l == L - 1) {
      launches += 3;
      break;   // the pass exists to fill the cache: the last layer's K and V rows are written, nothing reads the rest
    }
    if (context_pass) {
      HIPCHK(c, flk::prefill_attention(f.dtype, d, ln.q, kl, vl, aw, n, nh, f.max_seq, ln.att, st));
    } else {
      // level 1 times the attention launch of one layer in eight: a timed dispatch costs about as much as a small
      // kernel, and the layers' launches are alike
      const int pi = (prof && (c->profile >= 2 || l % 8 == 0)) ? prof_begin(c, FLOVER_PROF_ATTENTION, attn_bytes) : -1;
      HIPCHK(c, flk::decode_attention(f.dtype, d, ln.q, kl, vl, aw, n, nh, f.max_seq, ln.att, st,
                                      pi >= 0 ? c->ev[2 * pi] : nullptr, pi >= 0 ? c->ev[2 * pi + 1] : nullptr));
    }
    HIPCHK(c, timed_gemm(c, ln, FLOVER_PROF_GEMM_OUT, ln.att, w.wo, n, p_o, ss_h, mtt, gs));
    HIPCHK(c, flk::add_norm(f.dtype, !gpt, ln.x, ln.part, p_o.S, ss_h, p_o.ldc, w.bo, w.ln2_g, w.ln2_b, ln.h, n, H, f.norm_eps, mtt, st));
    if (p_1.paired) {
      // gated 16-bit model: the activation is the epilogue of the gate|up contraction wherever that is one launch
      HIPCHK(c, timed_gemm(c, ln, FLOVER_PROF_GEMM_FF1, ln.h, w.w1, n, p_1, ss_1, mtt, gs, ln.act));
      if (!context_pass && n <= flk::gated_fused_rows(p_1)) launches -= 1;
    } else {
      HIPCHK(c, timed_gemm(c, ln, FLOVER_PROF_GEMM_FF1, ln.h, w.w1, n, p_1, ss_1, mtt, gs));
      HIPCHK(c, flk::activation(f.dtype, !gpt, ln.part, p_1.S, ss_1, p_1.ldc, w.b1, ln.act, n, F, mtt, st, p_1.paired));
    }
    HIPCHK(c, timed_gemm(c, ln, FLOVER_PROF_GEMM_FF2, ln.act, w.w2, n, p_2, ss_h, mtt, gs));
    launches += 10;
  }
  if (want_tokens) {
    HIPCHK(c, flk::add_norm(f.dtype, !gpt, ln.x, ln.part, c->p_2.S, ss_h, c->p_2.ldc, c->lw[L - 1].b2, c->lnf_g, c->lnf_b, ln.h, n, H,
                            f.norm_eps, mtt, st));
    HIPCHK(c, timed_gemm(c, ln, FLOVER_PROF_GEMM_LM, ln.h, c->wlm, n, c->p_lm, ss_v, mtt, gemm_iter));
    HIPCHK(c, flk::logits_argmax(ln.part, c->p_lm.S, ss_v, c->p_lm.ldc, logits_out, ln.tok_out, n, V, st));
    const int ti = ln.tok_next;       // at most kStageRing - 1 iterations are outstanding, so this entry is free
    ln.tok_next = (ln.tok_next + 1) % kStageRing;
    if (ring_used) *ring_used = ti;
    HIPCHK(c, hipMemcpyAsync(ln.h_tok + (size_t)ti * R, ln.tok_out, (size_t)n * 4, hipMemcpyDeviceToHost, st));
    if (!wait) HIPCHK(c, hipEventRecord(ln.done[ti], st));
    launches += 3;
  }
  if (wait) {
    HIPCHK(c, hipStreamSynchronize(st));
    if (prof) prof_collect(c);
  }
  if (&ln == &c->step_lane) c->launches += launches;
  return FLOVER_OK;
}

// Pre-processing (Section V-B): the context decoder caches K/V of prompt positions 0..P-2 in the assigned slot.
// Synchronous mode: returns when the cache is complete.  Asynchronous mode: the passes are enqueued on the
// pre-processing lane and the slot's event marks their end; the request joins the first iteration that finds it done.
int preprocess(flover_ctx* c, int slot, const Waiting& r) {
  Slot& s = c->slots[slot];
  s.state = FLOVER_SLOT_READY;
  s.req_id = r.req_id;
  s.generated = 0;
  s.max_new = r.max_new;
  s.pending = false;
  s.ev = -1;
  s.dev_row = -1;
  const bool async = c->cfg.async_preprocess != 0;
  Lane& ln = async ? c->prep_lanes[c->prep_next++ % flover_ctx::kPrepLanes] : c->step_lane;
  const int P = (int)r.prompt.size();
  if (async && !c->inflight.empty())   // a submitted iteration may still read the slot's previous tenant
    HIPCHK(c, hipStreamWaitEvent(ln.st, c->step_lane.done[c->inflight.back().ring], 0));
  // ... and so may a shuffle copy enqueued after that iteration: the slot handed out here is often the one a move has
  // just vacated, and with iterations outstanding flover_reorder_evict does not wait for its copy
  if (async && c->compact_pending) HIPCHK(c, hipStreamWaitEvent(ln.st, c->compact_ev, 0));
  // ... and so may the context pass of a previous tenant that was marked finished before it ever joined: with two
  // pre-processing streams it need not be on this one (an event not yet recorded counts as complete)
  if (async) HIPCHK(c, hipStreamWaitEvent(ln.st, c->prep_ev[slot], 0));
  std::vector<Row> rows;
  for (int p0 = 0; p0 + 1 < P; p0 += c->rows_cap) {
    const int n = std::min(c->rows_cap, P - 1 - p0);
    rows.resize(n);
    for (int i = 0; i < n; ++i) rows[i] = Row{slot, r.prompt[p0 + i], p0 + i};
    int rc = run_rows(c, ln, rows.data(), n, false, nullptr, true, !async);
    if (rc != FLOVER_OK) {
      s.state = FLOVER_SLOT_DEAD;   // never joins an iteration; the next flover_reorder_evict frees the slot
      return rc;
    }
  }
  if (async && P > 1) {
    HIPCHK(c, hipEventRecord(c->prep_ev[slot], ln.st));
    s.pending = true;
    s.ev = slot;
  }
  s.len = P - 1;
  s.next_token = r.prompt[P - 1];
  return FLOVER_OK;
}

bool known(const flover_ctx* c, uint64_t id) {
  for (const Slot& s : c->slots)
    if ((s.state == FLOVER_SLOT_READY || s.state == FLOVER_SLOT_LIVE) && s.req_id == id) return true;
  for (const Waiting& r : c->reque)
    if (r.req_id == id) return true;
  return false;
}

// Algorithm 3 (Section V-D): where the compact region goes.  A window as long as the number of valid entries slides
// over the occupancy array once; the window that keeps the most weight inside leaves the least outside, which is the
// listing's cost.  The window at offset 0 is a candidate like every other (the listing as printed never scores it),
// and a later window replaces the choice only when it keeps strictly more, so the lowest offset wins ties.
// arr: 0 = empty, otherwise the entry's weight (1, or cached rows + 1 for FLOVER_SHUFFLE_BY_LENGTH).
int find_window(const int32_t* arr, int n, int* min_cost, int* non_zero) {
  int width = 0;
  long all = 0;
  for (int i = 0; i < n; ++i) {
    width += arr[i] != 0;
    all += arr[i];
  }
  long kept = 0;
  for (int i = 0; i < width; ++i) kept += arr[i];
  long most_kept = kept;
  int at = 0;
  for (int right = width; right < n; ++right) {   // the window now ends at `right`
    kept += arr[right] - arr[right - width];
    if (kept > most_kept) {
      most_kept = kept;
      at = right - width + 1;
    }
  }
  *min_cost = (int)(all - most_kept);
  *non_zero = width;
  return at;
}

int copy_in(flover_ctx* c, void* dst, const void* src, size_t bytes, const char* name) {
  if (!src) return fail(c, FLOVER_E_INVAL, std::string("missing weight: ") + name);
  HIPCHK(c, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, c->st));
  return FLOVER_OK;
}

// Copies (and re-tiles) layer l from w, whose per-layer tensors start at layer src_l of their stacks.
int load_layer(flover_ctx* c, int l, const flover_weights* w, int src_l) {
  const flover_config& f = c->cfg;
  const size_t e = esize(f.dtype), H = f.hidden, F = f.ffn, sl = src_l;
  const bool gpt = f.arch == FLOVER_ARCH_GPT;
  hipStream_t st = c->st;
  LayerW& lw = c->lw[l];
  auto at = [&](const void* p, size_t per_layer_elems) -> const char* {
    return p ? (const char*)p + sl * per_layer_elems * e : nullptr;
  };
  if (!w->wqkv || !w->wo || !w->w1 || !w->w2 || (!gpt && !w->wu)) return fail(c, FLOVER_E_INVAL, "missing weight matrix");
  int rc;
  if ((rc = copy_in(c, lw.ln1_g, at(w->ln1_g, H), H * e, "ln1_g")) != FLOVER_OK) return rc;
  if ((rc = copy_in(c, lw.ln2_g, at(w->ln2_g, H), H * e, "ln2_g")) != FLOVER_OK) return rc;
  if (f.dtype != FLOVER_F32) {   // padding tiles of the re-tiled matrices must read as zero
    HIPCHK(c, flk::zero_fill(lw.wqkv, flk::gemm_tiled_bytes(f.dtype, 3 * f.hidden, f.hidden), st));
    HIPCHK(c, flk::zero_fill(lw.wo, flk::gemm_tiled_bytes(f.dtype, f.hidden, f.hidden), st));
    HIPCHK(c, flk::zero_fill(lw.w1, flk::gemm_tiled_bytes(f.dtype, gpt ? f.ffn : 2 * f.ffn, f.hidden), st));
    HIPCHK(c, flk::zero_fill(lw.w2, flk::gemm_tiled_bytes(f.dtype, f.hidden, f.ffn), st));
  }
  HIPCHK(c, flk::retile(f.dtype, at(w->wqkv, 3 * H * H), 3 * f.hidden, f.hidden, lw.wqkv, 0, c->p_qkv.NT, st));
  HIPCHK(c, flk::retile(f.dtype, at(w->wo, H * H), f.hidden, f.hidden, lw.wo, 0, c->p_o.NT, st));
  if (c->p_1.paired) {   // gate and up tiles alternate: a 32-column group holds both projections of 16 MLP columns
    HIPCHK(c, flk::retile(f.dtype, at(w->w1, F * H), f.ffn, f.hidden, lw.w1, 0, c->p_1.NT, st, 2));
    HIPCHK(c, flk::retile(f.dtype, at(w->wu, F * H), f.ffn, f.hidden, lw.w1, 16, c->p_1.NT, st, 2));
  } else {
    HIPCHK(c, flk::retile(f.dtype, at(w->w1, F * H), f.ffn, f.hidden, lw.w1, 0, c->p_1.NT, st));
    if (!gpt) HIPCHK(c, flk::retile(f.dtype, at(w->wu, F * H), f.ffn, f.hidden, lw.w1, f.ffn, c->p_1.NT, st));
  }
  HIPCHK(c, flk::retile(f.dtype, at(w->w2, H * F), f.hidden, f.ffn, lw.w2, 0, c->p_2.NT, st));
  if (gpt) {
    if ((rc = copy_in(c, lw.ln1_b, at(w->ln1_b, H), H * e, "ln1_b")) != FLOVER_OK) return rc;
    if ((rc = copy_in(c, lw.ln2_b, at(w->ln2_b, H), H * e, "ln2_b")) != FLOVER_OK) return rc;
    if ((rc = copy_in(c, lw.bqkv, at(w->bqkv, 3 * H), 3 * H * e, "bqkv")) != FLOVER_OK) return rc;
    if ((rc = copy_in(c, lw.bo, at(w->bo, H), H * e, "bo")) != FLOVER_OK) return rc;
    if ((rc = copy_in(c, lw.b1, at(w->b1, F), F * e, "b1")) != FLOVER_OK) return rc;
    if ((rc = copy_in(c, lw.b2, at(w->b2, H), H * e, "b2")) != FLOVER_OK) return rc;
  }
  if (!c->layer_loaded[l]) {
    c->layer_loaded[l] = true;
    c->layers_loaded += 1;
  }
  return FLOVER_OK;
}

// Frees what the context owns outside the arena (pinned staging, events, the pre-processing stream).
void release(flover_ctx* c) {
  std::vector<Lane*> lanes{&c->step_lane};
  for (Lane& pl : c->prep_lanes) lanes.push_back(&pl);
  for (Lane* ln : lanes) {
    for (int i = 0; i < kStageRing; ++i) {
      if (ln->h_stage[i]) (void)hipHostFree(ln->h_stage[i]);
      if (ln->staged[i]) (void)hipEventDestroy(ln->staged[i]);
      if (ln->done[i]) (void)hipEventDestroy(ln->done[i]);
    }
    if (ln->h_tok) (void)hipHostFree(ln->h_tok);
  }
  for (int i = 0; i < kStageRing; ++i) {
    if (c->h_moves_ring[i]) (void)hipHostFree(c->h_moves_ring[i]);
    if (c->moves_ev[i]) (void)hipEventDestroy(c->moves_ev[i]);
  }
  if (c->compact_ev) (void)hipEventDestroy(c->compact_ev);
  for (hipEvent_t e : c->prep_ev)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  for (Lane& pl : c->prep_lanes)
    if (pl.st) (void)hipStreamDestroy(pl.st);
}

// True once the slot's context cache is complete; makes the iteration's stream wait for it.
bool context_ready(flover_ctx* c, Slot& s) {
  if (!s.pending) return true;
  // mode 2 never skips a request: the iteration's stream waits for the cache, however far the passes have got
  if (c->cfg.async_preprocess != 2 && hipEventQuery(c->prep_ev[s.ev]) != hipSuccess) return false;
  (void)hipStreamWaitEvent(c->st, c->prep_ev[s.ev], 0);
  s.pending = false;
  return true;
}

}  // namespace

// ===================================================================== public API

extern "C" {

const char* flover_last_error(const flover_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

int32_t flover_query_arena_bytes(const flover_config* cfg, uint64_t* out_bytes) {
  std::string why;
  if (!out_bytes) return fail(nullptr, FLOVER_E_INVAL, "null out_bytes");
  int rc = check_shape(cfg, &why);
  if (rc != FLOVER_OK) return fail(nullptr, rc, why);
  flover_ctx tmp{};
  tmp.cfg = *cfg;
  *out_bytes = layout(&tmp, nullptr);
  return FLOVER_OK;
}

int32_t flover_init(const flover_config* cfg, const flover_weights* w, flover_ctx** out_ctx) {
  std::string why;
  if (!out_ctx || !w) return fail(nullptr, FLOVER_E_INVAL, "null argument");
  *out_ctx = nullptr;
  int rc = check_shape(cfg, &why);
  if (rc != FLOVER_OK) return fail(nullptr, rc, why);
  if (!cfg->arena || ((uintptr_t)cfg->arena & 255)) return fail(nullptr, FLOVER_E_INVAL, "arena null or not 256-byte aligned");
  flover_ctx* c = new flover_ctx();
  c->cfg = *cfg;
  c->st = (hipStream_t)cfg->stream;
  const size_t need = layout(c, (char*)cfg->arena);
  if (need > cfg->arena_bytes) {
    delete c;
    return fail(nullptr, FLOVER_E_NOMEM, "arena too small: need " + std::to_string(need) + " bytes");
  }
  auto bail = [&](int code) {
    g_err = c->err;
    release(c);
    delete c;
    return code;
  };
#define TRY(expr)                  \
  do {                             \
    int rc_ = (expr);              \
    if (rc_ != FLOVER_OK) return bail(rc_); \
  } while (0)
#define HIPTRY(expr)                                                                  \
  do {                                                                                \
    hipError_t e_ = (expr);                                                           \
    if (e_ != hipSuccess) {                                                           \
      c->err = std::string(#expr) + ": " + hipGetErrorString(e_);                     \
      return bail(FLOVER_E_HIP);                                                      \
    }                                                                                 \
  } while (0)
  c->step_lane.st = c->st;
  c->step_lane.ring = kStageRing;
  for (int i = 0; i < kStageRing; ++i) {
    HIPTRY(hipHostMalloc((void**)&c->step_lane.h_stage[i], c->stage_ints * 4, hipHostMallocDefault));
    HIPTRY(hipEventCreateWithFlags(&c->step_lane.staged[i], hipEventDisableTiming));
    HIPTRY(hipEventCreateWithFlags(&c->step_lane.done[i], hipEventDisableTiming));
    HIPTRY(hipHostMalloc((void**)&c->h_moves_ring[i], (size_t)cfg->max_concurrency * sizeof(int4), hipHostMallocDefault));
    HIPTRY(hipEventCreateWithFlags(&c->moves_ev[i], hipEventDisableTiming));
  }
  HIPTRY(hipHostMalloc((void**)&c->step_lane.h_tok, (size_t)kStageRing * c->rows_cap * 4, hipHostMallocDefault));
  if (cfg->async_preprocess) {
    for (Lane& pl : c->prep_lanes) {
      HIPTRY(hipStreamCreateWithFlags(&pl.st, hipStreamNonBlocking));   // default priority
      pl.ring = kStageRing;
      for (int i = 0; i < kStageRing; ++i) {
        HIPTRY(hipHostMalloc((void**)&pl.h_stage[i], c->stage_ints * 4, hipHostMallocDefault));
        HIPTRY(hipEventCreateWithFlags(&pl.staged[i], hipEventDisableTiming));
      }
    }
    HIPTRY(hipEventCreateWithFlags(&c->compact_ev, hipEventDisableTiming));
    c->prep_ev.assign(cfg->max_concurrency, nullptr);
    for (int i = 0; i < cfg->max_concurrency; ++i) HIPTRY(hipEventCreateWithFlags(&c->prep_ev[i], hipEventDisableTiming));
  }

  const flover_config& f = c->cfg;
  const int e = esize(f.dtype), L = f.n_layer, H = f.hidden, V = f.vocab, S = f.max_seq;
  const bool gpt = f.arch == FLOVER_ARCH_GPT;
  hipStream_t st = c->st;
  // everything the kernels may read before it is written starts at zero (padding tiles, cache, row buffers)
  HIPTRY(flk::zero_fill((char*)cfg->arena + c->act_off, need - c->act_off, st));
  // every per-layer pointer NULL: the layers are handed over one by one with flover_set_layer_weights
  const bool deferred = !w->ln1_g && !w->ln2_g && !w->wqkv && !w->wo && !w->w1 && !w->w2 && !w->wu;
  c->layer_loaded.assign(L, false);
  if (!deferred)
    for (int l = 0; l < L; ++l) TRY(load_layer(c, l, w, l));
  TRY(copy_in(c, c->wte, w->wte, (size_t)V * H * e, "wte"));
  TRY(copy_in(c, c->lnf_g, w->lnf_g, (size_t)H * e, "lnf_g"));
  if (gpt) {
    TRY(copy_in(c, c->wpe, w->wpe, (size_t)S * H * e, "wpe"));
    TRY(copy_in(c, c->lnf_b, w->lnf_b, (size_t)H * e, "lnf_b"));
  }
  const void* lm = gpt ? w->wte : w->wlm;
  if (!lm) {
    c->err = "missing output projection";
    return bail(FLOVER_E_INVAL);
  }
  if (f.dtype != FLOVER_F32) HIPTRY(flk::zero_fill(c->wlm, flk::gemm_tiled_bytes(f.dtype, V, H), st));
  HIPTRY(flk::retile(f.dtype, lm, V, H, c->wlm, 0, c->p_lm.NT, st));
  if (!gpt) {
    // cos/sin of pos * theta^(-2i/d), evaluated in double and rounded once to fp32
    const int half = f.head_dim / 2;
    std::vector<float> cs((size_t)S * half * 2);
    for (int p = 0; p < S; ++p)
      for (int i = 0; i < half; ++i) {
        const double ang = (double)p * std::pow((double)f.rope_theta, -2.0 * i / f.head_dim);
        cs[((size_t)p * half + i) * 2] = (float)std::cos(ang);
        cs[((size_t)p * half + i) * 2 + 1] = (float)std::sin(ang);
      }
    HIPTRY(hipMemcpy(c->rope_cs, cs.data(), cs.size() * 4, hipMemcpyHostToDevice));
  }
  HIPTRY(hipStreamSynchronize(st));
  c->slots.assign(f.max_concurrency, Slot());
  *out_ctx = c;
  return FLOVER_OK;
#undef TRY
#undef HIPTRY
}

int32_t flover_set_layer_weights(flover_ctx* c, int32_t layer, const flover_weights* w) {
  if (!c || !w) return fail(c, FLOVER_E_INVAL, "null argument");
  std::lock_guard<std::mutex> lock(c->mu);
  if (layer < 0 || layer >= c->cfg.n_layer) return fail(c, FLOVER_E_INVAL, "layer out of range");
  for (const Slot& s : c->slots)
    if (s.state != FLOVER_SLOT_EMPTY) return fail(c, FLOVER_E_STATE, "requests are in flight");
  int rc = load_layer(c, layer, w, 0);
  if (rc != FLOVER_OK) return rc;
  HIPCHK(c, hipStreamSynchronize(c->st));   // the caller may free or overwrite its copy on return
  return FLOVER_OK;
}

int32_t flover_destroy(flover_ctx* ctx) {
  if (!ctx) return FLOVER_OK;
  (void)hipStreamSynchronize(ctx->st);
  for (Lane& pl : ctx->prep_lanes)
    if (pl.st) (void)hipStreamSynchronize(pl.st);
  release(ctx);
  delete ctx;
  return FLOVER_OK;
}

int32_t flover_add_request(flover_ctx* c, uint64_t req_id, const int32_t* prompt, int32_t P, int32_t max_new,
                           int32_t* out_slot) {
  if (!c || !prompt) return fail(c, FLOVER_E_INVAL, "null argument");
  const flover_config& f = c->cfg;
  if (P < 1 || max_new < 1 || P + max_new > f.max_seq) return fail(c, FLOVER_E_INVAL, "prompt_len / max_new_tokens out of range");
  for (int i = 0; i < P; ++i)
    if (prompt[i] < 0 || prompt[i] >= f.vocab) return fail(c, FLOVER_E_INVAL, "prompt token out of range");
  std::lock_guard<std::mutex> lock(c->mu);
  if (c->layers_loaded < f.n_layer) return fail(c, FLOVER_E_STATE, "layer weights are missing: flover_set_layer_weights for every layer first");
  if (known(c, req_id)) return fail(c, FLOVER_E_INVAL, "req_id already waiting or live");
  Waiting r{req_id, std::vector<int32_t>(prompt, prompt + P), max_new};
  int slot = -1;
  if (c->reque.empty()) slot = place(c);
  if (slot >= 0) {
    int rc = preprocess(c, slot, r);
    if (rc != FLOVER_OK) return rc;
  } else {
    c->reque.push_back(std::move(r));
  }
  if (out_slot) *out_slot = slot;
  return FLOVER_OK;
}

int32_t flover_add_request_cached(flover_ctx* c, uint64_t req_id, int32_t context_len, int32_t next_token,
                                  int32_t max_new, int32_t* out_slot) {
  if (!c) return FLOVER_E_INVAL;
  const flover_config& f = c->cfg;
  if (context_len < 0 || max_new < 1 || context_len + 1 + max_new > f.max_seq)
    return fail(c, FLOVER_E_INVAL, "context_len / max_new_tokens out of range");
  if (next_token < 0 || next_token >= f.vocab) return fail(c, FLOVER_E_INVAL, "token out of range");
  std::lock_guard<std::mutex> lock(c->mu);
  if (c->layers_loaded < f.n_layer) return fail(c, FLOVER_E_STATE, "layer weights are missing: flover_set_layer_weights for every layer first");
  if (known(c, req_id)) return fail(c, FLOVER_E_INVAL, "req_id already waiting or live");
  if (!c->reque.empty()) return fail(c, FLOVER_E_FULL, "requests are waiting for a slot");
  const int slot = place(c);
  if (slot < 0) return fail(c, FLOVER_E_FULL, "no adjacent slot free");
  Slot& s = c->slots[slot];
  s.state = FLOVER_SLOT_READY;
  s.req_id = req_id;
  s.generated = 0;
  s.max_new = max_new;
  s.len = context_len;
  s.next_token = next_token;
  s.pending = false;
  s.ev = -1;
  s.dev_row = -1;
  if (out_slot) *out_slot = slot;
  return FLOVER_OK;
}

int32_t flover_step(flover_ctx* c, flover_step_out* out) {
  if (!c || !out) return fail(c, FLOVER_E_INVAL, "null argument");
  std::unique_lock<std::mutex> lock(c->mu);
  if (!c->inflight.empty()) return fail(c, FLOVER_E_STATE, "submitted iterations are outstanding: collect them first");
  c->launches = 0;
  while (!c->reque.empty()) {        // waiting requests take freed adjacent slots in arrival order
    int slot = place(c);
    if (slot < 0) break;
    int rc = preprocess(c, slot, c->reque.front());
    if (rc != FLOVER_OK) return rc;
    c->reque.pop_front();
  }
  c->launches = 0;                   // pre-processing is not part of the fused iteration's count
  std::vector<Row> rows;
  std::vector<int> live;
  for (;;) {
    int oldest_pending = -1;
    for (int i = c->lo; i < c->hi; ++i) {   // Update(offset,size): every ready request joins
      Slot& s = c->slots[i];
      if (s.state == FLOVER_SLOT_READY) {
        if (context_ready(c, s)) s.state = FLOVER_SLOT_LIVE;
        else if (oldest_pending < 0) oldest_pending = s.ev;
      }
      if (s.state == FLOVER_SLOT_LIVE) {
        live.push_back(i);
        rows.push_back(Row{i, s.next_token, s.len});
      }
    }
    if (!live.empty() || oldest_pending < 0) break;
    // nothing to generate yet but a context cache is being written: wait for one instead of returning empty-handed
    hipEvent_t e = c->prep_ev[oldest_pending];
    lock.unlock();
    HIPCHK(c, hipEventSynchronize(e));
    lock.lock();
  }
  const int n = (int)live.size();
  if (out->capacity < n) return fail(c, FLOVER_E_INVAL, "flover_step_out.capacity too small");
  if (c->cfg.shuffle_mode == FLOVER_SHUFFLE_OFF)   // holes inside the window are still covered by the kernels (and ignored)
    for (int i = c->lo; i < c->hi; ++i)
      if (c->slots[i].state == FLOVER_SLOT_EMPTY || c->slots[i].state == FLOVER_SLOT_DEAD) rows.push_back(Row{i, 0, 0});
  out->n_live = n;
  c->last_launches = 0;
  if (n == 0) return FLOVER_OK;
  c->in_step = true;
  // with its own pre-processing lane flover_add_request may run beside the iteration: the scheduler lock is not
  // held while the GPU works
  const bool async = c->cfg.async_preprocess != 0;
  if (async) lock.unlock();
  int ring = 0;
  int rc = run_rows(c, c->step_lane, rows.data(), (int)rows.size(), true, out->logits, false, true, &ring);
  if (async) lock.lock();
  c->in_step = false;
  if (rc != FLOVER_OK) return rc;
  c->last_launches = c->launches;
  for (int j = 0; j < n; ++j) {
    Slot& s = c->slots[live[j]];
    const int t = c->step_lane.h_tok[(size_t)ring * c->rows_cap + j];
    s.len += 1;
    s.generated += 1;
    s.next_token = t;
    const bool fin = (t == c->cfg.eos_id) || (s.generated >= s.max_new);
    if (out->req_id) out->req_id[j] = s.req_id;
    if (out->slot) out->slot[j] = live[j];
    if (out->token) out->token[j] = t;
    if (out->finished) out->finished[j] = fin ? 1 : 0;
    if (fin) s.state = FLOVER_SLOT_DEAD;
  }
  return FLOVER_OK;
}

// Pipelined form of flover_step: the iteration is only enqueued.  Without an end-of-sequence token the scheduler
// knows from the budgets alone who finishes, so its state advances at submission; the chosen tokens stay on the
// device as the next iteration's input and reach the host when the iteration is collected.
int32_t flover_step_submit(flover_ctx* c, float* logits, int32_t* n_live_out) {
  if (!c) return fail(c, FLOVER_E_INVAL, "null argument");
  std::unique_lock<std::mutex> lock(c->mu);
  if (c->cfg.eos_id >= 0) return fail(c, FLOVER_E_STATE, "pipelined iterations need eos_id < 0");
  if ((int)c->inflight.size() >= kStageRing - 1) return fail(c, FLOVER_E_FULL, "too many iterations outstanding: collect one first");
  c->launches = 0;
  while (!c->reque.empty()) {
    int slot = place(c);
    if (slot < 0) break;
    int rc = preprocess(c, slot, c->reque.front());
    if (rc != FLOVER_OK) return rc;
    c->reque.pop_front();
  }
  c->launches = 0;
  std::vector<Row> rows;
  std::vector<int> live;
  for (int i = c->lo; i < c->hi; ++i) {
    Slot& s = c->slots[i];
    if (s.state == FLOVER_SLOT_READY && context_ready(c, s)) s.state = FLOVER_SLOT_LIVE;
    if (s.state == FLOVER_SLOT_LIVE) {
      live.push_back(i);
      rows.push_back(Row{i, s.dev_row >= 0 ? -1 - s.dev_row : s.next_token, s.len});
    }
  }
  const int n = (int)live.size();
  if (c->cfg.shuffle_mode == FLOVER_SHUFFLE_OFF)
    for (int i = c->lo; i < c->hi; ++i)
      if (c->slots[i].state == FLOVER_SLOT_EMPTY || c->slots[i].state == FLOVER_SLOT_DEAD) rows.push_back(Row{i, 0, 0});
  if (n_live_out) *n_live_out = n;
  c->last_launches = 0;
  if (n == 0) return FLOVER_OK;     // nothing enqueued, nothing to collect
  int ring = 0;
  c->in_step = true;
  int rc = run_rows(c, c->step_lane, rows.data(), (int)rows.size(), true, logits, false, false, &ring);
  c->in_step = false;
  if (rc != FLOVER_OK) return rc;
  c->last_launches = c->launches;
  flover_ctx::InFlight fl;
  fl.id = c->next_step_id++;
  fl.ring = ring;
  fl.n = n;
  fl.ev_end = c->ev_base + c->ev_kind.size();
  fl.req_id.resize(n);
  fl.slot.resize(n);
  fl.fin.resize(n);
  for (int j = 0; j < n; ++j) {
    Slot& s = c->slots[live[j]];
    s.len += 1;
    s.generated += 1;
    s.dev_row = j;
    s.dev_step = fl.id;
    const bool fin = s.generated >= s.max_new;
    fl.req_id[j] = s.req_id;
    fl.slot[j] = live[j];
    fl.fin[j] = fin ? 1 : 0;
    if (fin) s.state = FLOVER_SLOT_DEAD;
  }
  c->inflight.push_back(std::move(fl));
  return FLOVER_OK;
}

int32_t flover_step_collect(flover_ctx* c, flover_step_out* out) {
  if (!c || !out) return fail(c, FLOVER_E_INVAL, "null argument");
  std::unique_lock<std::mutex> lock(c->mu);
  if (c->inflight.empty()) return fail(c, FLOVER_E_STATE, "no submitted iteration to collect");
  flover_ctx::InFlight& fl = c->inflight.front();
  if (out->capacity < fl.n) return fail(c, FLOVER_E_INVAL, "flover_step_out.capacity too small");
  hipEvent_t done = c->step_lane.done[fl.ring];
  lock.unlock();
  HIPCHK(c, hipEventSynchronize(done));
  lock.lock();
  prof_collect(c, fl.ev_end);
  const int* tok = c->step_lane.h_tok + (size_t)fl.ring * c->rows_cap;
  out->n_live = fl.n;
  for (int j = 0; j < fl.n; ++j) {
    if (out->req_id) out->req_id[j] = fl.req_id[j];
    if (out->slot) out->slot[j] = fl.slot[j];
    if (out->token) out->token[j] = tok[j];
    if (out->finished) out->finished[j] = fl.fin[j];
  }
  // the host copy of each request's last token; a slot whose device-resident token was this iteration's is back on
  // host tokens (the request may have been moved by a shuffle since: found by id)
  for (Slot& s : c->slots)
    if (s.state != FLOVER_SLOT_EMPTY && s.dev_step == fl.id && s.dev_row >= 0) {
      s.next_token = tok[s.dev_row];
      s.dev_row = -1;
    }
  c->inflight.pop_front();
  return FLOVER_OK;
}

int32_t flover_mark_finished(flover_ctx* c, uint64_t req_id) {
  if (!c) return FLOVER_E_INVAL;
  std::lock_guard<std::mutex> lock(c->mu);
  for (Slot& s : c->slots)
    if ((s.state == FLOVER_SLOT_LIVE || s.state == FLOVER_SLOT_READY) && s.req_id == req_id) {
      s.state = FLOVER_SLOT_DEAD;
      return FLOVER_OK;
    }
  return fail(c, FLOVER_E_INVAL, "no such live request");
}

int32_t flover_set_next_token(flover_ctx* c, uint64_t req_id, int32_t token) {
  if (!c) return FLOVER_E_INVAL;
  if (token < 0 || token >= c->cfg.vocab) return fail(c, FLOVER_E_INVAL, "token out of range");
  std::lock_guard<std::mutex> lock(c->mu);
  for (Slot& s : c->slots)
    if ((s.state == FLOVER_SLOT_LIVE || s.state == FLOVER_SLOT_READY) && s.req_id == req_id) {
      s.next_token = token;
      s.dev_row = -1;
      return FLOVER_OK;
    }
  return fail(c, FLOVER_E_INVAL, "no such live request");
}

int32_t flover_reorder_evict(flover_ctx* c, flover_reorder_out* out) {
  if (!c || !out) return fail(c, FLOVER_E_INVAL, "null argument");
  const flover_config& f = c->cfg;
  const int C = f.max_concurrency;
  if (out->capacity < C) return fail(c, FLOVER_E_INVAL, "flover_reorder_out.capacity must be >= max_concurrency");
  std::lock_guard<std::mutex> lock(c->mu);
  int n_ev = 0;
  for (int i = 0; i < C; ++i)
    if (c->slots[i].state == FLOVER_SLOT_DEAD) {
      if (out->evicted_req_id) out->evicted_req_id[n_ev] = c->slots[i].req_id;
      if (c->slots[i].pending)   // a context pass may still be writing this slot: later copies into it wait
        HIPCHK(c, hipStreamWaitEvent(c->st, c->prep_ev[c->slots[i].ev], 0));
      ++n_ev;
      c->slots[i] = Slot();
    }
  const int old_lo = c->lo, n_old = c->hi - c->lo;
  int off = 0, min_cost = 0, n1 = 0, n_moves = 0;
  int64_t bytes = 0;
  if (f.shuffle_mode != FLOVER_SHUFFLE_OFF) {
    std::vector<int32_t> arr(std::max(n_old, 1), 0);
    for (int i = 0; i < n_old; ++i) {
      const Slot& s = c->slots[old_lo + i];
      arr[i] = s.state == FLOVER_SLOT_EMPTY ? 0 : f.shuffle_mode == FLOVER_SHUFFLE_BY_LENGTH ? s.len + 1 : 1;
    }
    off = find_window(arr.data(), n_old, &min_cost, &n1);
    if (n1 == 0) {
      off = 0;
      c->lo = c->hi = 0;
    } else {
      std::vector<int> holes, outside;
      for (int i = 0; i < n_old; ++i) {
        const bool inside = i >= off && i < off + n1;
        if (inside && !arr[i]) holes.push_back(old_lo + i);
        if (!inside && arr[i]) outside.push_back(old_lo + i);
      }
      n_moves = (int)holes.size();
      const int row_bytes = f.head_dim * esize(f.dtype);
      const int nseg = 2 * f.n_layer * f.n_head;
      int n_dev = 0, blocks = 0;
      const bool piped = !c->inflight.empty();   // submitted iterations still run: everything stays stream-ordered
      const int mi = c->moves_next;
      c->moves_next = (c->moves_next + 1) % kStageRing;
      if (c->moves_busy[mi]) {
        HIPCHK(c, hipEventSynchronize(c->moves_ev[mi]));
        c->moves_busy[mi] = false;
      }
      int4* h_moves = c->h_moves_ring[mi];
      for (int i = 0; i < n_moves; ++i) {
        const int a = outside[i], b = holes[i];
        if (out->move_src) out->move_src[i] = a;
        if (out->move_dst) out->move_dst[i] = b;
        const int len = c->slots[a].len;
        if (c->slots[a].pending) {   // its context cache is still being written: the copy, and with it every
          HIPCHK(c, hipStreamWaitEvent(c->st, c->prep_ev[c->slots[a].ev], 0));   // later iteration, waits for it
          c->slots[a].pending = false;
          c->slots[a].ev = -1;
        }
        bytes += 2LL * len * 2 * f.n_layer * f.hidden * esize(f.dtype);
        if (len > 0) {
          const int seg_bytes = len * row_bytes;
          h_moves[n_dev] = make_int4(a, b, seg_bytes, blocks);
          blocks += nseg * ((seg_bytes + flk::kCompactPiece - 1) / flk::kCompactPiece);
          ++n_dev;
        }
        c->slots[b] = c->slots[a];
        c->slots[a] = Slot();
      }
      if (n_dev > 0) {
        HIPCHK(c, hipMemcpyAsync(c->d_moves, h_moves, (size_t)n_dev * sizeof(int4), hipMemcpyHostToDevice, c->st));
        HIPCHK(c, hipEventRecord(c->moves_ev[mi], c->st));
        c->moves_busy[mi] = true;
        const int pi = prof_begin(c, FLOVER_PROF_COMPACT, bytes);
        if (pi >= 0) (void)hipEventRecord(c->ev[2 * pi], c->st);
        HIPCHK(c, flk::compact(c->kv, 2 * f.n_layer, C, f.n_head, c->slot_bytes, c->d_moves, n_dev, blocks,
                               flk::kCompactPiece, c->st));
        if (pi >= 0) (void)hipEventRecord(c->ev[2 * pi + 1], c->st);
        if (!piped) {
          HIPCHK(c, hipStreamSynchronize(c->st));   // following iterations wait until memory is in order (Section V-D)
          c->compact_pending = false;
          prof_collect(c);
        } else if (c->compact_ev) {                 // the pre-processing stream orders itself behind the copy
          HIPCHK(c, hipEventRecord(c->compact_ev, c->st));
          c->compact_pending = true;
        }
      }
      c->lo = old_lo + off;
      c->hi = c->lo + n1;
    }
  } else {
    while (c->lo < c->hi && c->slots[c->lo].state == FLOVER_SLOT_EMPTY) c->lo++;
    while (c->hi > c->lo && c->slots[c->hi - 1].state == FLOVER_SLOT_EMPTY) c->hi--;
    if (c->lo == c->hi) c->lo = c->hi = 0;
    off = c->lo == c->hi ? 0 : c->lo - old_lo;
  }
  out->n_evicted = n_ev;
  out->mem_offset = off;
  out->new_lo = c->lo;
  out->new_size = c->hi - c->lo;
  out->min_cost = min_cost;
  out->n_moves = n_moves;
  out->bytes_moved = bytes;
  return FLOVER_OK;
}

int32_t flover_get_state(const flover_ctx* c, int32_t* lo_hi_wait, int32_t* state, uint64_t* req_id, int32_t* len,
                         int32_t* next_token, int32_t* generated) {
  if (!c) return FLOVER_E_INVAL;
  std::lock_guard<std::mutex> lock(c->mu);
  if (lo_hi_wait) {
    lo_hi_wait[0] = c->lo;
    lo_hi_wait[1] = c->hi;
    lo_hi_wait[2] = (int)c->reque.size();
  }
  for (int i = 0; i < c->cfg.max_concurrency; ++i) {
    const Slot& s = c->slots[i];
    if (state) state[i] = s.state;
    if (req_id) req_id[i] = s.req_id;
    if (len) len[i] = s.len;
    if (next_token) next_token[i] = s.next_token;
    if (generated) generated[i] = s.generated;
  }
  return FLOVER_OK;
}

int32_t flover_get_kv_cache(const flover_ctx* c, void** base, uint64_t* bytes) {
  if (!c) return FLOVER_E_INVAL;
  if (base) *base = c->kv;
  if (bytes) *bytes = c->kv_bytes;
  return FLOVER_OK;
}

int32_t flover_set_profile(flover_ctx* c, int32_t level) {
  if (!c || level < 0 || level > 2) return fail(c, FLOVER_E_INVAL, "profile level must be 0, 1 or 2");
  std::lock_guard<std::mutex> lock(c->mu);
  c->profile = level;
  c->prof_iter = 0;
  for (int k = 0; k < FLOVER_PROF_KINDS; ++k) {
    c->prof_ms[k] = 0;
    c->prof_launches[k] = 0;
    c->prof_bytes[k] = 0;
  }
  return FLOVER_OK;
}

int32_t flover_get_profile(const flover_ctx* c, int32_t kind, double* ms, int64_t* launches, int64_t* bytes) {
  if (!c || kind < 0 || kind >= FLOVER_PROF_KINDS) return FLOVER_E_INVAL;
  std::lock_guard<std::mutex> lock(c->mu);
  if (ms) *ms = c->prof_ms[kind];
  if (launches) *launches = c->prof_launches[kind];
  if (bytes) *bytes = c->prof_bytes[kind];
  return FLOVER_OK;
}

int32_t flover_last_step_launches(const flover_ctx* c, int32_t* n) {
  if (!c || !n) return FLOVER_E_INVAL;
  *n = c->last_launches;
  return FLOVER_OK;
}

// --------------------------------------------------------------------- operation-level entry points

int32_t flover_k_find_window(const int32_t* arr, int32_t n, int32_t* mem_offset, int32_t* min_cost, int32_t* non_zero) {
  if (!arr || n < 0 || !mem_offset || !min_cost || !non_zero) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  int mc = 0, nz = 0;
  *mem_offset = find_window(arr, n, &mc, &nz);
  *min_cost = mc;
  *non_zero = nz;
  return FLOVER_OK;
}

static size_t attn_ws_layout(int M, int nh, int d, int max_len, size_t* o_items, size_t* o_pml, size_t* o_po) {
  const int chunks = (max_len + flk::attn_chunk() - 1) / flk::attn_chunk();
  const size_t items = (size_t)M * chunks;
  size_t off = align_up((size_t)4 * M * 4, 256);
  *o_items = off;
  off = align_up(off + items * 16, 256);
  *o_pml = off;
  off = align_up(off + items * nh * 2 * 4, 256);
  *o_po = off;
  off = align_up(off + items * nh * d * 4, 256);
  return off;
}

int32_t flover_k_attention_workspace_bytes(int32_t M, int32_t nh, int32_t d, int32_t max_len, uint64_t* out) {
  if (M < 0 || nh < 1 || (d != 64 && d != 128) || max_len < 1 || !out) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  size_t a, b, c2;
  *out = attn_ws_layout(M, nh, d, max_len, &a, &b, &c2);
  return FLOVER_OK;
}

int32_t flover_k_decode_attention(int32_t dtype, const void* q, const void* kcache, const void* vcache,
                                  const int32_t* slot, const int32_t* len, int32_t M, int32_t C, int32_t nh, int32_t d,
                                  int32_t S, void* out, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16) return fail(nullptr, FLOVER_E_INVAL, "bad dtype");
  if (M < 0 || nh < 4 || nh % 4 || (d != 64 && d != 128) || S < 1 || C < 1) return fail(nullptr, FLOVER_E_INVAL, "bad shape");
  if (M == 0) return FLOVER_OK;
  if (!q || !kcache || !vcache || !slot || !len || !out || !workspace) return fail(nullptr, FLOVER_E_INVAL, "null argument");
  int max_len = 0;
  for (int i = 0; i < M; ++i) {
    if (len[i] < 1 || len[i] > S || slot[i] < 0 || slot[i] >= C) return fail(nullptr, FLOVER_E_INVAL, "slot / len out of range");
    max_len = std::max(max_len, len[i]);
  }
  size_t o_items, o_pml, o_po;
  const size_t need = attn_ws_layout(M, nh, d, max_len, &o_items, &o_pml, &o_po);
  if (need > workspace_bytes) return fail(nullptr, FLOVER_E_NOMEM, "attention workspace too small");
  std::vector<int> hs((size_t)2 * M);       // slot[M] | len[M]
  std::vector<int> items;
  for (int i = 0; i < M; ++i) {
    hs[i] = slot[i];
    hs[M + i] = len[i];
    const int nc = (len[i] + flk::attn_chunk() - 1) / flk::attn_chunk();
    for (int ch = 0; ch < nc; ++ch) {
      items.push_back(i);
      items.push_back(ch);
      items.push_back(slot[i]);
      items.push_back(len[i]);
    }
  }
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  HIPCHK(nullptr, hipMemcpyAsync(ws, hs.data(), (size_t)2 * M * 4, hipMemcpyHostToDevice, st));
  HIPCHK(nullptr, hipMemcpyAsync(ws + o_items, items.data(), items.size() * 4, hipMemcpyHostToDevice, st));
  HIPCHK(nullptr, hipStreamSynchronize(st));
  int* ds = (int*)ws;
  flk::AttnWork aw{(const int4*)(ws + o_items), ds, ds + M, (float*)(ws + o_pml), (float*)(ws + o_po),
                   (int)items.size() / 4, flk::attn_chunk(), (max_len + flk::attn_chunk() - 1) / flk::attn_chunk()};
  HIPCHK(nullptr, flk::decode_attention(dtype, d, q, kcache, vcache, aw, M, nh, S, out, st));
  return FLOVER_OK;
}

// ---- decode attention for callers that cannot allocate: same kernels, workspace in a file-scope device array
}  // extern "C"

// One copy per GPU that loads the library, held until the process ends.  In host code this name is only a stand-in
// for the symbol; the device address comes from hipGetSymbolAddress (once per device) and is what the kernels get.
static __device__ __align__(256) unsigned char scratch[FLOVER_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr size_t kNoallocScratchBytes = (size_t)FLOVER_NOALLOC_SCRATCH_BYTES;
constexpr int kNoallocMaxRows = FLOVER_NOALLOC_MAX_ROWS;
constexpr int kMaxDevices = 64;

std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch`; looked up on the first call on that device.
int scratch_of_current_device(void** out) {
  int dev = -1;
  HIPCHK(nullptr, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, FLOVER_E_HIP, "device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIPCHK(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(nullptr, FLOVER_E_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FLOVER_OK;
}

// Row descriptors travel as a kernel argument (2 KiB), so the call needs no host-to-device copy either.
struct NoallocRows {
  int32_t slot[kNoallocMaxRows];
  int32_t len[kNoallocMaxRows];
};

// One block of kNoallocMaxRows threads: thread t owns row t, writes its descriptors and its (row, chunk, slot, len)
// work items; first-item indices are an exclusive scan of the rows' chunk counts.
__global__ __launch_bounds__(kNoallocMaxRows) void noalloc_rows_kernel(NoallocRows r, int M, int chunk, int* __restrict__ row_slot,
                                                                       int* __restrict__ row_len, int4* __restrict__ items) {
  __shared__ int scan[kNoallocMaxRows];
  const int t = threadIdx.x;
  const int slot = t < M ? r.slot[t] : 0, len = t < M ? r.len[t] : 0;
  const int nc = (len + chunk - 1) / chunk;
  scan[t] = nc;
  __syncthreads();
  for (int dlt = 1; dlt < kNoallocMaxRows; dlt <<= 1) {     // inclusive scan, log steps
    const int v = t >= dlt ? scan[t - dlt] : 0;
    __syncthreads();
    scan[t] += v;
    __syncthreads();
  }
  if (t >= M) return;
  const int first = scan[t] - nc;
  row_slot[t] = slot;
  row_len[t] = len;
  for (int ch = 0; ch < nc; ++ch) items[first + ch] = make_int4(t, ch, slot, len);
}

}  // namespace

extern "C" {

int32_t flover_k_decode_attention_noalloc(int32_t dtype, const void* q, const void* kcache, const void* vcache,
                                          const int32_t* slot, const int32_t* len, int32_t M, int32_t C, int32_t nh,
                                          int32_t d, int32_t S, void* out, void* stream) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16) return fail(nullptr, FLOVER_E_INVAL, "bad dtype");
  if (M < 0 || nh < 4 || nh % 4 || (d != 64 && d != 128) || S < 1 || C < 1) return fail(nullptr, FLOVER_E_INVAL, "bad shape");
  if (M == 0) return FLOVER_OK;
  if (!q || !kcache || !vcache || !slot || !len || !out) return fail(nullptr, FLOVER_E_INVAL, "null argument");
  if (M > kNoallocMaxRows)
    return fail(nullptr, FLOVER_E_NOMEM, "flover_k_decode_attention_noalloc serves at most " + std::to_string(kNoallocMaxRows) +
                                             " rows per call; got " + std::to_string(M));
  NoallocRows rows;
  int max_len = 0, n_items = 0;
  for (int i = 0; i < M; ++i) {
    if (len[i] < 1 || len[i] > S || slot[i] < 0 || slot[i] >= C) return fail(nullptr, FLOVER_E_INVAL, "slot / len out of range");
    rows.slot[i] = slot[i];
    rows.len[i] = len[i];
    max_len = std::max(max_len, len[i]);
    n_items += (len[i] + flk::attn_chunk() - 1) / flk::attn_chunk();
  }
  for (int i = M; i < kNoallocMaxRows; ++i) rows.slot[i] = rows.len[i] = 0;
  size_t o_items, o_pml, o_po;
  const size_t need = attn_ws_layout(M, nh, d, max_len, &o_items, &o_pml, &o_po);
  if (need > kNoallocScratchBytes)
    return fail(nullptr, FLOVER_E_NOMEM, "attention workspace of " + std::to_string(need) + " bytes exceeds the built-in scratch of " +
                                             std::to_string(kNoallocScratchBytes) + " bytes: fewer rows or shorter lengths per call");
  void* base = nullptr;
  int rc = scratch_of_current_device(&base);
  if (rc != FLOVER_OK) return rc;
  char* ws = (char*)base;
  int* ds = (int*)ws;
  hipStream_t st = (hipStream_t)stream;
  // every part of the scratch this call reads is written first by this call's own kernels: nothing has to start at zero
  noalloc_rows_kernel<<<1, kNoallocMaxRows, 0, st>>>(rows, M, flk::attn_chunk(), ds, ds + M, (int4*)(ws + o_items));
  HIPCHK(nullptr, hipGetLastError());
  flk::AttnWork aw{(const int4*)(ws + o_items), ds, ds + M, (float*)(ws + o_pml), (float*)(ws + o_po),
                   n_items, flk::attn_chunk(), (max_len + flk::attn_chunk() - 1) / flk::attn_chunk()};
  HIPCHK(nullptr, flk::decode_attention(dtype, d, q, kcache, vcache, aw, M, nh, S, out, st));
  return FLOVER_OK;
}

int32_t flover_k_compact_workspace_bytes(int32_t n_moves, uint64_t* out) {
  if (n_moves < 0 || !out) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  *out = align_up((size_t)std::max(n_moves, 1) * sizeof(int4), 256);
  return FLOVER_OK;
}

int32_t flover_k_compact(void* cache, int32_t L, int32_t C, int32_t nh, int32_t S, int32_t d, int32_t eb,
                         const int32_t* src, const int32_t* dst, const int32_t* len, int32_t n_moves, void* workspace,
                         uint64_t workspace_bytes, void* stream) {
  if (!cache || L < 1 || C < 1 || nh < 1 || S < 1 || d < 1 || (eb != 2 && eb != 4) || n_moves < 0 || (d * eb) % 16)
    return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  if (n_moves == 0) return FLOVER_OK;
  if (!src || !dst || !len || !workspace) return fail(nullptr, FLOVER_E_INVAL, "null argument");
  if ((size_t)n_moves * sizeof(int4) > workspace_bytes) return fail(nullptr, FLOVER_E_NOMEM, "compact workspace too small");
  std::vector<char> is_src(C, 0), is_dst(C, 0);
  for (int i = 0; i < n_moves; ++i) {
    if (src[i] < 0 || src[i] >= C || dst[i] < 0 || dst[i] >= C || len[i] < 0 || len[i] > S)
      return fail(nullptr, FLOVER_E_INVAL, "move out of range");
    if (is_src[src[i]] || is_dst[dst[i]]) return fail(nullptr, FLOVER_E_INVAL, "slot listed twice");
    is_src[src[i]] = 1;
    is_dst[dst[i]] = 1;
  }
  for (int i = 0; i < C; ++i)
    if (is_src[i] && is_dst[i]) return fail(nullptr, FLOVER_E_INVAL, "source and destination sets overlap");
  std::vector<int4> mv;
  int blocks = 0;
  const int nseg = 2 * L * nh;
  for (int i = 0; i < n_moves; ++i) {
    if (len[i] == 0) continue;
    const int seg_bytes = len[i] * d * eb;
    mv.push_back(make_int4(src[i], dst[i], seg_bytes, blocks));
    blocks += nseg * ((seg_bytes + flk::kCompactPiece - 1) / flk::kCompactPiece);
  }
  if (mv.empty()) return FLOVER_OK;
  hipStream_t st = (hipStream_t)stream;
  HIPCHK(nullptr, hipMemcpyAsync(workspace, mv.data(), mv.size() * sizeof(int4), hipMemcpyHostToDevice, st));
  HIPCHK(nullptr, hipStreamSynchronize(st));
  HIPCHK(nullptr, flk::compact(cache, 2 * L, C, nh, (size_t)nh * S * d * eb, workspace, (int)mv.size(), blocks,
                               flk::kCompactPiece, st));
  return FLOVER_OK;
}

int32_t flover_k_gemm_tiled_bytes(int32_t dtype, int32_t N, int32_t K, uint64_t* out) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16 || N < 1 || K < 32 || K % 32 || !out) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  *out = flk::gemm_tiled_bytes(dtype, N, K);
  return FLOVER_OK;
}

int32_t flover_k_gemm_workspace_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K, uint64_t* out) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16 || M < 0 || N < 1 || K < 32 || K % 32 || !out) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  const flk::GemmPlan p = flk::gemm_plan(dtype, N, K);
  *out = align_up((size_t)p.S * std::max(M, 1) * p.ldc * 4, 256);
  return FLOVER_OK;
}

int32_t flover_k_gemm_retile(int32_t dtype, const void* W, int32_t N, int32_t K, void* w_tiled, void* stream) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16 || !W || !w_tiled || N < 1 || K < 32 || K % 32) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  hipStream_t st = (hipStream_t)stream;
  if (dtype != FLOVER_F32) HIPCHK(nullptr, flk::zero_fill(w_tiled, flk::gemm_tiled_bytes(dtype, N, K), st));
  HIPCHK(nullptr, flk::retile(dtype, W, N, K, w_tiled, 0, flk::gemm_plan(dtype, N, K).NT, st));
  return FLOVER_OK;
}

}  // extern "C"

namespace flk {
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ a, uint4* __restrict__ b, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) b[i] = a[i];
}
}  // namespace flk

extern "C" int32_t flover_k_copy_probe(void* dst, const void* src, uint64_t bytes, void* stream) {
  if (!dst || !src || bytes % 16) return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  if (bytes == 0) return FLOVER_OK;
  flk::copy_probe_kernel<<<8192, 256, 0, (hipStream_t)stream>>>((const uint4*)src, (uint4*)dst, bytes / 16);
  HIPCHK(nullptr, hipGetLastError());
  return FLOVER_OK;
}

// y = sum of the split-K slices, in slice order (same order the step's consumers use)
namespace flk {
__global__ void slice_sum_kernel(const float* __restrict__ part, int S, size_t stride, int ldc, float* __restrict__ y, int M,
                                 int N) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)M * N) return;
  const size_t m = i / N, n = i - m * N;
  const size_t idx = m * ldc + n;
  float v = part[idx];
  for (int s = 1; s < S; ++s) v += part[(size_t)s * stride + idx];
  y[i] = v;
}
}  // namespace flk

extern "C" int32_t flover_k_gemm_plan(int32_t dtype, int32_t N, int32_t K, int32_t context_rows, int32_t* slices,
                                      int32_t* k_blocks_per_slice) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16 || N < 1 || K < 32 || K % 32 || context_rows < 0 || !slices ||
      !k_blocks_per_slice)
    return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  flk::GemmPlan p = flk::gemm_plan(dtype, N, K);
  if (context_rows > 0) p = flk::context_plan(p, dtype, context_rows, 16);
  *slices = p.S;
  *k_blocks_per_slice = dtype == FLOVER_F32 ? K / 32 : p.kbs;   // the fp32 kernel takes all of K in one slice
  return FLOVER_OK;
}

extern "C" int32_t flover_k_gemm(int32_t dtype, const void* x, const void* w_tiled, int32_t M, int32_t N, int32_t K,
                                 float* y, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (dtype < FLOVER_F32 || dtype > FLOVER_BF16 || M < 0 || N < 1 || K < 32 || K % 32)
    return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  if (M == 0) return FLOVER_OK;
  if (!x || !w_tiled || !workspace) return fail(nullptr, FLOVER_E_INVAL, "null argument");
  const flk::GemmPlan p = flk::gemm_plan(dtype, N, K);
  const size_t stride = (size_t)M * p.ldc;
  if ((size_t)p.S * stride * 4 > workspace_bytes) return fail(nullptr, FLOVER_E_NOMEM, "gemm workspace too small");
  hipStream_t st = (hipStream_t)stream;
  HIPCHK(nullptr, flk::gemm(dtype, x, w_tiled, M, p, (float*)workspace, stride, 0, st));
  if (y) {
    const size_t total = (size_t)M * N;
    flk::slice_sum_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>((const float*)workspace, p.S, stride, p.ldc, y, M, N);
    HIPCHK(nullptr, hipGetLastError());
  }
  return FLOVER_OK;
}

extern "C" int32_t flover_k_gated_retile(int32_t dtype, const void* Wgate, const void* Wup, int32_t F, int32_t K,
                                         void* w_tiled, void* stream) {
  if (dtype < FLOVER_F16 || dtype > FLOVER_BF16 || !Wgate || !Wup || !w_tiled || F < 32 || K < 32 || K % 32)
    return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  const flk::GemmPlan p = flk::gemm_plan_gated(dtype, F, K);
  if (!p.paired) return fail(nullptr, FLOVER_E_INVAL, "shape not served by the fused gated kernels");
  hipStream_t st = (hipStream_t)stream;
  HIPCHK(nullptr, flk::zero_fill(w_tiled, flk::gemm_tiled_bytes(dtype, 2 * F, K), st));
  HIPCHK(nullptr, flk::retile(dtype, Wgate, F, K, w_tiled, 0, p.NT, st, 2));
  HIPCHK(nullptr, flk::retile(dtype, Wup, F, K, w_tiled, 16, p.NT, st, 2));
  return FLOVER_OK;
}

extern "C" int32_t flover_k_gated_workspace_bytes(int32_t dtype, int32_t M, int32_t F, int32_t K, uint64_t* out) {
  if (dtype < FLOVER_F16 || dtype > FLOVER_BF16 || M < 0 || F < 32 || K < 32 || K % 32 || !out)
    return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  const flk::GemmPlan p = flk::gemm_plan_gated(dtype, F, K);
  if (!p.paired) return fail(nullptr, FLOVER_E_INVAL, "shape not served by the fused gated kernels");
  // enough for either use of M rows: the iteration's two halves, or the slices a context pass of M rows takes
  const int slices = std::max(p.S, flk::context_plan(p, dtype, M, 16).S);
  *out = M > flk::gated_fused_rows(p) ? align_up((size_t)slices * M * p.ldc * 4, 256) : 0;
  return FLOVER_OK;
}

extern "C" int32_t flover_k_gated_mlp(int32_t dtype, const void* x, const void* w_tiled, int32_t M, int32_t F, int32_t K,
                                      int32_t context_pass, void* act, void* workspace, uint64_t workspace_bytes,
                                      void* stream) {
  if (dtype < FLOVER_F16 || dtype > FLOVER_BF16 || M < 0 || F < 32 || K < 32 || K % 32)
    return fail(nullptr, FLOVER_E_INVAL, "bad argument");
  flk::GemmPlan p = flk::gemm_plan_gated(dtype, F, K);
  if (!p.paired) return fail(nullptr, FLOVER_E_INVAL, "shape not served by the fused gated kernels");
  if (M == 0) return FLOVER_OK;
  if (!x || !w_tiled || !act) return fail(nullptr, FLOVER_E_INVAL, "null argument");
  if (context_pass) p = flk::context_plan(p, dtype, M, 16);
  const size_t stride = (size_t)M * p.ldc;
  const bool one_launch = (p.S == 2 && M <= flk::gated_fused_rows(p)) || (p.S == 1 && M > 128);
  if (!one_launch && (!workspace || (size_t)p.S * stride * 4 > workspace_bytes))
    return fail(nullptr, FLOVER_E_NOMEM, "gated workspace too small");
  HIPCHK(nullptr, flk::gemm_gated(dtype, x, w_tiled, M, p, act, (float*)workspace, stride, 0, (hipStream_t)stream));
  return FLOVER_OK;
}
