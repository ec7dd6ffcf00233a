// CPU oracle for the fused decoder step of temporal fusion (Flover).
//
// TEST INFRASTRUCTURE ONLY.  Plain, slow, written for checking by eye.  Only the tests,
// the smoke entry and the benchmark's cpu_baseline leg may call this; the product library
// shares no code with it.
//
// What it computes (paper passages followed):
//   * Request model: prompt, maximum generation length, stop at EOS or at the length limit  -- Section IV.
//   * Slot assignment adjacent to the live region, pre-processing into the assigned slot,
//     ready queue                                                                         -- Algorithm 1, Section V-B.
//   * One generation iteration over the contiguous live window: admit ready requests
//     (Update(offset,size)), run the decoder once per live request, detect finished ones   -- Algorithm 2, Section V-C.
//   * Sliding-window search for the region needing the fewest moved slots                  -- Algorithm 3, Section V-D.
//   * Memory shuffle: copy live slots outside the region into holes inside it              -- Section V-D.
// The decoder mathematics itself (GPT: LayerNorm, learned positions, biases, tanh-GELU; LLaMA:
// RMSNorm, rotary embedding, SwiGLU) is not given by the paper; it is the textbook pre-norm
// decoder, pinned by the tests against a no-cache recomputation and against PyTorch CPU ops.
//
// Arithmetic: double precision throughout.  Storage precision is the configuration's: weights,
// KV cache, q, attention output and MLP activation are rounded (nearest-even) to the model
// dtype; the residual stream and the logits are rounded to fp32.  Greedy argmax is taken on the
// fp32 logits, lowest index on ties.
//
// Readings of the paper where it is silent or inconsistent (each also applied by the product):
//   R1  Algorithm 3 as printed never scores the window at offset 0: its running sum starts from zero and
//       its loop from the first index after that window.  Section V-D claims minimal movement, which the
//       listing then misses (for [1,1,0] it settles on offset 1, one move, where offset 0 needs none).
//       Here every window is scored; a better window replaces the best only when strictly better, as in
//       the listing, so the lowest offset wins ties.
//   R2  arr covers the window [lo,hi) of slots the kernels currently span; entries are 0/1.
//   R3  i-th hole inside the chosen region (ascending) receives the i-th occupied slot outside (ascending).
//   R4  A new request takes slot hi if hi < C, else lo-1 if lo > 0, else waits; an empty region restarts at 0.
//   R5  Every ready request is admitted at the start of an iteration (not just one).
//   R6  Pre-processing caches K/V of prompt positions 0..P-2; the first iteration feeds prompt token P-1,
//       so each of the G generated tokens comes from one fused iteration.
//   R7  EOS token is returned and counted, then the request finishes.
//   R8  Only persistent per-slot state moves in a shuffle: KV rows [0,len) and the scheduler's record.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <deque>
#include <limits>
#include <vector>
#include <omp.h>

namespace {

enum { ARCH_GPT = 0, ARCH_LLAMA = 1 };
enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

// ---------------------------------------------------------------- storage formats

double load_elem(const void* p, int dtype, size_t i) {
  if (dtype == DT_F32) return (double)((const float*)p)[i];
  uint16_t h = ((const uint16_t*)p)[i];
  if (dtype == DT_BF16) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
  }
  // IEEE binary16
  int sign = (h >> 15) & 1, ex = (h >> 10) & 31, man = h & 1023;
  double v;
  if (ex == 0) v = std::ldexp((double)man, -24);
  else if (ex == 31) v = man ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
  else v = std::ldexp((double)(man + 1024), ex - 25);
  return sign ? -v : v;
}

// Round to a binary format with `sig` significant bits, minimum normal exponent emin, nearest-even
// (the FPU's default rounding mode does the tie-breaking in nearbyint).
double round_format(double x, int sig, int emin, double maxfinite) {
  if (x == 0.0 || !std::isfinite(x)) return x;
  int e = std::ilogb(x);
  if (e < emin) e = emin;
  double scale = std::ldexp(1.0, sig - 1 - e);
  double r = std::nearbyint(x * scale) / scale;
  if (std::fabs(r) > maxfinite) r = std::copysign(std::numeric_limits<double>::infinity(), x);
  return r;
}

double rd(double x, int dtype) {
  if (dtype == DT_F32) return (double)(float)x;
  if (dtype == DT_BF16) return round_format(x, 8, -126, 3.3895313892515355e38);
  return round_format(x, 11, -14, 65504.0);
}
double rd32(double x) { return (double)(float)x; }

// ---------------------------------------------------------------- configuration

struct Config {
  int32_t arch, dtype, L, H, nh, d, F, V, S, C, eos_id, shuffle_mode;   // 0 shuffle by slots, 1 off, 2 by cached length
  double ln_eps, rope_theta;
};
struct Weights {   // every linear weight [out][in]; per-layer tensors stacked over layers
  const void *wte, *wpe, *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *wu, *w2, *b2, *lnf_g,
      *lnf_b, *wlm;
};

// ---------------------------------------------------------------- decoder pieces

// y[j] = sum_k x[k] * W[j][k] (+ b[j]); one thread per output, k ascending.
void linear(const Config& c, const double* x, const void* W, size_t w_off, const void* b, size_t b_off, int N, int K,
            double* y) {
#pragma omp parallel for schedule(static)
  for (int j = 0; j < N; ++j) {
    double acc = 0.0;
    size_t base = w_off + (size_t)j * K;
    for (int k = 0; k < K; ++k) acc += x[k] * load_elem(W, c.dtype, base + k);
    if (b) acc += load_elem(b, c.dtype, b_off + j);
    y[j] = acc;
  }
}

// LayerNorm (GPT: mean/variance, gain and bias) or RMSNorm (LLaMA: root mean square, gain); output in model dtype.
void norm(const Config& c, const double* x, const void* g, const void* b, size_t off, double* y) {
  int H = c.H;
  if (c.arch == ARCH_GPT) {
    double mean = 0.0;
    for (int i = 0; i < H; ++i) mean += x[i];
    mean /= H;
    double var = 0.0;
    for (int i = 0; i < H; ++i) var += (x[i] - mean) * (x[i] - mean);
    var /= H;
    double inv = 1.0 / std::sqrt(var + c.ln_eps);
    for (int i = 0; i < H; ++i)
      y[i] = rd((x[i] - mean) * inv * load_elem(g, c.dtype, off + i) + load_elem(b, c.dtype, off + i), c.dtype);
  } else {
    double ms = 0.0;
    for (int i = 0; i < H; ++i) ms += x[i] * x[i];
    ms /= H;
    double inv = 1.0 / std::sqrt(ms + c.ln_eps);
    for (int i = 0; i < H; ++i) y[i] = rd(x[i] * inv * load_elem(g, c.dtype, off + i), c.dtype);
  }
}

// Rotary embedding, "rotate-half" pairing (i, i + d/2), angle = pos * theta^(-2i/d).
void rope(const Config& c, double* v, int pos) {
  int half = c.d / 2;
  for (int i = 0; i < half; ++i) {
    double ang = (double)pos * std::pow(c.rope_theta, -2.0 * i / c.d);
    double cs = std::cos(ang), sn = std::sin(ang);
    double a = v[i], b = v[i + half];
    v[i] = a * cs - b * sn;
    v[i + half] = b * cs + a * sn;
  }
}

double gelu_tanh(double x) {
  const double k = 0.7978845608028654;   // sqrt(2/pi)
  return 0.5 * x * (1.0 + std::tanh(k * (x + 0.044715 * x * x * x)));
}
double silu(double x) { return x / (1.0 + std::exp(-x)); }

// softmax(q.K_j / sqrt(d)) V over rows j = 0..n-1 of one head; K, V rows are d contiguous values.
template <class GetK, class GetV>
void attend_head(int d, int n, const double* q, GetK getk, GetV getv, double* o) {
  std::vector<double> s(n);
  double mx = -std::numeric_limits<double>::infinity();
  double scale = 1.0 / std::sqrt((double)d);
  for (int j = 0; j < n; ++j) {
    double acc = 0.0;
    for (int i = 0; i < d; ++i) acc += q[i] * getk(j, i);
    s[j] = acc * scale;
    mx = std::max(mx, s[j]);
  }
  double den = 0.0;
  for (int j = 0; j < n; ++j) {
    s[j] = std::exp(s[j] - mx);
    den += s[j];
  }
  for (int i = 0; i < d; ++i) o[i] = 0.0;
  for (int j = 0; j < n; ++j)
    for (int i = 0; i < d; ++i) o[i] += s[j] * getv(j, i);
  for (int i = 0; i < d; ++i) o[i] /= den;
}

// ---------------------------------------------------------------- model with slot cache

struct Model {
  Config c;
  Weights w;
  std::vector<float> kv;   // [L][2][C][nh][S][d], values already rounded to the model dtype

  size_t kv_index(int l, int which, int slot, int h, int pos) const {
    return (((((size_t)l * 2 + which) * c.C + slot) * c.nh + h) * c.S + pos) * c.d;
  }

  // One decoder pass for the token `tok` of the request in `slot` at position `pos`:
  // appends its K/V row at `pos`, attends over rows 0..pos, returns fp32-rounded logits if asked.
  void decode_row(int slot, int tok, int pos, double* logits) {
    const int H = c.H, F = c.F, d = c.d, nh = c.nh;
    std::vector<double> x(H), h(H), qkv(3 * (size_t)H), att(H), t(H), g(F), u(F), a(F);
    for (int i = 0; i < H; ++i) {
      double e = load_elem(w.wte, c.dtype, (size_t)tok * H + i);
      if (c.arch == ARCH_GPT) e += load_elem(w.wpe, c.dtype, (size_t)pos * H + i);
      x[i] = rd32(e);
    }
    for (int l = 0; l < c.L; ++l) {
      norm(c, x.data(), w.ln1_g, w.ln1_b, (size_t)l * H, h.data());
      linear(c, h.data(), w.wqkv, (size_t)l * 3 * H * H, c.arch == ARCH_GPT ? w.bqkv : nullptr, (size_t)l * 3 * H,
             3 * H, H, qkv.data());
      for (int hd = 0; hd < nh; ++hd) {
        double* q = &qkv[(size_t)hd * d];
        double* k = &qkv[(size_t)H + hd * d];
        double* v = &qkv[2 * (size_t)H + hd * d];
        if (c.arch == ARCH_LLAMA) {
          rope(c, q, pos);
          rope(c, k, pos);
        }
        float* kc = &kv[kv_index(l, 0, slot, hd, pos)];
        float* vc = &kv[kv_index(l, 1, slot, hd, pos)];
        for (int i = 0; i < d; ++i) {
          q[i] = rd(q[i], c.dtype);
          kc[i] = (float)rd(k[i], c.dtype);
          vc[i] = (float)rd(v[i], c.dtype);
        }
      }
#pragma omp parallel for schedule(static)
      for (int hd = 0; hd < nh; ++hd) {
        const float* kc = &kv[kv_index(l, 0, slot, hd, 0)];
        const float* vc = &kv[kv_index(l, 1, slot, hd, 0)];
        attend_head(
            d, pos + 1, &qkv[(size_t)hd * d], [&](int j, int i) { return (double)kc[(size_t)j * d + i]; },
            [&](int j, int i) { return (double)vc[(size_t)j * d + i]; }, &att[(size_t)hd * d]);
        for (int i = 0; i < d; ++i) att[(size_t)hd * d + i] = rd(att[(size_t)hd * d + i], c.dtype);
      }
      linear(c, att.data(), w.wo, (size_t)l * H * H, c.arch == ARCH_GPT ? w.bo : nullptr, (size_t)l * H, H, H,
             t.data());
      for (int i = 0; i < H; ++i) x[i] = rd32(x[i] + t[i]);
      norm(c, x.data(), w.ln2_g, w.ln2_b, (size_t)l * H, h.data());
      if (c.arch == ARCH_GPT) {
        linear(c, h.data(), w.w1, (size_t)l * F * H, w.b1, (size_t)l * F, F, H, g.data());
        for (int i = 0; i < F; ++i) a[i] = rd(gelu_tanh(g[i]), c.dtype);
        linear(c, a.data(), w.w2, (size_t)l * H * F, w.b2, (size_t)l * H, H, F, t.data());
      } else {
        linear(c, h.data(), w.w1, (size_t)l * F * H, nullptr, 0, F, H, g.data());
        linear(c, h.data(), w.wu, (size_t)l * F * H, nullptr, 0, F, H, u.data());
        for (int i = 0; i < F; ++i) a[i] = rd(silu(g[i]) * u[i], c.dtype);
        linear(c, a.data(), w.w2, (size_t)l * H * F, nullptr, 0, H, F, t.data());
      }
      for (int i = 0; i < H; ++i) x[i] = rd32(x[i] + t[i]);
    }
    if (!logits) return;
    norm(c, x.data(), w.lnf_g, w.lnf_b, 0, h.data());
    linear(c, h.data(), c.arch == ARCH_GPT ? w.wte : w.wlm, 0, nullptr, 0, c.V, H, logits);
    for (int j = 0; j < c.V; ++j) logits[j] = rd32(logits[j]);
  }
};

int argmax_lowest(const double* v, int n) {
  int best = 0;
  for (int j = 1; j < n; ++j)
    if (v[j] > v[best]) best = j;
  return best;
}

// ---------------------------------------------------------------- Algorithm 3 (reading R1)

// What Algorithm 3 (Section V-D) is stated to deliver, written out as its definition: among all windows of `valid`
// consecutive entries, valid = number of non-zero entries, the one that leaves the least weight outside -- for 0/1
// input the fewest slots to move -- and, of equally good ones, the lowest offset (the listing replaces its best
// only on a strictly smaller cost).  Every window is scored, the one at offset 0 included (R1).  Window sums come
// from a prefix-sum table; nothing slides.
// arr: 0 = empty, non-zero = valid with weight arr[i].  Returns the offset; *min_cost_out = weight left outside.
int find_window(const int32_t* arr, int n, int* min_cost_out, int* non_zero_out) {
  std::vector<long> upto(n + 1, 0);   // upto[i] = arr[0] + ... + arr[i-1]
  int valid = 0;
  for (int i = 0; i < n; ++i) {
    upto[i + 1] = upto[i] + arr[i];
    if (arr[i] != 0) valid += 1;
  }
  const long everything = upto[n];
  int best_offset = 0;
  long least_outside = everything - upto[valid];
  for (int offset = 1; offset + valid <= n; ++offset) {
    const long outside = everything - (upto[offset + valid] - upto[offset]);
    if (outside < least_outside) {
      least_outside = outside;
      best_offset = offset;
    }
  }
  if (min_cost_out) *min_cost_out = (int)least_outside;
  if (non_zero_out) *non_zero_out = valid;
  return best_offset;
}

// Moves for a window (reading R3): src[i] -> dst[i], absolute indices into arr.
int plan_moves(const int32_t* arr, int n, int off, int non_zero, int32_t* src, int32_t* dst) {
  std::vector<int> holes, outside;
  for (int i = 0; i < n; ++i) {
    bool inside = i >= off && i < off + non_zero;
    if (inside && arr[i] == 0) holes.push_back(i);
    if (!inside && arr[i] != 0) outside.push_back(i);
  }
  for (size_t i = 0; i < holes.size(); ++i) {
    src[i] = outside[i];
    dst[i] = holes[i];
  }
  return (int)holes.size();
}

// ---------------------------------------------------------------- scheduler (Algorithms 1 and 2)

enum SlotState { EMPTY = 0, READY = 1, LIVE = 2, DEAD = 3 };

struct Slot {
  int state = EMPTY;
  uint64_t req_id = 0;
  int len = 0;         // KV rows cached = position of the next token fed
  int next_token = 0;  // token fed in the next iteration
  int generated = 0;
  int max_new = 0;
};
struct Waiting {
  uint64_t req_id;
  std::vector<int32_t> prompt;
  int max_new;
};

struct Server {
  Model m;
  std::vector<Slot> slots;
  std::deque<Waiting> reque;   // Q_R: arrived, no slot yet
  int lo = 0, hi = 0;          // the kernels' window [lo,hi): buffer_offset = lo, buffer_size = hi - lo

  int place() {   // AssignMemId (R4)
    if (lo == hi) {
      lo = 0;
      hi = 1;
      return 0;
    }
    if (hi < m.c.C) return hi++;
    if (lo > 0) return --lo;
    return -1;
  }
  void preprocess(int slot, const Waiting& r) {   // context cache for prompt positions 0..P-2 (R6)
    Slot& s = slots[slot];
    s.state = READY;
    s.req_id = r.req_id;
    s.generated = 0;
    s.max_new = r.max_new;
    int P = (int)r.prompt.size();
    for (int p = 0; p + 1 < P; ++p) m.decode_row(slot, r.prompt[p], p, nullptr);
    s.len = P - 1;
    s.next_token = r.prompt[P - 1];
  }
  bool known(uint64_t id) const {
    for (const Slot& s : slots)
      if (s.state != EMPTY && s.state != DEAD && s.req_id == id) return true;
    for (const Waiting& r : reque)
      if (r.req_id == id) return true;
    return false;
  }
};

}  // namespace

// ================================================================= C interface (ctypes)

extern "C" {

struct orc_config {
  int32_t arch, dtype, L, H, nh, d, F, V, S, C, eos_id, shuffle_mode;
  double ln_eps, rope_theta;
};
struct orc_weights {
  const void *wte, *wpe, *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *wu, *w2, *b2, *lnf_g, *lnf_b,
      *wlm;
};

static Config to_config(const orc_config* c) {
  Config k;
  std::memcpy(&k, c, sizeof(Config));
  return k;
}
static Weights to_weights(const orc_weights* w) {
  Weights k;
  std::memcpy(&k, w, sizeof(Weights));
  return k;
}

int orc_num_threads() { return omp_get_max_threads(); }

void* orc_create(const orc_config* cfg, const orc_weights* w) {
  Server* s = new Server();
  s->m.c = to_config(cfg);
  s->m.w = to_weights(w);
  const Config& c = s->m.c;
  s->m.kv.assign((size_t)c.L * 2 * c.C * c.nh * c.S * c.d, 0.0f);
  s->slots.resize(c.C);
  return s;
}
void orc_destroy(void* h) { delete (Server*)h; }

// Returns 0 and the slot (or -1 when the request has to wait); -1 on invalid arguments.
int orc_add_request(void* h, uint64_t req_id, const int32_t* prompt, int32_t P, int32_t max_new, int32_t* out_slot) {
  Server* s = (Server*)h;
  const Config& c = s->m.c;
  if (P < 1 || max_new < 1 || P + max_new > c.S) return -1;
  for (int i = 0; i < P; ++i)
    if (prompt[i] < 0 || prompt[i] >= c.V) return -1;
  if (s->known(req_id)) return -1;
  Waiting r{req_id, std::vector<int32_t>(prompt, prompt + P), max_new};
  int slot = -1;
  if (s->reque.empty()) slot = s->place();
  if (slot >= 0) s->preprocess(slot, r);
  else s->reque.push_back(r);
  if (out_slot) *out_slot = slot;
  return 0;
}

// One iteration of Algorithm 2 up to the detection of finished requests.  Output arrays hold one entry
// per live request in ascending slot order; logits (optional) is [n_live][V] doubles holding fp32 values.
int orc_step(void* h, int32_t* n_live_out, uint64_t* req_id, int32_t* slot_out, int32_t* token, int32_t* finished,
             double* logits) {
  Server* s = (Server*)h;
  const Config& c = s->m.c;
  while (!s->reque.empty()) {   // waiting requests take freed slots in arrival order
    int slot = s->place();
    if (slot < 0) break;
    s->preprocess(slot, s->reque.front());
    s->reque.pop_front();
  }
  for (int i = s->lo; i < s->hi; ++i)   // Update(offset,size); inmap.insert (R5)
    if (s->slots[i].state == READY) s->slots[i].state = LIVE;
  std::vector<double> row(c.V);
  int n = 0;
  for (int i = s->lo; i < s->hi; ++i) {
    Slot& sl = s->slots[i];
    if (sl.state != LIVE) continue;   // a finished slot left inside the window is covered but ignored
    s->m.decode_row(i, sl.next_token, sl.len, row.data());
    int tok = argmax_lowest(row.data(), c.V);
    sl.len += 1;
    sl.generated += 1;
    sl.next_token = tok;
    bool fin = (tok == c.eos_id) || (sl.generated >= sl.max_new);
    req_id[n] = sl.req_id;
    slot_out[n] = i;
    token[n] = tok;
    finished[n] = fin ? 1 : 0;
    if (logits) std::memcpy(logits + (size_t)n * c.V, row.data(), sizeof(double) * c.V);
    if (fin) sl.state = DEAD;
    ++n;
  }
  *n_live_out = n;
  return 0;
}

int orc_mark_finished(void* h, uint64_t req_id) {
  Server* s = (Server*)h;
  for (Slot& sl : s->slots)
    if ((sl.state == LIVE || sl.state == READY) && sl.req_id == req_id) {
      sl.state = DEAD;
      return 0;
    }
  return -1;
}

int orc_set_next_token(void* h, uint64_t req_id, int32_t tok) {
  Server* s = (Server*)h;
  for (Slot& sl : s->slots)
    if ((sl.state == LIVE || sl.state == READY) && sl.req_id == req_id) {
      sl.next_token = tok;
      return 0;
    }
  return -1;
}

// FindAndEvict's removal, Algorithm 3, and the shuffle.  out6 = {n_evicted, mem_offset (relative to the
// old window start), new_size, n_moves, new_lo, min_cost}; bytes_moved counts read + write of KV rows [0,len).
int orc_reorder_evict(void* h, int32_t* out6, uint64_t* evicted_req_id, int32_t* move_src, int32_t* move_dst,
                      int64_t* bytes_moved) {
  Server* s = (Server*)h;
  const Config& c = s->m.c;
  int n_ev = 0;
  for (int i = 0; i < c.C; ++i)
    if (s->slots[i].state == DEAD) {
      evicted_req_id[n_ev++] = s->slots[i].req_id;
      s->slots[i] = Slot();
    }
  int old_lo = s->lo, n_old = s->hi - s->lo;
  int n_moves = 0, off = 0, min_cost = 0, n1 = 0;
  int64_t bytes = 0;
  const int ebytes = c.dtype == DT_F32 ? 4 : 2;
  if (c.shuffle_mode != 1) {
    // occupancy array of Algorithm 3: 0/1, or (length-weighted variant) cached rows + 1 for a valid slot
    std::vector<int32_t> arr(std::max(n_old, 1), 0);
    for (int i = 0; i < n_old; ++i) {
      const Slot& sl = s->slots[old_lo + i];
      arr[i] = sl.state == EMPTY ? 0 : (c.shuffle_mode == 2 ? sl.len + 1 : 1);
    }
    off = find_window(arr.data(), n_old, &min_cost, &n1);
    if (n1 == 0) {
      off = 0;
      s->lo = s->hi = 0;
    } else {
      std::vector<int32_t> src(n_old), dst(n_old);
      n_moves = plan_moves(arr.data(), n_old, off, n1, src.data(), dst.data());
      for (int i = 0; i < n_moves; ++i) {
        int a = old_lo + src[i], b = old_lo + dst[i];
        move_src[i] = a;
        move_dst[i] = b;
        int len = s->slots[a].len;
        for (int l = 0; l < c.L; ++l)
          for (int which = 0; which < 2; ++which)
            for (int hd = 0; hd < c.nh; ++hd)
              std::memcpy(&s->m.kv[s->m.kv_index(l, which, b, hd, 0)], &s->m.kv[s->m.kv_index(l, which, a, hd, 0)],
                          sizeof(float) * (size_t)len * c.d);
        bytes += 2LL * len * 2 * c.L * c.H * ebytes;
        s->slots[b] = s->slots[a];
        s->slots[a] = Slot();
      }
      s->lo = old_lo + off;
      s->hi = s->lo + n1;
    }
  } else {   // the variant without memory shuffle: holes stay, only the window's empty ends are dropped
    while (s->lo < s->hi && s->slots[s->lo].state == EMPTY) s->lo++;
    while (s->hi > s->lo && s->slots[s->hi - 1].state == EMPTY) s->hi--;
    if (s->lo == s->hi) s->lo = s->hi = 0;
    off = s->lo == s->hi ? 0 : s->lo - old_lo;
  }
  out6[0] = n_ev;
  out6[1] = off;
  out6[2] = s->hi - s->lo;
  out6[3] = n_moves;
  out6[4] = s->lo;
  out6[5] = min_cost;
  *bytes_moved = bytes;
  return 0;
}

// Snapshot: lo, hi, waiting count, then per slot state / req_id / len / next_token / generated.
int orc_get_state(void* h, int32_t* lo_hi_wait, int32_t* state, uint64_t* req_id, int32_t* len, int32_t* next_token,
                  int32_t* generated) {
  Server* s = (Server*)h;
  lo_hi_wait[0] = s->lo;
  lo_hi_wait[1] = s->hi;
  lo_hi_wait[2] = (int)s->reque.size();
  for (int i = 0; i < s->m.c.C; ++i) {
    const Slot& sl = s->slots[i];
    state[i] = sl.state;
    req_id[i] = sl.req_id;
    len[i] = sl.len;
    next_token[i] = sl.next_token;
    generated[i] = sl.generated;
  }
  return 0;
}

// KV rows [0,n) of one (layer, K/V, slot, head) as doubles.
int orc_read_kv(void* h, int l, int which, int slot, int head, int n, double* out) {
  Server* s = (Server*)h;
  const float* p = &s->m.kv[s->m.kv_index(l, which, slot, head, 0)];
  for (size_t i = 0; i < (size_t)n * s->m.c.d; ++i) out[i] = (double)p[i];
  return 0;
}

// Decoder over a whole token sequence with NO cache: every layer sees all positions at once and
// applies the causal mask explicitly.  Logits ([T][V], fp32 values) for every position.
int orc_full_forward(const orc_config* cfg, const orc_weights* wts, const int32_t* tokens, int T, double* logits) {
  Config c = to_config(cfg);
  Weights w = to_weights(wts);
  const int H = c.H, F = c.F, d = c.d, nh = c.nh;
  std::vector<double> X((size_t)T * H), Q((size_t)T * H), K((size_t)T * H), Vv((size_t)T * H), A((size_t)T * H);
  std::vector<double> h(H), qkv(3 * (size_t)H), t(H), g(F), u(F), a(F);
  for (int p = 0; p < T; ++p)
    for (int i = 0; i < H; ++i) {
      double e = load_elem(w.wte, c.dtype, (size_t)tokens[p] * H + i);
      if (c.arch == ARCH_GPT) e += load_elem(w.wpe, c.dtype, (size_t)p * H + i);
      X[(size_t)p * H + i] = rd32(e);
    }
  for (int l = 0; l < c.L; ++l) {
    for (int p = 0; p < T; ++p) {
      norm(c, &X[(size_t)p * H], w.ln1_g, w.ln1_b, (size_t)l * H, h.data());
      linear(c, h.data(), w.wqkv, (size_t)l * 3 * H * H, c.arch == ARCH_GPT ? w.bqkv : nullptr, (size_t)l * 3 * H,
             3 * H, H, qkv.data());
      for (int hd = 0; hd < nh; ++hd) {
        if (c.arch == ARCH_LLAMA) {
          rope(c, &qkv[(size_t)hd * d], p);
          rope(c, &qkv[(size_t)H + hd * d], p);
        }
      }
      for (int i = 0; i < H; ++i) {
        Q[(size_t)p * H + i] = rd(qkv[i], c.dtype);
        K[(size_t)p * H + i] = rd(qkv[(size_t)H + i], c.dtype);
        Vv[(size_t)p * H + i] = rd(qkv[2 * (size_t)H + i], c.dtype);
      }
    }
    for (int p = 0; p < T; ++p)
      for (int hd = 0; hd < nh; ++hd) {
        attend_head(
            d, p + 1, &Q[(size_t)p * H + hd * d], [&](int j, int i) { return K[(size_t)j * H + hd * d + i]; },
            [&](int j, int i) { return Vv[(size_t)j * H + hd * d + i]; }, &A[(size_t)p * H + hd * d]);
        for (int i = 0; i < d; ++i) A[(size_t)p * H + hd * d + i] = rd(A[(size_t)p * H + hd * d + i], c.dtype);
      }
    for (int p = 0; p < T; ++p) {
      double* x = &X[(size_t)p * H];
      linear(c, &A[(size_t)p * H], w.wo, (size_t)l * H * H, c.arch == ARCH_GPT ? w.bo : nullptr, (size_t)l * H, H, H,
             t.data());
      for (int i = 0; i < H; ++i) x[i] = rd32(x[i] + t[i]);
      norm(c, x, w.ln2_g, w.ln2_b, (size_t)l * H, h.data());
      if (c.arch == ARCH_GPT) {
        linear(c, h.data(), w.w1, (size_t)l * F * H, w.b1, (size_t)l * F, F, H, g.data());
        for (int i = 0; i < F; ++i) a[i] = rd(gelu_tanh(g[i]), c.dtype);
        linear(c, a.data(), w.w2, (size_t)l * H * F, w.b2, (size_t)l * H, H, F, t.data());
      } else {
        linear(c, h.data(), w.w1, (size_t)l * F * H, nullptr, 0, F, H, g.data());
        linear(c, h.data(), w.wu, (size_t)l * F * H, nullptr, 0, F, H, u.data());
        for (int i = 0; i < F; ++i) a[i] = rd(silu(g[i]) * u[i], c.dtype);
        linear(c, a.data(), w.w2, (size_t)l * H * F, nullptr, 0, H, F, t.data());
      }
      for (int i = 0; i < H; ++i) x[i] = rd32(x[i] + t[i]);
    }
  }
  for (int p = 0; p < T; ++p) {
    norm(c, &X[(size_t)p * H], w.lnf_g, w.lnf_b, 0, h.data());
    double* out = logits + (size_t)p * c.V;
    linear(c, h.data(), c.arch == ARCH_GPT ? w.wte : w.wlm, 0, nullptr, 0, c.V, H, out);
    for (int j = 0; j < c.V; ++j) out[j] = rd32(out[j]);
  }
  return 0;
}

// ---------------------------------------------------------------- operation-level entry points

int orc_find_window(const int32_t* arr, int n, int32_t* mem_offset, int32_t* min_cost, int32_t* non_zero) {
  int mc = 0, nz = 0;
  *mem_offset = find_window(arr, n, &mc, &nz);
  *min_cost = mc;
  *non_zero = nz;
  return 0;
}
int orc_plan_moves(const int32_t* arr, int n, int off, int non_zero, int32_t* src, int32_t* dst) {
  return plan_moves(arr, n, off, non_zero, src, dst);
}

// Ragged decode attention on a given cache (one layer): for each listed (row, head) pair,
// out = softmax(q . K[slot][head][0..len) / sqrt(d)) V[slot][head][0..len), unrounded doubles.
// q [M][nh][d]; kcache/vcache [C][nh][S][d] in `dtype`; pairs = n_pairs x (row, head); out [n_pairs][d].
int orc_attention(int dtype, const void* q, const void* kcache, const void* vcache, const int32_t* slot,
                  const int32_t* len, int nh, int d, int S, const int32_t* pairs, int n_pairs, double* out) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int p = 0; p < n_pairs; ++p) {
    int row = pairs[2 * p], hd = pairs[2 * p + 1];
    std::vector<double> qv(d);
    for (int i = 0; i < d; ++i) qv[i] = load_elem(q, dtype, ((size_t)row * nh + hd) * d + i);
    size_t base = ((size_t)slot[row] * nh + hd) * S * d;
    attend_head(
        d, len[row], qv.data(), [&](int j, int i) { return load_elem(kcache, dtype, base + (size_t)j * d + i); },
        [&](int j, int i) { return load_elem(vcache, dtype, base + (size_t)j * d + i); }, out + (size_t)p * d);
  }
  return 0;
}

// y[m][n] = sum_k x[m][k] W[n][k] for listed output columns (cols == NULL: all N); out [M][n_cols] doubles.
int orc_gemm(int dtype, const void* x, const void* W, int M, int N, int K, const int32_t* cols, int n_cols,
             double* out) {
  int nc = cols ? n_cols : N;
#pragma omp parallel for schedule(static)
  for (int ci = 0; ci < nc; ++ci) {
    int n = cols ? cols[ci] : ci;
    for (int m = 0; m < M; ++m) {
      double acc = 0.0;
      for (int k = 0; k < K; ++k) acc += load_elem(x, dtype, (size_t)m * K + k) * load_elem(W, dtype, (size_t)n * K + k);
      out[(size_t)m * nc + ci] = acc;
    }
  }
  return 0;
}

// Slot-to-slot copy of KV rows [0,len) for every (layer, K/V, head) of a cache [L][2][C][nh][S][d] with
// `ebytes` bytes per element; a byte copy, applied move by move.
int orc_compact(void* cache, int L, int C, int nh, int S, int d, int ebytes, const int32_t* src, const int32_t* dst,
                const int32_t* len, int n_moves) {
  uint8_t* base = (uint8_t*)cache;
  size_t row = (size_t)d * ebytes;
  for (int i = 0; i < n_moves; ++i)
    for (int l = 0; l < L; ++l)
      for (int which = 0; which < 2; ++which)
        for (int hd = 0; hd < nh; ++hd) {
          size_t a = (((((size_t)l * 2 + which) * C + src[i]) * nh + hd) * S) * row;
          size_t b = (((((size_t)l * 2 + which) * C + dst[i]) * nh + hd) * S) * row;
          std::memcpy(base + b, base + a, (size_t)len[i] * row);
        }
  return 0;
}

double orc_round(double x, int dtype) { return rd(x, dtype); }

// Rotary embedding of one head vector (d doubles, in place) at position pos.
int orc_rope(double* v, int d, int pos, double theta) {
  Config c{};
  c.d = d;
  c.rope_theta = theta;
  rope(c, v, pos);
  return 0;
}

}  // extern "C"
