// Session state machine and C ABI of the draft / verify / rollback calls (Algorithm 2 of the paper
// with the KV-cache and hidden-state reuse of its Sec. 3.2).  Host code only decides shapes and
// keeps the integer bookkeeping; every arithmetic step runs in the kernels of kernels_*.hip.
#include "kernels.h"
#include <algorithm>
#include <cstring>
#include <mutex>

// With further verifier exits (n levels > 2) C also holds the tokens that wait for the levels above L_i,
// deepest verdict first: C = committed || V[n-1] || ... || V[2], where V[j] are the tokens accepted at exit j that
// exit j+1 has not seen; cut[j] = |committed || V[n-1] || ... || V[j]|, so cut[n] tokens are committed and
// cut[2] == |C| always.  V stays the buffer of L_i (level 1).  With the paper's three exits cut[2] = |C| is all there is.
struct SeqState {
  std::vector<int> C, V, S;   // (see above), tentative at L_i, pending draft block
  int cut[EE_MAX_GROUPS] = {0, 0, 0, 0, 0, 0, 0};
  int len[EE_MAX_GROUPS] = {0, 0, 0, 0, 0, 0, 0};     // KV length per layer group
  int n_hd = 0;               // buffered L_d hidden rows (pending draft block incl. bonus row)
  int n_pi = 0;               // rejection sampling: tokens of V whose L_i distribution is stored
  int n_pu[4] = {0, 0, 0, 0}; // ... and tokens of the buffers at the further verifier exits (levels 2..n-1) whose distribution is stored
  bool sampled = false;       // the pending draft block was drawn from p_{L_d} (its distributions are stored)
  std::vector<int> pages;     // block table
  bool started = false;
};

struct MetaSlot {             // one upload region: host (pinned) + device copy, same layout
  int* h = nullptr;
  int* d = nullptr;
  hipEvent_t copied = nullptr;
  bool in_flight = false;
};

struct KTimer { int fam; hipEvent_t a, b; };

struct ee_session {
  ee_model* m = nullptr;
  hipStream_t st = nullptr;
  int B = 0, max_ctx = 0, max_rows = 0, pps = 0, n_pages = 0, maxM = 0, Mp = 0, maxQT = 0, chunk = 0;
  char* base = nullptr;
  size_t bytes = 0;
  // device buffers (inside the caller's arena)
  void* kv = nullptr;
  float *X = nullptr, *QKV = nullptr, *GU = nullptr, *LOGITS = nullptr, *Hd = nullptr, *Hi = nullptr;
  float* Hup[4] = {nullptr, nullptr, nullptr, nullptr};   // hidden rows buffered at the further verifier exits (levels 2..n-1)
  int n_levels = 2;             // verifier levels: exits after L_d (2 = Alg. 2: L_i and L_f)
  void *XN = nullptr, *Qb = nullptr, *AO = nullptr, *H = nullptr;
  float2* cs = nullptr;
  int4* rowinfo = nullptr;    // [maxM] per-row lookups of the QKV epilogue, resolved once per call
  int *vtok = nullptr, *tok_next = nullptr, *draft_dev = nullptr, *out_dev = nullptr, *page_scratch = nullptr;
  // rejection-sampling acceptance (attached separately): the distributions the draft tokens were drawn from,
  // the L_i distributions of the tokens in V (rows [batch][max_rows][vocab]), and the call's uniform numbers
  float *Pd = nullptr, *Pi = nullptr, *u_dev = nullptr;
  float* Pup[4] = {nullptr, nullptr, nullptr, nullptr};   // the same for the buffers of levels 2..n-1
  bool need_logits = false;
  float *part_o = nullptr, *part_ml = nullptr, *pmax = nullptr, *ssq = nullptr, *gemm_part = nullptr, *inv_rms = nullptr;
  // auxiliary exit heads: adapter output rows z [maxM][d], its rank-r intermediate (fp32 rows and, for bf16
  // models, the bf16 operand of the up projection), that operand's unused sum-of-squares partials, unit gains
  float *Z = nullptr, *T = nullptr, *ssq_t = nullptr, *ones = nullptr;
  void* TF = nullptr;
  size_t part_units = 0;        // capacity of the attention split scratch in (q-tile, split) units per KV head
  int* pidx = nullptr;
  int max_splits = 64;
  // host side
  MetaSlot slot[2];
  size_t meta_ints = 0;
  int* out_host = nullptr;    // pinned: n_accept[B], next[B], draft [B*max_rows]
  std::vector<SeqState> seq;
  std::vector<int> free_pages;
  bool debug_logits = false, time_kernels = false;
  int last_rows = 0;
  std::vector<KTimer> timers;
  int launches[KF_COUNT] = {0};
  // meta layout (offsets in ints)
  size_t o_row_seq, o_row_pos, o_row_tok, o_row_src, o_row_dst, o_seq_row0, o_seq_m, o_seq_p0, o_seq_qt0, o_qt_seq,
      o_qt_local, o_cand, o_n_cand, o_bt;
  int cand_stride = 0;
};

static const char* kFamName[KF_COUNT] = {"embed", "rmsnorm", "gemm_qkv", "rope_append", "attention", "attn_combine", "gemm_o",
                                         "gemm_gate_up", "gemm_down", "gemm_head", "argmax", "accept", "copy_rows", "misc"};

// ---------------------------------------------------------------------------------------------
// arena carving
// ---------------------------------------------------------------------------------------------
struct Carver {
  char* base; size_t cur = 0;
  template <class T> T* take(size_t n) {
    cur = align_up(cur, 256);
    T* p = base ? (T*)(base + cur) : nullptr;
    cur += n * sizeof(T);
    return p;
  }
};

static void layout_meta(ee_session* s) {
  size_t o = 0;
  auto take = [&](size_t n) { size_t r = o; o += (n + 3) / 4 * 4; return r; };
  s->cand_stride = s->max_rows + 1;
  s->o_row_seq = take(s->maxM); s->o_row_pos = take(s->maxM); s->o_row_tok = take(s->maxM);
  s->o_row_src = take(s->maxM); s->o_row_dst = take(s->maxM);
  s->o_seq_row0 = take(s->B); s->o_seq_m = take(s->B); s->o_seq_p0 = take(s->B); s->o_seq_qt0 = take(s->B);
  s->o_qt_seq = take(s->maxQT); s->o_qt_local = take(s->maxQT);
  s->o_cand = take((size_t)s->B * s->cand_stride); s->o_n_cand = take(s->B);
  s->o_bt = take((size_t)s->B * s->pps);
  s->meta_ints = o;
}

static size_t carve(ee_session* s, char* base) {
  const ee_model* m = s->m;
  const ee_config& c = m->cfg;
  const bool bf = m->bf16;
  const int d = c.d_model, D = c.head_dim, Hq = c.n_q_heads, Hkv = c.n_kv_heads;
  const int rep = Hq / Hkv;
  Carver cv{base};
  const size_t es = bf ? 2 : 4;
  const int Mp = s->Mp;
  s->kv = cv.take<char>((size_t)c.n_layers * s->n_pages * Hkv * 2 * EE_PAGE * D * es);
  s->X = cv.take<float>((size_t)s->maxM * d);
  s->XN = bf ? (void*)cv.take<bf16_t>((size_t)Mp * ceil_div(d, 32) * 32) : (void*)cv.take<float>((size_t)s->maxM * d);
  const int nqkv = (Hq + 2 * Hkv) * D, nqkv_p = bf ? ceil_div(nqkv, 16) * 16 : nqkv;
  s->QKV = bf ? nullptr : cv.take<float>((size_t)s->maxM * nqkv_p);
  s->Qb = bf ? (void*)cv.take<bf16_t>((size_t)Hkv * s->maxQT * 16 * D) : (void*)cv.take<float>((size_t)s->maxM * Hq * D);
  s->AO = bf ? (void*)cv.take<bf16_t>((size_t)Mp * ceil_div(Hq * D, 32) * 32) : (void*)cv.take<float>((size_t)s->maxM * Hq * D);
  s->GU = bf ? nullptr : cv.take<float>((size_t)s->maxM * 2 * m->Fp);
  s->H = bf ? (void*)cv.take<bf16_t>((size_t)Mp * ceil_div(c.d_ffn, 32) * 32) : (void*)cv.take<float>((size_t)s->maxM * c.d_ffn);
  s->LOGITS = cv.take<float>((size_t)s->maxM * c.vocab);
  if (c.head_rank > 0) {
    s->Z = cv.take<float>((size_t)s->maxM * d);
    s->T = cv.take<float>((size_t)s->maxM * c.head_rank);
    if (bf) {
      s->TF = cv.take<bf16_t>((size_t)Mp * c.head_rank);
      s->ssq_t = cv.take<float>((size_t)ceil_div(c.head_rank, 16) * Mp);
      s->ones = cv.take<float>(c.head_rank);
    }
  }
  s->Hd = cv.take<float>((size_t)s->B * s->max_rows * d);
  s->Hi = cv.take<float>((size_t)s->B * s->max_rows * d);
  for (int j = 2; j < s->n_levels; ++j) s->Hup[j - 2] = cv.take<float>((size_t)s->B * s->max_rows * d);
  s->cs = cv.take<float2>((size_t)s->maxM * (D / 2));
  s->rowinfo = cv.take<int4>((size_t)s->maxM);
  s->vtok = cv.take<int>(s->maxM);
  s->tok_next = cv.take<int>(s->maxM);
  s->draft_dev = cv.take<int>((size_t)s->B * s->max_rows);
  s->out_dev = cv.take<int>(2 * (size_t)s->B);
  s->page_scratch = cv.take<int>(s->pps);
  if (bf) {
    // attention split scratch: all 64 splits for verify-sized calls (<= 64 rows), 8 for context-build passes
    const size_t qt_small = (size_t)ceil_div(std::min(s->maxM, 64) * rep, 16) + s->B;
    s->part_units = std::max(qt_small * s->max_splits, (size_t)s->maxQT * 8);
    s->part_o = cv.take<float>(s->part_units * Hkv * 16 * D);
    s->part_ml = cv.take<float>(s->part_units * Hkv * 32);
    s->pmax = cv.take<float>((size_t)m->head.ntiles() * Mp);
    s->pidx = cv.take<int>((size_t)m->head.ntiles() * Mp);
    s->ssq = cv.take<float>((size_t)ceil_div(d, 16) * Mp);            // deferred-RMSNorm partials [d/16][Mp]
    size_t gp = 0;                                                    // K-share scratch of the row-tiled GEMM
    for (const MatLoc* ml : {&m->L[0].qkv, &m->L[0].o, &m->L[0].gu, &m->L[0].down, &m->head, &m->auxA[0], &m->auxB[0]})
      if (ml->Np > 0) gp = std::max(gp, bf16_gemm_rows_scratch_floats(ml->ntiles(), ml->ktiles()));
    s->gemm_part = s->maxM > 64 ? cv.take<float>(gp) : nullptr;
    s->inv_rms = cv.take<float>(512);
  }
  s->slot[0].d = cv.take<int>(s->meta_ints);
  s->slot[1].d = cv.take<int>(s->meta_ints);
  (void)rep;
  return align_up(cv.cur, 256);
}

static int shape_session(ee_session* s, const ee_model* m, int batch, int max_ctx, int max_rows, int total_pages) {
  if (!m || batch < 1 || max_ctx < 2 || max_rows < 2) { ee_set_error("bad session shape"); return EE_ERR_ARG; }
  if (!m->bf16 && max_ctx > 8192) { ee_set_error("EE_F32 sessions support max_ctx <= 8192"); return EE_ERR_ARG; }
  const int rep = m->cfg.n_q_heads / m->cfg.n_kv_heads;
  s->m = const_cast<ee_model*>(m);
  s->n_levels = (int)m->exits.size() - 1;
  s->B = batch; s->max_ctx = max_ctx; s->max_rows = max_rows;
  s->pps = ceil_div(max_ctx, EE_PAGE);
  s->n_pages = total_pages > 0 ? total_pages : batch * s->pps;
  s->chunk = m->bf16 ? 512 : 64;                        // context-build rows per pass
  s->maxM = std::max(batch * max_rows, s->chunk);
  // activation rows padded to whole GEMM passes: 64 rows (skinny kernel), blocks of 512 (the row-tiled kernel requests up to 32 row tiles)
  s->Mp = s->maxM <= 64 ? 64 : ceil_div(s->maxM, 512) * 512;
  s->maxQT = ceil_div(s->maxM * rep, 16) + batch;
  layout_meta(s);
  return EE_OK;
}

extern "C" size_t ee_session_bytes(const ee_model* m, int batch, int max_ctx, int max_rows, int total_pages) {
  ee_session tmp;
  if (shape_session(&tmp, m, batch, max_ctx, max_rows, total_pages) != EE_OK) return 0;
  return carve(&tmp, nullptr);
}

extern "C" int ee_session_create(ee_model* m, int batch, int max_ctx, int max_rows, int total_pages, void* dev_arena,
                                 size_t arena_bytes, void* stream, ee_session** out) {
  if (!out || !dev_arena || ((uintptr_t)dev_arena & 255)) { ee_set_error("arena must be non-null and 256-byte aligned"); return EE_ERR_ARG; }
  ee_session* s = new ee_session();
  int rc = shape_session(s, m, batch, max_ctx, max_rows, total_pages);
  if (rc != EE_OK) { delete s; return rc; }
  s->st = (hipStream_t)stream;
  s->base = (char*)dev_arena;
  s->bytes = carve(s, s->base);
  if (arena_bytes < s->bytes) {
    ee_set_error("session arena too small: %zu < %zu", arena_bytes, s->bytes);
    delete s; return EE_ERR_CAPACITY;
  }
  hipError_t e = hipMemsetAsync(s->base, 0, s->bytes, s->st);
  const std::vector<float> unit(s->ones ? m->cfg.head_rank : 0, 1.0f);
  if (e == hipSuccess && s->ones) e = hipMemcpyAsync(s->ones, unit.data(), unit.size() * sizeof(float), hipMemcpyHostToDevice, s->st);
  for (int i = 0; i < 2 && e == hipSuccess; ++i) {
    e = hipHostMalloc((void**)&s->slot[i].h, s->meta_ints * sizeof(int), hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->slot[i].copied, hipEventDisableTiming);
  }
  if (e == hipSuccess) e = hipHostMalloc((void**)&s->out_host, (2 * (size_t)batch + (size_t)batch * max_rows) * sizeof(int), hipHostMallocDefault);
  if (e == hipSuccess) e = hipStreamSynchronize(s->st);
  if (e != hipSuccess) { ee_set_error("session create: %s", hipGetErrorString(e)); ee_session_free(s); return EE_ERR_HIP; }
  s->seq.resize(batch);
  s->free_pages.resize(s->n_pages);
  for (int i = 0; i < s->n_pages; ++i) s->free_pages[i] = s->n_pages - 1 - i;   // pop_back hands out 0, 1, 2, ...
  *out = s;
  return EE_OK;
}

extern "C" void ee_session_free(ee_session* s) {
  if (!s) return;
  if (s->st) (void)hipStreamSynchronize(s->st);
  for (auto& t : s->timers) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
  for (int i = 0; i < 2; ++i) {
    if (s->slot[i].h) (void)hipHostFree(s->slot[i].h);
    if (s->slot[i].copied) (void)hipEventDestroy(s->slot[i].copied);
  }
  if (s->out_host) (void)hipHostFree(s->out_host);
  delete s;
}

// ---------------------------------------------------------------------------------------------
// pages
// ---------------------------------------------------------------------------------------------
static int pages_needed_total(const ee_session* s, const std::vector<int>& want_positions) {
  int need = 0;
  for (int b = 0; b < s->B; ++b) {
    int have = (int)s->seq[b].pages.size(), want = ceil_div(want_positions[b], EE_PAGE);
    if (want > have) need += want - have;
  }
  return need;
}
// make sure sequence b owns pages for positions [0, n)
static int grow_pages(ee_session* s, int b, int n) {
  SeqState& q = s->seq[b];
  while ((int)q.pages.size() * EE_PAGE < n) {
    if (s->free_pages.empty() || (int)q.pages.size() >= s->pps) { ee_set_error("KV page pool exhausted"); return EE_ERR_CAPACITY; }
    q.pages.push_back(s->free_pages.back());
    s->free_pages.pop_back();
  }
  return EE_OK;
}
static int max_len(const ee_session* s, const SeqState& q) {
  int m = 0;
  for (int g = 0; g <= s->n_levels; ++g) m = std::max(m, q.len[g]);
  return m;
}
// every group at the same length, nothing waiting above L_i: the state after a prompt, a vanilla step or the last level
static void settle(const ee_session* s, SeqState& q) {
  for (int g = 0; g <= s->n_levels; ++g) { q.len[g] = (int)q.C.size() - 1; q.cut[g] = (int)q.C.size(); }
}
// give back pages no group needs any more (Sec. 3.2 pruning: only the table tail changes)
static void trim_pages(ee_session* s, int b) {
  SeqState& q = s->seq[b];
  int keep = ceil_div(max_len(s, q) + 1, EE_PAGE);
  while ((int)q.pages.size() > keep) { s->free_pages.push_back(q.pages.back()); q.pages.pop_back(); }
}
static int check_capacity(ee_session* s, const std::vector<int>& want_positions) {
  for (int b = 0; b < s->B; ++b)
    if (want_positions[b] > s->max_ctx) { ee_set_error("sequence %d would need %d positions (max_ctx %d)", b, want_positions[b], s->max_ctx); return EE_ERR_CAPACITY; }
  if (pages_needed_total(s, want_positions) > (int)s->free_pages.size()) { ee_set_error("KV page pool exhausted"); return EE_ERR_CAPACITY; }
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// per-call metadata
// ---------------------------------------------------------------------------------------------
struct CallPlan {
  int M = 0, n_active = 0, max_m = 0, total_qt = 0, max_kv_end = 0;
  std::vector<int> m, p0;        // per sequence rows and first position (m = 0: not taking part)
};

static CallMeta meta_ptrs(const ee_session* s, const int* d) {
  CallMeta c;
  c.row_seq = d + s->o_row_seq; c.row_pos = d + s->o_row_pos; c.row_tok = d + s->o_row_tok;
  c.row_src = d + s->o_row_src; c.row_dst = d + s->o_row_dst;
  c.seq_row0 = d + s->o_seq_row0; c.seq_m = d + s->o_seq_m; c.seq_p0 = d + s->o_seq_p0; c.seq_qt0 = d + s->o_seq_qt0;
  c.qt_seq = d + s->o_qt_seq; c.qt_local = d + s->o_qt_local; c.cand = d + s->o_cand; c.n_cand = d + s->o_n_cand;
  c.block_table = d + s->o_bt;
  return c;
}

// Fill slot `si` from the plan: rows are packed sequence by sequence.  The callbacks give the
// per-row token / gather source / scatter destination; candidates are filled by the caller.
template <class RowFn>
static int build_meta(ee_session* s, int si, CallPlan& p, RowFn row_fn) {
  MetaSlot& sl = s->slot[si];
  if (sl.in_flight) { HIP_TRY(hipEventSynchronize(sl.copied)); sl.in_flight = false; }
  int* h = sl.h;
  const int rep = s->m->cfg.n_q_heads / s->m->cfg.n_kv_heads;
  int row = 0, qt = 0;
  p.M = 0; p.n_active = 0; p.max_m = 0; p.max_kv_end = 0;
  for (int b = 0; b < s->B; ++b) {
    int m = p.m[b];
    h[s->o_seq_row0 + b] = row; h[s->o_seq_m + b] = m; h[s->o_seq_p0 + b] = p.p0[b]; h[s->o_seq_qt0 + b] = qt;
    h[s->o_n_cand + b] = 0;
    if (m == 0) continue;
    p.n_active++; p.max_m = std::max(p.max_m, m); p.max_kv_end = std::max(p.max_kv_end, p.p0[b] + m);
    for (int r = 0; r < m; ++r, ++row) {
      h[s->o_row_seq + row] = b; h[s->o_row_pos + row] = p.p0[b] + r;
      int tok = 0, src = 0, dst = 0;
      row_fn(b, r, tok, src, dst);
      h[s->o_row_tok + row] = tok; h[s->o_row_src + row] = src; h[s->o_row_dst + row] = dst;
    }
    int nqt = ceil_div(m * rep, 16);
    for (int t = 0; t < nqt; ++t, ++qt) { h[s->o_qt_seq + qt] = b; h[s->o_qt_local + qt] = t; }
  }
  p.M = row; p.total_qt = qt;
  if (row > s->maxM || qt > s->maxQT) { ee_set_error("internal: call exceeds work buffers (%d rows)", row); return EE_ERR_CAPACITY; }
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    for (size_t i = 0; i < q.pages.size(); ++i) h[s->o_bt + (size_t)b * s->pps + i] = q.pages[i];
  }
  return EE_OK;
}
static int upload_meta(ee_session* s, int si) {
  MetaSlot& sl = s->slot[si];
  HIP_TRY(hipMemcpyAsync(sl.d, sl.h, s->meta_ints * sizeof(int), hipMemcpyHostToDevice, s->st));
  HIP_TRY(hipEventRecord(sl.copied, s->st));
  sl.in_flight = true;
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// launch accounting
// ---------------------------------------------------------------------------------------------
// With timing on, a family call is bracketed by two recorded events; a call that is one skinny-GEMM launch takes
// the second pair instead, attached to its dispatch (the kernel's own start and end: what a kernel trace reports,
// 2-5 us less than the bracket, which also spans the launch gap).
struct Scope {
  ee_session* s; int fam; hipEvent_t a = nullptr, b = nullptr;
  LaunchEvents own{nullptr, nullptr, false};
  Scope(ee_session* s_, int f) : s(s_), fam(f) {
    s->launches[fam]++;
    if (s->time_kernels) {
      (void)hipEventCreate(&a); (void)hipEventCreate(&b); (void)hipEventRecord(a, s->st);
      (void)hipEventCreate(&own.start); (void)hipEventCreate(&own.stop);
      g_launch_events = &own;
    }
  }
  ~Scope() {
    if (!a) return;
    g_launch_events = nullptr;
    if (own.used) {
      s->timers.push_back({fam, own.start, own.stop});
      (void)hipEventDestroy(a); (void)hipEventDestroy(b);
    } else {
      (void)hipEventRecord(b, s->st);
      s->timers.push_back({fam, a, b});
      (void)hipEventDestroy(own.start); (void)hipEventDestroy(own.stop);
    }
  }
};
#define KF(fam, call) do { Scope sc_(s, fam); call; } while (0)

static void reset_accounting(ee_session* s) {
  for (auto& t : s->timers) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
  s->timers.clear();
  memset(s->launches, 0, sizeof(s->launches));
}

// ---------------------------------------------------------------------------------------------
// forward pass pieces
// ---------------------------------------------------------------------------------------------
// weights cross HBM once per call: up to 16 rows the skinny kernel, from 33 to 512 the row-tiled one, in
// between the row-tiled one for matrices of 128 MB and more (measured: the small projections are quicker
// without its K-share reduction pass); beyond 512 rows the row-tiled kernel goes over the rows in blocks of 512
static void gemm(ee_session* s, int epi, const MatLoc& ml, const bf16_t* A, int M, const GemmOut& o) {
  const bf16_t* W = (const bf16_t*)(s->m->base + ml.off);
  const bool big = (size_t)ml.ntiles() * ml.ktiles() * 1024 >= ((size_t)128 << 20);
  if (M > (big ? 16 : 32)) bf16_gemm_rows(s->st, epi, W, ml.ntiles(), ml.ktiles(), A, M, ml.N, o, s->gemm_part, s->inv_rms);
  else bf16_gemm(s->st, epi, W, ml.ntiles(), ml.ktiles(), A, M, ml.N, o);
}

// offset of the gain that normalises the hidden state behind layer l1: the adapter's own gain at an early exit
// with an auxiliary head, else the shared final gain
static size_t closing_gain(const ee_model* m, int l1) {
  if (m->cfg.head_rank > 0)
    for (size_t e = 0; e + 1 < m->exits.size(); ++e)
      if (l1 == m->exits[e]) return m->auxg[e];
  return m->gfinal;
}

// attention split plan of a call (the same for all its layers): pages per KV split and the scratch handed to the
// kernels; nsplit_out = KV splits of the longest sequence = stride of the partial slots
static int attention_plan(const ee_session* s, const CallPlan& p, int pos_add, AttnScratch& scr, int* nsplit_out) {
  const ee_config& c = s->m->cfg;
  scr = AttnScratch{s->part_o, s->part_ml, (int)std::min<size_t>(s->max_splits, s->part_units / std::max(1, p.total_qt))};
  int per = 1;
  if (s->m->bf16) {
    std::vector<int> kv_end(s->B);
    for (int b = 0; b < s->B; ++b) kv_end[b] = p.m[b] > 0 ? p.p0[b] + p.m[b] + pos_add : 0;
    per = bf16_attention_pages_per_split(kv_end.data(), p.m.data(), s->B, c.n_q_heads, c.n_kv_heads, scr.max_splits);
  }
  const int max_pages = ceil_div(p.max_kv_end + pos_add, EE_PAGE);
  per = std::max(1, std::min(per, max_pages));
  if (nsplit_out) *nsplit_out = ceil_div(max_pages, per);
  return per;
}

// where the rows of a pass come from: the embedding of tokens (a1 of a pass that starts at layer 0), kept hidden rows
// gathered by index (hidden-state reuse of Alg. 2), or the residual stream as it stands
struct PassSource {
  const int* tok = nullptr;
  const float* rows = nullptr; const int* row_idx = nullptr;
};
// where the hidden rows behind the last layer of a pass are kept besides the stream (H_d, H_i, a level's rows): row r
// goes to rows[row_idx[r] + add]; the last down projection's epilogue writes them
struct PassSink {
  float* rows = nullptr; const int* row_idx = nullptr; int add = 0;
};

static void run_layers(ee_session* s, int l0, int l1, const CallPlan& p, const CallMeta& mt, int pos_add, const PassSource& src = PassSource(),
                       const PassSink& sink = PassSink()) {
  const ee_model* m = s->m;
  const ee_config& c = m->cfg;
  const int d = c.d_model, D = c.head_dim, Hq = c.n_q_heads, Hkv = c.n_kv_heads, M = p.M;
  hipStream_t st = s->st;
  if (m->bf16 && l0 < l1) {
    // one launch: rows into the stream, the first layer's operand, the rotary table and the epilogue lookups
    KF(KF_NORM, bf16_begin_pass(st, src.tok ? (const bf16_t*)(m->base + m->emb) : nullptr, src.tok, src.rows, src.row_idx, s->X,
                                (const float*)(m->base + m->L[l0].g1), c.rms_eps, (bf16_t*)s->XN, m->L[l0].qkv.ktiles(), M, d, mt,
                                pos_add, m->inv_freq, s->cs, D / 2, s->pps, s->rowinfo));
  } else {
    if (src.tok) KF(KF_EMBED, k_embed(st, m->bf16, m->base + m->emb, src.tok, s->X, M, d));
    else if (src.rows) KF(KF_COPY, k_copy_rows(st, s->X, nullptr, 0, src.rows, src.row_idx, M, d));
    KF(KF_ROPE, k_rope_table(st, mt, pos_add, m->inv_freq, s->cs, M, D / 2, s->pps, s->rowinfo));
  }
  AttnScratch scr;
  const int per = attention_plan(s, p, pos_add, scr, nullptr);
  for (int l = l0; l < l1; ++l) {
    const LayerLoc& L = m->L[l];
    const float* g1 = (const float*)(m->base + L.g1);
    const float* g2 = (const float*)(m->base + L.g2);
    if (m->bf16) {
      // five launches per layer (six with the merge of a split attention); RMSNorm is deferred into the projections (see NormIn / NormOut)
      const int Mp = s->Mp;
      NormIn nin;         // operand left by the previous EPI_ADD launch
      nin.ssq = s->ssq; nin.n_part = d / 16; nin.stride = Mp; nin.inv_d = 1.0f / (float)d; nin.eps = c.rms_eps;
      NormOut nout;
      nout.xn = (bf16_t*)s->XN; nout.ktiles = ceil_div(d, 32); nout.ssq = s->ssq; nout.stride = Mp;
      GemmOut o;
      if (l != l0) o.nin = nin;            // (the first layer's operand was normalised when the pass was opened)
      RopeOut& R = o.rope;
      R.cs = s->cs; R.rowinfo = s->rowinfo; R.Hq = Hq; R.Hkv = Hkv; R.D = D; R.layer = l;
      R.n_pages = s->n_pages; R.total_qt = p.total_qt; R.Q = (bf16_t*)s->Qb; R.kv = (bf16_t*)s->kv;
      KF(KF_GEMM_QKV, gemm(s, EPI_ROPE, L.qkv, (const bf16_t*)s->XN, M, o));
      KF(KF_ATTN, bf16_attention(st, (const bf16_t*)s->Qb, (const bf16_t*)s->kv, mt, pos_add, s->B, p.max_m, p.total_qt,
                                 p.max_kv_end + pos_add, Hq, Hkv, D, l, s->n_pages, s->pps, scr, (bf16_t*)s->AO, L.o.ktiles(), per));
      o = GemmOut(); o.Y = s->X; o.ldy = d; o.nout = nout; o.nout.g = g2;
      KF(KF_GEMM_O, gemm(s, EPI_ADD, L.o, (const bf16_t*)s->AO, M, o));
      o = GemmOut(); o.H = (bf16_t*)s->H; o.h_ktiles = L.down.ktiles(); o.nin = nin;
      KF(KF_GEMM_GU, gemm(s, EPI_SWIGLU, L.gu, (const bf16_t*)s->XN, M, o));
      // the down projection leaves the operand of whatever reads the stream next: the next layer's QKV
      // projection, or the shared exit head behind the last layer of the pass
      o = GemmOut(); o.Y = s->X; o.ldy = d; o.nout = nout;
      o.nout.g = l + 1 < l1 ? (const float*)(m->base + m->L[l + 1].g1) : (const float*)(m->base + closing_gain(m, l1));
      if (l + 1 == l1) { o.Y2 = sink.rows; o.y2_idx = sink.row_idx; o.y2_add = sink.add; }
      KF(KF_GEMM_DOWN, gemm(s, EPI_ADD, L.down, (const bf16_t*)s->H, M, o));
    } else {
      const float* Wqkv = (const float*)(m->base + L.qkv.off);
      const float* Wo = (const float*)(m->base + L.o.off);
      const float* Wgu = (const float*)(m->base + L.gu.off);
      const float* Wd = (const float*)(m->base + L.down.off);
      KF(KF_NORM, f32_rmsnorm(st, s->X, g1, c.rms_eps, (float*)s->XN, M, d));
      KF(KF_GEMM_QKV, f32_gemm(st, (const float*)s->XN, d, Wqkv, s->QKV, L.qkv.N, M, L.qkv.N, d, false));
      KF(KF_ROPE, f32_rope_append(st, s->QKV, L.qkv.N, s->cs, mt, pos_add, M, Hq, Hkv, D, l, s->n_pages, s->pps, (float*)s->Qb, (float*)s->kv));
      KF(KF_ATTN, f32_attention(st, (const float*)s->Qb, (const float*)s->kv, mt, pos_add, M, Hq, Hkv, D, l, s->n_pages, s->pps,
                                s->max_ctx, (float*)s->AO));
      KF(KF_GEMM_O, f32_gemm(st, (const float*)s->AO, Hq * D, Wo, s->X, d, M, d, Hq * D, true));
      KF(KF_NORM, f32_rmsnorm(st, s->X, g2, c.rms_eps, (float*)s->XN, M, d));
      KF(KF_GEMM_GU, f32_gemm(st, (const float*)s->XN, d, Wgu, s->GU, 2 * m->Fp, M, 2 * m->Fp, d, false));
      KF(KF_GEMM_GU, f32_silu_mul(st, s->GU, 2 * m->Fp, (float*)s->H, M, c.d_ffn));
      KF(KF_GEMM_DOWN, f32_gemm(st, (const float*)s->H, c.d_ffn, Wd, s->X, d, M, d, c.d_ffn, true));
    }
  }
  if (sink.rows && (!m->bf16 || l0 >= l1)) KF(KF_COPY, k_copy_rows(st, sink.rows, sink.row_idx, sink.add, s->X, nullptr, M, d));
}

// Prediction head of exit `which` (0 = L_d, 1 = L_i, ..., n_levels = L_f) + arg max for rows 0..M-1 of X -> vtok.
// The shared final RMSNorm and LM head (Sec. 3.1); at an early exit of a model with auxiliary heads
// (App. I) behind that exit's rank-r adapter  z = x + B (A RMSNorm(x; g)),  which leaves X itself alone.
static void exit_head(ee_session* s, int M, int which) {
  const ee_model* m = s->m;
  const ee_config& c = m->cfg;
  hipStream_t st = s->st;
  const int d = c.d_model, r = c.head_rank;
  const float* gf = (const float*)(m->base + m->gfinal);
  const bool aux = r > 0 && which < s->n_levels;
  if (m->bf16) {
    // the last down projection of the pass left XN = bf16(x * gain) and the partial sums of squares
    const int Mp = s->Mp;
    NormIn nin;
    nin.ssq = s->ssq; nin.n_part = d / 16; nin.stride = Mp; nin.inv_d = 1.0f / (float)d; nin.eps = c.rms_eps;
    if (aux) {
      // t = A n(x): rows into T (cleared: the epilogue adds to what it finds) and as the next operand TF;
      // z = x + B t: into a copy of the rows, leaving the shared head's operand XN = bf16(z * gfinal)
      (void)hipMemsetAsync(s->T, 0, (size_t)M * r * sizeof(float), st);
      (void)hipMemcpyAsync(s->Z, s->X, (size_t)M * d * sizeof(float), hipMemcpyDeviceToDevice, st);
      GemmOut o;
      o.nin = nin; o.Y = s->T; o.ldy = r;
      o.nout.xn = (bf16_t*)s->TF; o.nout.ktiles = r / 32; o.nout.ssq = s->ssq_t; o.nout.stride = Mp; o.nout.g = s->ones;
      KF(KF_GEMM_HEAD, gemm(s, EPI_ADD, m->auxA[which], (const bf16_t*)s->XN, M, o));
      o = GemmOut(); o.Y = s->Z; o.ldy = d;
      o.nout.xn = (bf16_t*)s->XN; o.nout.ktiles = ceil_div(d, 32); o.nout.ssq = s->ssq; o.nout.stride = Mp; o.nout.g = gf;
      KF(KF_GEMM_HEAD, gemm(s, EPI_ADD, m->auxB[which], (const bf16_t*)s->TF, M, o));
    }
    GemmOut o;
    o.nin = nin;
    // (max, arg max) partials [row][tile]: the reduction of a row then reads one contiguous strip
    const int pstride = m->head.ntiles();
    o.pmax = s->pmax; o.pidx = s->pidx; o.pstride = pstride;
    if (s->debug_logits || s->need_logits) { o.Y = s->LOGITS; o.ldy = c.vocab; }
    KF(KF_GEMM_HEAD, gemm(s, EPI_ARGMAX, m->head, (const bf16_t*)s->XN, M, o));
    KF(KF_ARGMAX, bf16_argmax_reduce(st, s->pmax, s->pidx, m->head.ntiles(), pstride, M, s->vtok));
  } else {
    const float* hidden = s->X;
    if (aux) {
      KF(KF_NORM, f32_rmsnorm(st, s->X, (const float*)(m->base + m->auxg[which]), c.rms_eps, (float*)s->XN, M, d));
      KF(KF_GEMM_HEAD, f32_gemm(st, (const float*)s->XN, d, (const float*)(m->base + m->auxA[which].off), s->T, r, M, r, d, false));
      (void)hipMemcpyAsync(s->Z, s->X, (size_t)M * d * sizeof(float), hipMemcpyDeviceToDevice, st);
      KF(KF_GEMM_HEAD, f32_gemm(st, (const float*)s->T, r, (const float*)(m->base + m->auxB[which].off), s->Z, d, M, d, r, true));
      hidden = s->Z;
    }
    KF(KF_NORM, f32_rmsnorm(st, hidden, gf, c.rms_eps, (float*)s->XN, M, d));
    KF(KF_GEMM_HEAD, f32_gemm(st, (const float*)s->XN, d, (const float*)(m->base + m->head.off), s->LOGITS, c.vocab, M,
                              c.vocab, d, false));
    KF(KF_ARGMAX, f32_argmax(st, s->LOGITS, M, c.vocab, s->vtok));
  }
  s->last_rows = M;
}

static int finish(ee_session* s) {
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(s->st));
  for (int i = 0; i < 2; ++i) s->slot[i].in_flight = false;
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: prefill
// ---------------------------------------------------------------------------------------------
// (Re)start the sequences with lens[b] > 0 from their prompts (tokens: those prompts packed in sequence order);
// sequences with lens[b] == 0 keep their state.  Pages of a restarted sequence go back to the pool first.
static int prefill_impl(ee_session* s, const int32_t* tokens, const int32_t* lens, int32_t* first_token) {
  const ee_config& c = s->m->cfg;
  std::vector<int> want(s->B);
  size_t total = 0;
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    want[b] = lens[b] > 0 ? lens[b] + 1 : (q.started ? max_len(s, q) : 0);
    total += lens[b];
  }
  for (size_t i = 0; i < total; ++i)
    if (tokens[i] < 0 || tokens[i] >= c.vocab) { ee_set_error("token id out of range"); return EE_ERR_ARG; }
  // capacity is checked against the pool as it will be once the restarted sequences have given their pages back
  {
    size_t freed = 0, need = 0;
    for (int b = 0; b < s->B; ++b) {
      if (lens[b] <= 0) continue;
      if (want[b] > s->max_ctx) { ee_set_error("sequence %d would need %d positions (max_ctx %d)", b, want[b], s->max_ctx); return EE_ERR_CAPACITY; }
      freed += s->seq[b].pages.size();
      need += (size_t)ceil_div(want[b], EE_PAGE);
    }
    if (need > s->free_pages.size() + freed) { ee_set_error("KV page pool exhausted"); return EE_ERR_CAPACITY; }
  }
  for (int b = 0; b < s->B; ++b) {
    if (lens[b] <= 0) continue;
    SeqState& q = s->seq[b];
    for (int pg : q.pages) s->free_pages.push_back(pg);
    q = SeqState();
  }
  reset_accounting(s);
  std::vector<size_t> off0(s->B, 0);
  std::vector<int> done(s->B, 0);
  {
    size_t o = 0;
    for (int b = 0; b < s->B; ++b) {
      off0[b] = o;
      if (lens[b] <= 0) continue;
      o += lens[b];
      EE_TRY(grow_pages(s, b, want[b]));
    }
  }
  // Passes of up to `chunk` rows.  A pass takes one contiguous piece of every prompt that still has rows, in
  // sequence order, until it is full: a long prompt fills passes by itself, short prompts share one (the weights
  // cross HBM once per pass).  A sequence's next piece comes in a later pass, after its earlier rows are cached.
  for (int ci = 0;; ++ci) {
    const int si = ci & 1;        // alternate upload slots so the host runs one pass ahead
    CallPlan p;
    p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
    int room = s->chunk;
    for (int b = 0; b < s->B && room > 0; ++b) {
      if (lens[b] <= 0 || done[b] >= lens[b]) continue;
      p.m[b] = std::min(lens[b] - done[b], room); p.p0[b] = done[b];
      room -= p.m[b];
    }
    if (room == s->chunk) break;
    EE_TRY(build_meta(s, si, p, [&](int b, int r, int& tok, int&, int&) { tok = tokens[off0[b] + done[b] + r]; }));
    EE_TRY(upload_meta(s, si));
    CallMeta mt = meta_ptrs(s, s->slot[si].d);
    PassSource from_tokens; from_tokens.tok = mt.row_tok;
    run_layers(s, 0, c.n_layers, p, mt, 0, from_tokens);
    bool head_done = false;
    for (int b = 0, row = 0; b < s->B; row += p.m[b], ++b) {
      if (!p.m[b] || done[b] + p.m[b] < lens[b]) continue;
      // the prompt ends in this pass: its last row decides the first committed token
      if (!head_done) { exit_head(s, p.M, s->n_levels); head_done = true; }
      HIP_TRY(hipMemcpyAsync(s->out_host + b, s->vtok + (row + p.m[b] - 1), sizeof(int), hipMemcpyDeviceToHost, s->st));
    }
    for (int b = 0; b < s->B; ++b) done[b] += p.m[b];
  }
  size_t off = 0;
  EE_TRY(finish(s));
  off = 0;
  for (int b = 0; b < s->B; ++b) {
    if (lens[b] <= 0) continue;
    SeqState& q = s->seq[b];
    q.C.assign(tokens + off, tokens + off + lens[b]);
    q.C.push_back(s->out_host[b]);
    settle(s, q);
    q.started = true;
    first_token[b] = s->out_host[b];
    off += lens[b];
  }
  return EE_OK;
}

extern "C" int ee_prefill(ee_session* s, const int32_t* tokens, const int32_t* lens, int32_t* first_token) {
  if (!s || !tokens || !lens || !first_token) { ee_set_error("null argument"); return EE_ERR_ARG; }
  for (int b = 0; b < s->B; ++b)
    if (lens[b] < 1) { ee_set_error("prompt %d is empty", b); return EE_ERR_ARG; }
  return prefill_impl(s, tokens, lens, first_token);
}

extern "C" int ee_prefill_seq(ee_session* s, int seq, const int32_t* tokens, int len, int32_t* first_token) {
  if (!s || !tokens || !first_token || seq < 0 || seq >= s->B) { ee_set_error("bad argument"); return EE_ERR_ARG; }
  if (len < 1) { ee_set_error("prompt is empty"); return EE_ERR_ARG; }
  std::vector<int32_t> lens(s->B, 0), first(s->B, -1);
  lens[seq] = len;
  EE_TRY(prefill_impl(s, tokens, lens.data(), first.data()));
  *first_token = first[seq];
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: vanilla greedy generation at full depth (Sec. 3.1)
// ---------------------------------------------------------------------------------------------
extern "C" int ee_seq_release(ee_session* s, int seq) {
  if (!s || seq < 0 || seq >= s->B) { ee_set_error("bad sequence index"); return EE_ERR_ARG; }
  SeqState& q = s->seq[seq];
  while (!q.pages.empty()) { s->free_pages.push_back(q.pages.back()); q.pages.pop_back(); }
  q = SeqState();
  return EE_OK;
}

extern "C" int ee_free_pages(const ee_session* s) { return s ? (int)s->free_pages.size() : -1; }

extern "C" int ee_decode_ar(ee_session* s, int n, int32_t* out) {
  if (!s || !out) { ee_set_error("null argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  if (n < 1 || n > s->max_rows) { ee_set_error("%d tokens per call do not fit max_rows %d", n, s->max_rows); return EE_ERR_ARG; }
  std::vector<int> want(s->B, 0);
  int live = 0;
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (!q.started) continue;                         // an idle slot takes no part
    if (q.n_hd || !q.V.empty() || q.cut[s->n_levels] != (int)q.C.size()) { ee_set_error("sequence %d has unverified tokens", b); return EE_ERR_STATE; }
    want[b] = (int)q.C.size() + n;
    live++;
  }
  if (!live) { ee_set_error("no sequence has a context (call ee_prefill)"); return EE_ERR_STATE; }
  EE_TRY(check_capacity(s, want));
  reset_accounting(s);
  CallPlan p;
  p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
  for (int b = 0; b < s->B; ++b) {
    if (!s->seq[b].started) continue;
    p.m[b] = 1;
    p.p0[b] = (int)s->seq[b].C.size() - 1;          // the pending token's position
    EE_TRY(grow_pages(s, b, want[b]));
  }
  EE_TRY(build_meta(s, 0, p, [&](int b, int, int& tok, int&, int&) { tok = s->seq[b].C.back(); }));
  EE_TRY(upload_meta(s, 0));
  CallMeta mt = meta_ptrs(s, s->slot[0].d);
  for (int j = 0; j < n; ++j) {       // the next token stays on the device; positions advance through pos_add
    PassSource from_tokens; from_tokens.tok = j == 0 ? mt.row_tok : s->tok_next;
    run_layers(s, 0, c.n_layers, p, mt, j, from_tokens);
    exit_head(s, p.M, s->n_levels);
    KF(KF_MISC, k_take_token(s->st, s->vtok, mt.row_seq, p.M, s->tok_next, s->draft_dev, s->max_rows, j));
  }
  int* dh = s->out_host + 2 * s->B;
  HIP_TRY(hipMemcpyAsync(dh, s->draft_dev, (size_t)s->B * s->max_rows * sizeof(int), hipMemcpyDeviceToHost, s->st));
  EE_TRY(finish(s));
  for (int b = 0; b < s->B; ++b) {
    SeqState& q = s->seq[b];
    if (!p.m[b]) { for (int j = 0; j < n; ++j) out[b * n + j] = -1; continue; }
    for (int j = 0; j < n; ++j) { out[b * n + j] = dh[b * s->max_rows + j]; q.C.push_back(dh[b * s->max_rows + j]); }
    settle(s, q);
  }
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: drafting at exit L_d
// ---------------------------------------------------------------------------------------------
static int draft_precheck(ee_session* s, int k, int rows) {
  if (k < 1 || rows > s->max_rows) { ee_set_error("draft length %d does not fit max_rows %d", k, s->max_rows); return EE_ERR_ARG; }
  std::vector<int> want(s->B, 0);
  int live = 0;
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (!q.started) continue;                         // an idle slot takes no part
    live++;
    if (q.n_hd) { ee_set_error("sequence %d already has an unverified draft block", b); return EE_ERR_STATE; }
    int nT = (int)(q.C.size() + q.V.size());
    if ((int)q.V.size() + rows + 1 > s->max_rows) { ee_set_error("tentative buffer of sequence %d would overflow max_rows", b); return EE_ERR_CAPACITY; }
    want[b] = nT - 1 + rows + 1;   // one spare position for the pending token's later catch-up
  }
  if (!live) { ee_set_error("no sequence has a context (call ee_prefill)"); return EE_ERR_STATE; }
  return check_capacity(s, want);
}

// uniform numbers of a call: host -> the session's device buffer (sampling attached)
static int upload_uniforms(ee_session* s, const float* u, size_t n, size_t at) {
  for (size_t i = 0; i < n; ++i)
    if (!(u[i] >= 0.0f && u[i] < 1.0f)) { ee_set_error("uniform numbers must lie in [0, 1)"); return EE_ERR_ARG; }
  HIP_TRY(hipMemcpyAsync(s->u_dev + at, u, n * sizeof(float), hipMemcpyHostToDevice, s->st));
  return EE_OK;
}

// u == null: arg max of p_{L_d} (Alg. 2); otherwise token j of sequence b is drawn from p_{L_d} with u[b*k + j] (App. G)
static int draft_impl(ee_session* s, int k, int32_t* draft, const float* u) {
  if (!s || !draft) { ee_set_error("null argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const int rows = k + (c.bonus_inter ? 1 : 0);
  if (u && !s->Pd) { ee_set_error("sampling buffers are not attached (ee_sampling_attach)"); return EE_ERR_STATE; }
  EE_TRY(draft_precheck(s, k, rows));
  if (u)
    for (int b = 0; b < s->B; ++b)      // an idle slot's numbers are neither read nor checked
      if (s->seq[b].started) EE_TRY(upload_uniforms(s, u + (size_t)b * k, k, (size_t)b * k));
  reset_accounting(s);
  s->need_logits = u != nullptr;
  CallPlan p;
  p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (!q.started) continue;
    p.m[b] = 1;
    p.p0[b] = (int)(q.C.size() + q.V.size()) - 1;
    EE_TRY(grow_pages(s, b, p.p0[b] + rows + 1));
  }
  EE_TRY(build_meta(s, 0, p, [&](int b, int, int& tok, int&, int& dst) {
    const SeqState& q = s->seq[b];
    tok = q.V.empty() ? q.C.back() : q.V.back();
    dst = b * s->max_rows;
  }));
  EE_TRY(upload_meta(s, 0));
  CallMeta mt = meta_ptrs(s, s->slot[0].d);
  for (int j = 0; j < rows; ++j) {
    PassSource from_tokens; from_tokens.tok = j == 0 ? mt.row_tok : s->tok_next;
    PassSink keep; keep.rows = s->Hd; keep.row_idx = mt.row_dst; keep.add = j;
    run_layers(s, 0, c.exit_draft, p, mt, j, from_tokens, keep);
    if (j < k) {
      exit_head(s, p.M, 0);
      if (u) {      // p_{L_d} of this position into the draft-distribution store, then the draw
        KF(KF_MISC, k_softmax_rows(s->st, s->LOGITS, c.vocab, s->Pd, mt.row_dst, j, p.M, c.vocab));
        KF(KF_MISC, k_draw_rows(s->st, s->Pd, s->max_rows, j, c.vocab, s->u_dev, k, mt.row_seq, p.M, s->tok_next, s->draft_dev, s->max_rows));
      } else {
        KF(KF_MISC, k_take_token(s->st, s->vtok, mt.row_seq, p.M, s->tok_next, s->draft_dev, s->max_rows, j));
      }
    }
  }
  s->need_logits = false;
  int* dh = s->out_host + 2 * s->B;
  HIP_TRY(hipMemcpyAsync(dh, s->draft_dev, (size_t)s->B * s->max_rows * sizeof(int), hipMemcpyDeviceToHost, s->st));
  EE_TRY(finish(s));
  for (int b = 0; b < s->B; ++b) {
    SeqState& q = s->seq[b];
    if (!p.m[b]) { for (int j = 0; j < k; ++j) draft[b * k + j] = -1; continue; }
    q.S.assign(dh + b * s->max_rows, dh + b * s->max_rows + k);
    q.n_hd = rows;
    q.sampled = u != nullptr;
    q.len[0] = p.p0[b] + rows;
    for (int j = 0; j < k; ++j) draft[b * k + j] = q.S[j];
  }
  return EE_OK;
}

extern "C" int ee_draft(ee_session* s, int k, int32_t* draft) { return draft_impl(s, k, draft, nullptr); }

extern "C" int ee_draft_sample(ee_session* s, int k, const float* u, int32_t* draft) {
  if (!u) { ee_set_error("null argument"); return EE_ERR_ARG; }
  return draft_impl(s, k, draft, u);
}

extern "C" int ee_draft_inject(ee_session* s, int k, const int32_t* draft) {
  if (!s || !draft) { ee_set_error("null argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const int rows = k + (c.bonus_inter ? 1 : 0);
  EE_TRY(draft_precheck(s, k, rows));
  for (int i = 0; i < s->B * k; ++i)
    if (s->seq[i / k].started && (draft[i] < 0 || draft[i] >= c.vocab)) { ee_set_error("draft token out of range"); return EE_ERR_ARG; }
  reset_accounting(s);
  CallPlan p;
  p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (!q.started) continue;                         // an idle slot's entries of `draft` are ignored
    p.m[b] = rows;
    p.p0[b] = (int)(q.C.size() + q.V.size()) - 1;
    EE_TRY(grow_pages(s, b, p.p0[b] + rows + 1));
  }
  EE_TRY(build_meta(s, 0, p, [&](int b, int r, int& tok, int&, int& dst) {
    const SeqState& q = s->seq[b];
    tok = r == 0 ? (q.V.empty() ? q.C.back() : q.V.back()) : draft[b * k + r - 1];
    dst = b * s->max_rows + r;
  }));
  EE_TRY(upload_meta(s, 0));
  CallMeta mt = meta_ptrs(s, s->slot[0].d);
  PassSource from_tokens; from_tokens.tok = mt.row_tok;
  PassSink keep; keep.rows = s->Hd; keep.row_idx = mt.row_dst;
  run_layers(s, 0, c.exit_draft, p, mt, 0, from_tokens, keep);
  HIP_TRY(hipGetLastError());
  for (int b = 0; b < s->B; ++b) {
    SeqState& q = s->seq[b];
    if (!p.m[b]) continue;
    q.S.assign(draft + b * k, draft + b * k + k);
    q.n_hd = rows;
    q.sampled = false;
    q.len[0] = p.p0[b] + rows;
  }
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// Scratch of one call in the library's own static device array, for callers that cannot allocate
// ---------------------------------------------------------------------------------------------
// What a verify call needs beyond its inputs, outputs and the session's state -- the attention's split partials, the
// exit head's (max, arg max) tile partials, the deferred-RMSNorm partial sums and factors, the K-share partials of
// the row-tiled GEMM -- normally sits in the caller's session arena.  ee_verify_intermediate_static places it in
// this array instead.  Every GPU holds its own copy of the array at its own address, found once per device with
// hipGetSymbolAddress; the array's name itself is only a host-side stand-in and never goes to a kernel.
#define EE_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
#define EE_STATIC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[EE_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[EE_STATIC_MAX_DEVICES] = {nullptr};
static std::mutex g_scratch_mutex;

static int static_scratch_base(char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= EE_STATIC_MAX_DEVICES) { ee_set_error("device %d outside the static scratch table", dev); return EE_ERR_HIP; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) { ee_set_error("static scratch has no device address"); return EE_ERR_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = (char*)g_scratch_ptr[dev];
  return EE_OK;
}

// the session's scratch pointers, swapped for the length of one call and put back whatever happens
struct ScratchSwap {
  ee_session* s;
  float *part_o, *part_ml, *pmax, *ssq, *gemm_part, *inv_rms;
  int* pidx;
  explicit ScratchSwap(ee_session* s_) : s(s_), part_o(s_->part_o), part_ml(s_->part_ml), pmax(s_->pmax), ssq(s_->ssq),
                                         gemm_part(s_->gemm_part), inv_rms(s_->inv_rms), pidx(s_->pidx) {}
  ~ScratchSwap() {
    s->part_o = part_o; s->part_ml = part_ml; s->pmax = pmax; s->ssq = ssq; s->gemm_part = gemm_part; s->inv_rms = inv_rms;
    s->pidx = pidx;
  }
};

// Lay the scratch of the call with plan p (pass over layers [l0, l1), then the shared exit head) out in the static
// array and point the session at it.  The split plan is the one the session arena would have given (its capacity
// only enters as a number), so the call computes exactly what ee_verify_intermediate computes.
static int place_scratch_static(ee_session* s, const CallPlan& p) {
  const ee_model* m = s->m;
  const ee_config& c = m->cfg;
  if (!m->bf16) return EE_OK;                       // the fp32 kernels use no scratch
  char* base = nullptr;
  EE_TRY(static_scratch_base(&base));
  AttnScratch scr;
  int nsplit = 1;
  (void)attention_plan(s, p, 0, scr, &nsplit);
  Carver cv{base};
  const size_t slots = (size_t)p.total_qt * c.n_kv_heads * nsplit;
  float* part_o = cv.take<float>(slots * 16 * c.head_dim);
  float* part_ml = cv.take<float>(slots * 32);
  const size_t pstride = (size_t)ceil_div(p.M, 16) * 16;
  float* pmax = cv.take<float>((size_t)m->head.ntiles() * pstride);
  int* pidx = cv.take<int>((size_t)m->head.ntiles() * pstride);
  float* ssq = cv.take<float>((size_t)ceil_div(c.d_model, 16) * s->Mp);
  float* inv_rms = cv.take<float>(512);
  float* gemm_part = nullptr;
  if (p.M > 16) {                                   // the row-tiled GEMM may run: room for its K shares
    size_t gp = 0;
    for (const MatLoc* ml : {&m->L[0].qkv, &m->L[0].o, &m->L[0].gu, &m->L[0].down, &m->head, &m->auxA[0], &m->auxB[0]})
      if (ml->Np > 0) gp = std::max(gp, bf16_gemm_rows_scratch_floats(ml->ntiles(), ml->ktiles()));
    gemm_part = cv.take<float>(gp);
  }
  if (cv.cur > EE_STATIC_SCRATCH_BYTES) {
    ee_set_error("this call needs %zu bytes of scratch, the static array holds %zu: use ee_verify_intermediate", cv.cur,
                 (size_t)EE_STATIC_SCRATCH_BYTES);
    return EE_ERR_CAPACITY;
  }
  s->part_o = part_o; s->part_ml = part_ml; s->pmax = pmax; s->pidx = pidx; s->ssq = ssq; s->inv_rms = inv_rms;
  s->gemm_part = gemm_part;
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: intermediate verification at exit L_i
// ---------------------------------------------------------------------------------------------
// u_acc == null: LeadingSubstringVerify on arg max tokens (Alg. 2); otherwise the acceptance rule of App. G with the
// uniform numbers u_acc [batch, u_stride] (one per draft token) and u_res [batch] (the replacement / next-token draw)
static int verify_intermediate_impl(ee_session* s, int32_t* n_accept, int32_t* next_token, const float* u_acc, int u_stride,
                                    const float* u_res, bool static_scratch = false) {
  if (!s || !n_accept || !next_token) { ee_set_error("null argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const bool rs = u_acc != nullptr;
  ScratchSwap restore(s);
  CallPlan p;
  p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
  int any = 0;
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (!q.n_hd) continue;
    if (rs && (!q.sampled || q.n_pi != (int)q.V.size())) {
      ee_set_error("sequence %d: the pending block or the tentative tokens were not produced by the sampling calls", b);
      return EE_ERR_STATE;
    }
    p.m[b] = q.n_hd; p.p0[b] = (int)(q.C.size() + q.V.size()) - 1;
    any++;
  }
  if (!any) { ee_set_error("no draft block is pending"); return EE_ERR_STATE; }
  if (rs) {
    if (!s->Pd) { ee_set_error("sampling buffers are not attached (ee_sampling_attach)"); return EE_ERR_STATE; }
    if (u_stride < 1 || u_stride > s->max_rows) { ee_set_error("bad stride of the uniform numbers"); return EE_ERR_ARG; }
    for (int b = 0; b < s->B; ++b) {                         // idle sequences' numbers are neither read nor checked
      if (!p.m[b]) continue;
      if ((int)s->seq[b].S.size() > u_stride) { ee_set_error("sequence %d: %d draft tokens need as many uniform numbers (u_stride %d)", b, (int)s->seq[b].S.size(), u_stride); return EE_ERR_ARG; }
      EE_TRY(upload_uniforms(s, u_acc + (size_t)b * u_stride, u_stride, (size_t)b * s->max_rows));
      EE_TRY(upload_uniforms(s, u_res + b, 1, (size_t)s->B * s->max_rows + b));
    }
  }
  reset_accounting(s);
  EE_TRY(build_meta(s, 0, p, [&](int b, int r, int&, int& src, int& dst) {
    src = b * s->max_rows + r;                               // H_d row
    dst = b * s->max_rows + (int)s->seq[b].V.size() + r;     // H_i row
  }));
  if (static_scratch) EE_TRY(place_scratch_static(s, p));
  int* h = s->slot[0].h;
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (!p.m[b]) continue;
    h[s->o_n_cand + b] = (int)q.S.size();
    for (size_t j = 0; j < q.S.size(); ++j) h[s->o_cand + (size_t)b * s->cand_stride + j] = q.S[j];
  }
  EE_TRY(upload_meta(s, 0));
  CallMeta mt = meta_ptrs(s, s->slot[0].d);
  PassSource kept; kept.rows = s->Hd; kept.row_idx = mt.row_src;       // a1: consume buffered H_d
  PassSink keep; keep.rows = s->Hi; keep.row_idx = mt.row_dst;          // keep L_i hidden rows
  run_layers(s, c.exit_draft, c.exit_inter, p, mt, 0, kept, keep);
  s->need_logits = rs;
  exit_head(s, p.M, 1);
  s->need_logits = false;
  if (rs) {
    KF(KF_MISC, k_softmax_rows(s->st, s->LOGITS, c.vocab, s->LOGITS, nullptr, 0, p.M, c.vocab));          // p_{L_i}, in place
    KF(KF_ACCEPT, k_rs_accept(s->st, s->LOGITS, s->Pd, s->max_rows, c.vocab, mt, s->cand_stride, s->B, s->u_dev, s->max_rows, s->out_dev));
    KF(KF_ACCEPT, k_rs_draw(s->st, s->LOGITS, s->Pd, s->max_rows, c.vocab, mt, s->B, s->out_dev, s->u_dev + (size_t)s->B * s->max_rows,
                            s->out_dev + s->B));
    KF(KF_COPY, k_copy_rows(s->st, s->Pi, mt.row_dst, 0, s->LOGITS, nullptr, p.M, c.vocab));  // p_{L_i} of the rows that may stay
  } else {
    KF(KF_ACCEPT, k_accept(s->st, s->vtok, mt, s->cand_stride, s->B, s->out_dev, s->out_dev + s->B));
  }
  HIP_TRY(hipMemcpyAsync(s->out_host, s->out_dev, 2 * (size_t)s->B * sizeof(int), hipMemcpyDeviceToHost, s->st));
  EE_TRY(finish(s));
  for (int b = 0; b < s->B; ++b) {
    SeqState& q = s->seq[b];
    n_accept[b] = s->out_host[b]; next_token[b] = s->out_host[s->B + b];
    if (!p.m[b]) continue;
    const int a = n_accept[b];
    q.V.insert(q.V.end(), q.S.begin(), q.S.begin() + a);
    int keep = a;
    if (a < p.m[b]) { q.V.push_back(next_token[b]); keep = a + 1; }
    q.len[0] = q.len[1] = p.p0[b] + keep;                    // prune rejected rows (lengths only)
    q.n_hd = 0; q.S.clear(); q.sampled = false;
    if (rs) q.n_pi = (int)q.V.size();
    trim_pages(s, b);
  }
  return EE_OK;
}

extern "C" int ee_verify_intermediate(ee_session* s, int32_t* n_accept, int32_t* next_token) {
  return verify_intermediate_impl(s, n_accept, next_token, nullptr, 0, nullptr);
}

extern "C" int ee_verify_intermediate_static(ee_session* s, int32_t* n_accept, int32_t* next_token) {
  if (s && s->time_kernels) { ee_set_error("kernel timing creates events: switch it off for the call that allocates nothing"); return EE_ERR_STATE; }
  return verify_intermediate_impl(s, n_accept, next_token, nullptr, 0, nullptr, true);
}

extern "C" int ee_verify_intermediate_rs(ee_session* s, const float* u_acc, int u_stride, const float* u_res, int32_t* n_accept,
                                         int32_t* next_token) {
  if (!u_acc || !u_res) { ee_set_error("null argument"); return EE_ERR_ARG; }
  return verify_intermediate_impl(s, n_accept, next_token, u_acc, u_stride, u_res);
}

// ---------------------------------------------------------------------------------------------
// C ABI: verification at the levels above L_i -- full verification at L_f (Alg. 2) and, with further
// verifier exits, the levels in between (the hierarchy of the paper's Future Work section)
// ---------------------------------------------------------------------------------------------
static float* level_rows(const ee_session* s, int j) { return j == 0 ? s->Hd : (j == 1 ? s->Hi : s->Hup[j - 2]); }
// stored distributions of the tokens in level j's buffer (0: the draft block's)
static float* level_dist(const ee_session* s, int j) { return j == 0 ? s->Pd : (j == 1 ? s->Pi : s->Pup[j - 2]); }

// Level j (2 <= j <= n) takes the buffer of level j-1 as its draft: V for j = 2, else the tail C[cut[j]..) (every
// buffer below it must be empty).  The buffered rows of exit j-1 plus, in bonus mode, one row for the buffer's
// last token (through the groups below first) run through layer group j; LeadingSubstringVerify keeps the
// matching prefix and exit j's own next token.  What is kept joins level j's buffer (the committed tokens at
// the last level); the KV lengths of the groups up to j are pruned to it.
static int verify_upper_impl(ee_session* s, int level, const uint8_t* active, int32_t* n_accept, int32_t* next_token,
                             int32_t* committed, int32_t* n_committed, const float* u_acc, int u_stride, const float* u_res) {
  if (!s || !n_accept || !next_token || !committed || !n_committed) { ee_set_error("null argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const int n = s->n_levels, j = level;
  if (j < 2 || j > n) { ee_set_error("level must be 2..%d", n); return EE_ERR_ARG; }
  const std::vector<int>& ex = s->m->exits;
  const int bonus = c.bonus_full ? 1 : 0;
  const bool rs = u_acc != nullptr;
  std::vector<int> act(s->B, 0), m_src(s->B, 0), base(s->B, 0);
  int any = 0;
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    if (active && !active[b]) continue;
    // base: tokens already past level j; m_src: tokens of the buffer below it
    base[b] = j == 2 ? (int)q.C.size() : q.cut[j];
    m_src[b] = j == 2 ? (int)q.V.size() : (int)q.C.size() - q.cut[j];
    if (!q.started || m_src[b] == 0) continue;
    if (q.n_hd) { ee_set_error("sequence %d still has an unverified draft block", b); return EE_ERR_STATE; }
    if (j > 2 && (!q.V.empty() || q.cut[j - 1] != (int)q.C.size())) {
      ee_set_error("sequence %d: the buffers below level %d must be verified first", b, j - 1); return EE_ERR_STATE;
    }
    if (rs && (j == 2 ? q.n_pi : q.n_pu[j - 3]) != m_src[b]) {
      ee_set_error("sequence %d: the tokens waiting below level %d were not produced by the sampling calls", b, j);
      return EE_ERR_STATE;
    }
    // level j's buffer is level j+1's draft: its rows sit in a [max_rows] slab per sequence together with the
    // catch-up row that level j+1 appends behind them, so it may hold max_rows - bonus tokens at most
    if (j < n && (q.cut[j] - q.cut[j + 1]) + m_src[b] + bonus > s->max_rows - bonus) {
      ee_set_error("level %d buffer of sequence %d would exceed %d tokens", j, b, s->max_rows - bonus); return EE_ERR_CAPACITY;
    }
    if (m_src[b] + bonus > s->max_rows) {      // (cannot happen given the bound above and the one on V in the draft calls)
      ee_set_error("sequence %d: %d rows do not fit max_rows", b, m_src[b] + bonus); return EE_ERR_CAPACITY;
    }
    act[b] = 1; any++;
  }
  if (!any) { ee_set_error("no sequence has tentative tokens to verify"); return EE_ERR_STATE; }
  if (rs) {
    if (!s->Pi) { ee_set_error("sampling buffers are not attached (ee_sampling_attach)"); return EE_ERR_STATE; }
    if (u_stride < 1 || u_stride > s->max_rows) { ee_set_error("bad stride of the uniform numbers"); return EE_ERR_ARG; }
    for (int b = 0; b < s->B; ++b) {                         // idle sequences' numbers are neither read nor checked
      if (!act[b]) continue;
      if (m_src[b] > u_stride) { ee_set_error("sequence %d: %d tentative tokens need as many uniform numbers (u_stride %d)", b, m_src[b], u_stride); return EE_ERR_ARG; }
      EE_TRY(upload_uniforms(s, u_acc + (size_t)b * u_stride, u_stride, (size_t)b * s->max_rows));
      EE_TRY(upload_uniforms(s, u_res + b, 1, (size_t)s->B * s->max_rows + b));
    }
  }
  auto src_tok = [&](int b, int i) { const SeqState& q = s->seq[b]; return j == 2 ? q.V[i] : q.C[q.cut[j] + i]; };
  float* rows_below = level_rows(s, j - 1);
  reset_accounting(s);
  if (bonus) {
    // the buffer's last token owns no hidden state yet: one row per sequence through the groups below level j
    CallPlan p;
    p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
    for (int b = 0; b < s->B; ++b) {
      if (!act[b]) continue;
      p.m[b] = 1; p.p0[b] = base[b] + m_src[b] - 1;
      EE_TRY(grow_pages(s, b, p.p0[b] + 1));
    }
    EE_TRY(build_meta(s, 1, p, [&](int b, int, int& tok, int&, int& dst) {
      tok = src_tok(b, m_src[b] - 1);
      dst = b * s->max_rows + m_src[b];
    }));
    EE_TRY(upload_meta(s, 1));
    CallMeta mt = meta_ptrs(s, s->slot[1].d);
    PassSource from_tokens; from_tokens.tok = mt.row_tok;
    PassSink keep; keep.rows = rows_below; keep.row_idx = mt.row_dst;
    run_layers(s, 0, ex[j - 1], p, mt, 0, from_tokens, keep);
  }
  CallPlan p;
  p.m.assign(s->B, 0); p.p0.assign(s->B, 0);
  for (int b = 0; b < s->B; ++b) {
    if (!act[b]) continue;
    p.m[b] = m_src[b] + bonus; p.p0[b] = base[b] - 1;
  }
  EE_TRY(build_meta(s, 0, p, [&](int b, int r, int&, int& src, int& dst) {
    src = b * s->max_rows + r;
    dst = b * s->max_rows + (j < n ? s->seq[b].cut[j] - s->seq[b].cut[j + 1] : 0) + r;     // row of level j's own buffer
  }));
  int* h = s->slot[0].h;
  for (int b = 0; b < s->B; ++b) {
    if (!act[b]) continue;
    h[s->o_n_cand + b] = m_src[b];
    for (int i = 0; i < m_src[b]; ++i) h[s->o_cand + (size_t)b * s->cand_stride + i] = src_tok(b, i);
  }
  EE_TRY(upload_meta(s, 0));
  CallMeta mt = meta_ptrs(s, s->slot[0].d);
  PassSource kept; kept.rows = rows_below; kept.row_idx = mt.row_src;  // consume the buffered rows
  PassSink keep;
  if (j < n) { keep.rows = level_rows(s, j); keep.row_idx = mt.row_dst; }   // keep exit j's rows
  run_layers(s, ex[j - 1], ex[j], p, mt, 0, kept, keep);
  s->need_logits = rs;
  exit_head(s, p.M, j);
  s->need_logits = false;
  if (rs) {      // a further stage of App. G: the buffer below, distributed as exit j-1's p, is the draft; exit j's p the target
    const float* q_below = level_dist(s, j - 1);
    KF(KF_MISC, k_softmax_rows(s->st, s->LOGITS, c.vocab, s->LOGITS, nullptr, 0, p.M, c.vocab));
    KF(KF_ACCEPT, k_rs_accept(s->st, s->LOGITS, q_below, s->max_rows, c.vocab, mt, s->cand_stride, s->B, s->u_dev, s->max_rows, s->out_dev));
    KF(KF_ACCEPT, k_rs_draw(s->st, s->LOGITS, q_below, s->max_rows, c.vocab, mt, s->B, s->out_dev, s->u_dev + (size_t)s->B * s->max_rows,
                            s->out_dev + s->B));
    // exit j's distributions of the rows that may stay: the law of the tokens that wait for exit j+1
    if (j < n) KF(KF_COPY, k_copy_rows(s->st, level_dist(s, j), mt.row_dst, 0, s->LOGITS, nullptr, p.M, c.vocab));
  } else {
    KF(KF_ACCEPT, k_accept(s->st, s->vtok, mt, s->cand_stride, s->B, s->out_dev, s->out_dev + s->B));
  }
  HIP_TRY(hipMemcpyAsync(s->out_host, s->out_dev, 2 * (size_t)s->B * sizeof(int), hipMemcpyDeviceToHost, s->st));
  EE_TRY(finish(s));
  for (int b = 0; b < s->B; ++b) {
    SeqState& q = s->seq[b];
    n_accept[b] = s->out_host[b]; next_token[b] = s->out_host[s->B + b];
    n_committed[b] = 0;
    if (!act[b]) continue;
    const int f = n_accept[b];
    int32_t* out = committed + (size_t)b * (s->max_rows + 1);
    int cnt = 0;
    for (int i = 0; i < f; ++i) out[cnt++] = src_tok(b, i);
    if (f < p.m[b]) out[cnt++] = next_token[b];
    n_committed[b] = cnt;
    if (j > 2) q.C.resize(q.cut[j]);
    const int held = j < n ? q.cut[j] - q.cut[j + 1] : 0;      // tokens level j's buffer held before this call
    q.C.insert(q.C.end(), out, out + cnt);
    q.V.clear(); q.n_pi = 0;
    for (int i = 2; i < j; ++i) q.n_pu[i - 2] = 0;
    if (j < n) q.n_pu[j - 2] = (rs && q.n_pu[j - 2] == held) ? held + cnt : -1;   // -1: holds tokens without a stored law
    for (int g = 2; g <= j; ++g) q.cut[g] = (int)q.C.size();
    for (int g = 0; g <= j; ++g) q.len[g] = (int)q.C.size() - 1;
    trim_pages(s, b);
  }
  return EE_OK;
}

extern "C" int ee_verify_full(ee_session* s, const uint8_t* active, int32_t* n_accept, int32_t* next_token,
                              int32_t* committed, int32_t* n_committed) {
  if (!s) { ee_set_error("null argument"); return EE_ERR_ARG; }
  return verify_upper_impl(s, s->n_levels, active, n_accept, next_token, committed, n_committed, nullptr, 0, nullptr);
}

extern "C" int ee_verify_level(ee_session* s, int level, const uint8_t* active, int32_t* n_accept, int32_t* next_token,
                               int32_t* moved, int32_t* n_moved) {
  return verify_upper_impl(s, level, active, n_accept, next_token, moved, n_moved, nullptr, 0, nullptr);
}

extern "C" int ee_verify_level_rs(ee_session* s, int level, const uint8_t* active, const float* u_acc, int u_stride, const float* u_res,
                                  int32_t* n_accept, int32_t* next_token, int32_t* moved, int32_t* n_moved) {
  if (!s || !u_acc || !u_res) { ee_set_error("null argument"); return EE_ERR_ARG; }
  return verify_upper_impl(s, level, active, n_accept, next_token, moved, n_moved, u_acc, u_stride, u_res);
}

extern "C" int ee_n_levels(const ee_session* s) { return s ? s->n_levels : -1; }

extern "C" int ee_verify_full_rs(ee_session* s, const uint8_t* active, const float* u_acc, int u_stride, const float* u_res,
                                 int32_t* n_accept, int32_t* next_token, int32_t* committed, int32_t* n_committed) {
  if (!s || !u_acc || !u_res) { ee_set_error("null argument"); return EE_ERR_ARG; }
  return verify_upper_impl(s, s->n_levels, active, n_accept, next_token, committed, n_committed, u_acc, u_stride, u_res);
}

// ---------------------------------------------------------------------------------------------
// C ABI: buffers of the rejection-sampling acceptance (caller-owned, like the session arena)
// ---------------------------------------------------------------------------------------------
static size_t sampling_floats(const ee_session* s) {
  const size_t rows = (size_t)s->B * s->max_rows;
  return (size_t)s->n_levels * rows * s->m->cfg.vocab + rows + s->B + 64;     // one store per level below L_f, and the uniform numbers
}
extern "C" size_t ee_sampling_bytes(const ee_session* s) { return s ? sampling_floats(s) * sizeof(float) : 0; }

extern "C" int ee_sampling_attach(ee_session* s, void* dev_arena, size_t arena_bytes) {
  if (!s || !dev_arena || ((uintptr_t)dev_arena & 255)) { ee_set_error("arena must be non-null and 256-byte aligned"); return EE_ERR_ARG; }
  if (arena_bytes < sampling_floats(s) * sizeof(float)) { ee_set_error("sampling arena too small"); return EE_ERR_ARG; }
  const size_t rows = (size_t)s->B * s->max_rows;
  float* f = (float*)dev_arena;
  const size_t store = rows * s->m->cfg.vocab;
  s->Pd = f; s->Pi = f + store;
  for (int j = 2; j < s->n_levels; ++j) s->Pup[j - 2] = f + (size_t)j * store;
  s->u_dev = f + (size_t)s->n_levels * store;
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: rollback
// ---------------------------------------------------------------------------------------------
extern "C" int kv_rollback(ee_session* s, int seq, int group_mask, int new_len) {
  if (!s || seq < 0 || seq >= s->B) { ee_set_error("bad sequence index"); return EE_ERR_ARG; }
  SeqState& q = s->seq[seq];
  if (!q.started) { ee_set_error("sequence %d has no context", seq); return EE_ERR_STATE; }
  const int n = s->n_levels;
  const int m12 = group_mask & 3;
  if (m12 != 0 && m12 != 3) { ee_set_error("G1 and G2 roll back together"); return EE_ERR_ARG; }
  if (group_mask & ~((1 << (n + 1)) - 1)) { ee_set_error("bad group mask"); return EE_ERR_ARG; }
  if (m12 == 0) {
    for (int g = 2; g <= n; ++g)
      if ((group_mask & (1 << g)) && new_len != q.len[g]) { ee_set_error("the groups above G2 cannot roll back alone"); return EE_ERR_ARG; }
    q.n_hd = 0; q.S.clear(); q.sampled = false; q.len[0] = q.len[1];
    trim_pages(s, seq);
    return EE_OK;
  }
  if (new_len < 0 || new_len > q.len[1]) { ee_set_error("rollback can only shrink (len %d -> %d)", q.len[1], new_len); return EE_ERR_ARG; }
  const int nT = new_len + 1;
  if (nT <= (int)q.C.size()) {
    for (int g = 2; g <= n; ++g)
      if (new_len < q.len[g] && !(group_mask & (1 << g))) {
        ee_set_error("cut reaches tokens that group %d has seen: it must roll back too", g + 1); return EE_ERR_ARG;
      }
    q.C.resize(nT); q.V.clear();
    for (int g = 2; g <= n; ++g) { q.len[g] = std::min(q.len[g], new_len); q.cut[g] = std::min(q.cut[g], nT); }
  } else {
    q.V.resize(nT - q.C.size());
  }
  q.n_pi = std::min(q.n_pi, (int)q.V.size());
  for (int g = 2; g < n; ++g) q.n_pu[g - 2] = std::min(q.n_pu[g - 2], q.cut[g] - q.cut[g + 1]);
  q.n_hd = 0; q.S.clear(); q.sampled = false;
  q.len[0] = q.len[1] = new_len;
  trim_pages(s, seq);
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: introspection
// ---------------------------------------------------------------------------------------------
extern "C" int ee_get_lengths(const ee_session* s, int32_t* out) {
  if (!s || !out) { ee_set_error("null argument"); return EE_ERR_ARG; }
  const int G = s->n_levels + 1;
  for (int b = 0; b < s->B; ++b) for (int g = 0; g < G; ++g) out[b * G + g] = s->seq[b].len[g];
  return EE_OK;
}
extern "C" int ee_get_counts(const ee_session* s, int32_t* nc, int32_t* nv) {
  if (!s || !nc || !nv) { ee_set_error("null argument"); return EE_ERR_ARG; }
  for (int b = 0; b < s->B; ++b) {
    const SeqState& q = s->seq[b];
    nc[b] = q.cut[s->n_levels]; nv[b] = (int)(q.C.size() + q.V.size()) - nc[b];
  }
  return EE_OK;
}
extern "C" int ee_get_tokens(const ee_session* s, int seq, int32_t* out, int cap, int32_t* n_out) {
  if (!s || !out || !n_out || seq < 0 || seq >= s->B) { ee_set_error("bad argument"); return EE_ERR_ARG; }
  const SeqState& q = s->seq[seq];
  int n = (int)(q.C.size() + q.V.size());
  if (n > cap) { ee_set_error("buffer too small: %d tokens", n); return EE_ERR_CAPACITY; }
  std::copy(q.C.begin(), q.C.end(), out);
  std::copy(q.V.begin(), q.V.end(), out + q.C.size());
  *n_out = n;
  return EE_OK;
}
extern "C" int ee_debug_enable_logits(ee_session* s, int on) {
  if (!s) { ee_set_error("null session"); return EE_ERR_ARG; }
  s->debug_logits = on != 0;
  return EE_OK;
}
extern "C" int ee_debug_last_logits(ee_session* s, float* host_out, int max_rows, int32_t* n_rows) {
  if (!s || !host_out || !n_rows) { ee_set_error("null argument"); return EE_ERR_ARG; }
  if (s->m->bf16 && !s->debug_logits) { ee_set_error("logits were not kept: call ee_debug_enable_logits first"); return EE_ERR_STATE; }
  int n = std::min(max_rows, s->last_rows);
  HIP_TRY(hipMemcpy(host_out, s->LOGITS, (size_t)n * s->m->cfg.vocab * sizeof(float), hipMemcpyDeviceToHost));
  *n_rows = n;
  return EE_OK;
}
extern "C" int ee_debug_last_hidden(ee_session* s, float* host_out, int max_rows, int32_t* n_rows) {
  if (!s || !host_out || !n_rows) { ee_set_error("null argument"); return EE_ERR_ARG; }
  int n = std::min(max_rows, s->last_rows);
  HIP_TRY(hipMemcpy(host_out, s->X, (size_t)n * s->m->cfg.d_model * sizeof(float), hipMemcpyDeviceToHost));
  *n_rows = n;
  return EE_OK;
}
extern "C" int ee_debug_read_dist(ee_session* s, int which, int seq, int row0, int n, float* host_out) {
  if (!s || !host_out || seq < 0 || seq >= s->B || (which != 0 && which != 1)) { ee_set_error("bad argument"); return EE_ERR_ARG; }
  if (!s->Pd) { ee_set_error("sampling buffers are not attached"); return EE_ERR_STATE; }
  if (row0 < 0 || n < 0 || row0 + n > s->max_rows) { ee_set_error("rows outside the store"); return EE_ERR_ARG; }
  const size_t V = s->m->cfg.vocab;
  const float* src = (which == 0 ? s->Pd : s->Pi) + ((size_t)seq * s->max_rows + row0) * V;
  HIP_TRY(hipStreamSynchronize(s->st));
  HIP_TRY(hipMemcpy(host_out, src, (size_t)n * V * sizeof(float), hipMemcpyDeviceToHost));
  return EE_OK;
}

static int upload_pages(ee_session* s, int seq) {
  const SeqState& q = s->seq[seq];
  if (q.pages.empty()) return EE_OK;
  HIP_TRY(hipMemcpy(s->page_scratch, q.pages.data(), q.pages.size() * sizeof(int), hipMemcpyHostToDevice));
  return EE_OK;
}
extern "C" int ee_debug_read_kv(ee_session* s, int seq, int layer, int pos0, int n, float* k_out, float* v_out) {
  if (!s || !k_out || !v_out || seq < 0 || seq >= s->B) { ee_set_error("bad argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const SeqState& q = s->seq[seq];
  if (layer < 0 || layer >= c.n_layers || pos0 < 0 || n < 0 || pos0 + n > (int)q.pages.size() * EE_PAGE) { ee_set_error("KV range not owned by the sequence"); return EE_ERR_ARG; }
  if (!n) return EE_OK;
  size_t cnt = (size_t)n * c.n_kv_heads * c.head_dim;
  float* stage = nullptr;
  HIP_TRY(hipMalloc(&stage, 2 * cnt * sizeof(float)));
  int rc = upload_pages(s, seq);
  if (rc == EE_OK) {
    k_read_kv(s->st, s->m->bf16, s->kv, s->page_scratch, layer, pos0, n, s->n_pages, c.n_kv_heads, c.head_dim, stage, stage + cnt);
    hipError_t e = hipStreamSynchronize(s->st);
    if (e == hipSuccess) e = hipMemcpy(k_out, stage, cnt * sizeof(float), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(v_out, stage + cnt, cnt * sizeof(float), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { ee_set_error("read_kv: %s", hipGetErrorString(e)); rc = EE_ERR_HIP; }
  }
  (void)hipFree(stage);
  return rc;
}
extern "C" int ee_debug_write_kv(ee_session* s, int seq, int layer, int pos0, int n, const float* k_in, const float* v_in) {
  if (!s || !k_in || !v_in || seq < 0 || seq >= s->B) { ee_set_error("bad argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const SeqState& q = s->seq[seq];
  if (layer < 0 || layer >= c.n_layers || pos0 < 0 || n < 0 || pos0 + n > (int)q.pages.size() * EE_PAGE) { ee_set_error("KV range not owned by the sequence"); return EE_ERR_ARG; }
  if (!n) return EE_OK;
  size_t cnt = (size_t)n * c.n_kv_heads * c.head_dim;
  float* stage = nullptr;
  HIP_TRY(hipMalloc(&stage, 2 * cnt * sizeof(float)));
  int rc = upload_pages(s, seq);
  if (rc == EE_OK) {
    hipError_t e = hipMemcpy(stage, k_in, cnt * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(stage + cnt, v_in, cnt * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) {
      k_write_kv(s->st, s->m->bf16, s->kv, s->page_scratch, layer, pos0, n, s->n_pages, c.n_kv_heads, c.head_dim, stage, stage + cnt);
      e = hipStreamSynchronize(s->st);
    }
    if (e != hipSuccess) { ee_set_error("write_kv: %s", hipGetErrorString(e)); rc = EE_ERR_HIP; }
  }
  (void)hipFree(stage);
  return rc;
}

extern "C" int ee_debug_poison_dead_kv(ee_session* s, int seq) {
  if (!s || seq < 0 || seq >= s->B) { ee_set_error("bad argument"); return EE_ERR_ARG; }
  const ee_config& c = s->m->cfg;
  const SeqState& q = s->seq[seq];
  EE_TRY(upload_pages(s, seq));
  std::vector<int> bounds = {0};
  bounds.insert(bounds.end(), s->m->exits.begin(), s->m->exits.end());
  for (int g = 0; g <= s->n_levels; ++g)
    k_fill_nan_dead_kv(s->st, s->m->bf16, s->kv, s->page_scratch, (int)q.pages.size(), q.len[g], bounds[g], bounds[g + 1],
                       s->n_pages, c.n_kv_heads, c.head_dim);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(s->st));
  return EE_OK;
}
extern "C" int ee_debug_gemm_row_blocks(int row_tiles) {
  if (row_tiles == 1000 || row_tiles == 1016) {      // wide matrices at 257..512 rows: one block of 32 row tiles / two of 16
    g_rows_wide = row_tiles == 1016;
    return EE_OK;
  }
  if (row_tiles != -1 && row_tiles != 0 && row_tiles != 4 && row_tiles != 8 && row_tiles != 16 && row_tiles != 104 && row_tiles != 108) {
    ee_set_error("row_tiles must be -1, 0, 4, 8, 16, 104, 108, 1000 or 1016");
    return EE_ERR_ARG;
  }
  if (row_tiles == -1) g_rows_wide = 1;
  g_rows_blocks_override = row_tiles;
  return EE_OK;
}

extern "C" int ee_debug_attention_split_pages(int pages) {
  if (pages < 0 || pages > 65536) { ee_set_error("pages per split must be 0 (built-in choice) or positive"); return EE_ERR_ARG; }
  g_attn_pages_override = pages;
  return EE_OK;
}

extern "C" int ee_debug_time_kernels(ee_session* s, int on) {
  if (!s) { ee_set_error("null session"); return EE_ERR_ARG; }
  s->time_kernels = on != 0;
  return EE_OK;
}
extern "C" int ee_debug_kernel_times(ee_session* s, int32_t* n_families, const char** names, float* ms, int32_t* launches) {
  if (!s || !n_families || !names || !ms || !launches) { ee_set_error("null argument"); return EE_ERR_ARG; }
  HIP_TRY(hipStreamSynchronize(s->st));
  for (int f = 0; f < KF_COUNT; ++f) { names[f] = kFamName[f]; ms[f] = 0.f; launches[f] = s->launches[f]; }
  for (auto& t : s->timers) {
    float x = 0.f;
    if (hipEventElapsedTime(&x, t.a, t.b) == hipSuccess) ms[t.fam] += x;
  }
  *n_families = KF_COUNT;
  return EE_OK;
}
