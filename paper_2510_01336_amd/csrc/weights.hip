// Model arena layout, on-device synthetic weight generator, tensor import / export.
#include "common.h"
#include <cmath>
#include <cstdarg>
#include <cstdio>

// ---------------------------------------------------------------------------------------------
// error string (thread local)
// ---------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";
void ee_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
extern "C" const char* ee_last_error(void) { return g_err; }

// ---------------------------------------------------------------------------------------------
// layout
// ---------------------------------------------------------------------------------------------
static int check_config(const ee_config* c) {
  if (!c) { ee_set_error("null config"); return EE_ERR_ARG; }
  if (c->n_layers < 3 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 || c->vocab < 2) {
    ee_set_error("bad model shape"); return EE_ERR_ARG;
  }
  if (!(0 < c->exit_draft && c->exit_draft < c->exit_inter && c->exit_inter < c->n_layers)) {
    ee_set_error("exits must satisfy 0 < L_d < L_i < L_f"); return EE_ERR_ARG;
  }
  if (c->n_q_heads % c->n_kv_heads) { ee_set_error("n_q_heads must be a multiple of n_kv_heads"); return EE_ERR_ARG; }
  if (c->dtype != EE_F32 && c->dtype != EE_BF16) { ee_set_error("dtype must be EE_F32 or EE_BF16"); return EE_ERR_ARG; }
  if (c->dtype == EE_BF16 && c->head_dim != 64 && c->head_dim != 128) {
    ee_set_error("EE_BF16 models need head_dim 64 or 128"); return EE_ERR_ARG;
  }
  if (c->dtype == EE_BF16 && (c->d_model % 16 || c->d_model > 16384)) {
    ee_set_error("EE_BF16 models need d_model to be a multiple of 16, at most 16384"); return EE_ERR_ARG;
  }
  if (c->head_dim % 2 || c->head_dim > 256) { ee_set_error("head_dim must be even and <= 256"); return EE_ERR_ARG; }
  if (c->n_q_heads / c->n_kv_heads > 16) { ee_set_error("at most 16 query heads per KV head"); return EE_ERR_ARG; }
  if (!(c->rope_theta > 1.f) || !(c->rms_eps > 0.f)) { ee_set_error("bad rope_theta / rms_eps"); return EE_ERR_ARG; }
  if (c->n_extra_exits < 0 || c->n_extra_exits > 4) { ee_set_error("0..4 extra verifier exits"); return EE_ERR_ARG; }
  for (int i = 0, prev = c->exit_inter; i < c->n_extra_exits; prev = c->extra_exits[i++])
    if (!(prev < c->extra_exits[i] && c->extra_exits[i] < c->n_layers)) {
      ee_set_error("extra verifier exits must increase strictly between L_i and L_f"); return EE_ERR_ARG;
    }
  if (c->head_rank < 0 || c->head_rank > 16384 || (c->dtype == EE_BF16 && c->head_rank % 32)) {
    ee_set_error("head_rank must be 0 or a rank up to 16384 (a multiple of 32 for EE_BF16 models)"); return EE_ERR_ARG;
  }
  return EE_OK;
}

static MatLoc place(size_t& cur, int N, int K, bool bf16) {
  MatLoc m;
  m.N = N; m.K = K;
  if (bf16) { m.Np = ceil_div(N, 16) * 16; m.Kp = ceil_div(K, 32) * 32; }
  else      { m.Np = N; m.Kp = K; }
  cur = align_up(cur, 256);
  m.off = cur;
  cur += (size_t)m.Np * m.Kp * (bf16 ? 2 : 4);
  return m;
}

int ee_layout_model(ee_model* m) {
  const ee_config& c = m->cfg;
  m->bf16 = c.dtype == EE_BF16;
  m->exits = {c.exit_draft, c.exit_inter};
  for (int i = 0; i < c.n_extra_exits; ++i) m->exits.push_back(c.extra_exits[i]);
  m->exits.push_back(c.n_layers);
  const size_t es = m->bf16 ? 2 : 4;
  const int d = c.d_model, D = c.head_dim;
  m->Fp = ceil_div(c.d_ffn, 16) * 16;
  size_t cur = 0;
  m->emb = cur; cur += (size_t)c.vocab * d * es;
  cur = align_up(cur, 256); m->gfinal = cur; cur += (size_t)d * 4;
  m->head = place(cur, c.vocab, d, m->bf16);
  for (int e = 0; e + 1 < (int)m->exits.size() && c.head_rank > 0; ++e) {      // every exit but the last
    cur = align_up(cur, 256); m->auxg[e] = cur; cur += (size_t)d * 4;
    m->auxA[e] = place(cur, c.head_rank, d, m->bf16);
    m->auxB[e] = place(cur, d, c.head_rank, m->bf16);
  }
  m->L.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    LayerLoc& L = m->L[l];
    cur = align_up(cur, 256); L.g1 = cur; cur += (size_t)d * 4;
    cur = align_up(cur, 256); L.g2 = cur; cur += (size_t)d * 4;
    L.qkv = place(cur, (c.n_q_heads + 2 * c.n_kv_heads) * D, d, m->bf16);
    L.o = place(cur, d, c.n_q_heads * D, m->bf16);
    L.gu = place(cur, 2 * m->Fp, d, m->bf16);
    L.down = place(cur, d, c.d_ffn, m->bf16);
  }
  cur = align_up(cur, 256);
  size_t inv_off = cur; cur += (size_t)(D / 2) * 8;
  m->bytes = align_up(cur, 256);
  if (m->base) m->inv_freq = (double*)(m->base + inv_off);
  return EE_OK;
}

int ee_tensor_map(const ee_model* m, int tid, int layer, TensorMap* t) {
  const ee_config& c = m->cfg;
  const int d = c.d_model, D = c.head_dim;
  if (tid >= EE_T_AUX_G && tid <= EE_T_AUX_B) {
    if (c.head_rank <= 0) { ee_set_error("the model has no auxiliary exit heads"); return EE_ERR_ARG; }
    if (layer < 0 || layer + 1 >= (int)m->exits.size()) { ee_set_error("exit index must name an early exit (0 = L_d, 1 = L_i, ...)"); return EE_ERR_ARG; }
    if (tid == EE_T_AUX_G) *t = {1, d, 1, m->auxg[layer], 0, 0, 0, D};
    else if (tid == EE_T_AUX_A) *t = {0, c.head_rank, d, m->auxA[layer].off, 0, 0, m->auxA[layer].Kp, D};
    else *t = {0, d, c.head_rank, m->auxB[layer].off, 0, 0, m->auxB[layer].Kp, D};
    return EE_OK;
  }
  if (tid >= EE_T_G1 && (layer < 0 || layer >= c.n_layers)) { ee_set_error("layer out of range"); return EE_ERR_ARG; }
  t->row_off = 0; t->interleave = 0; t->Kp = 0; t->hd = D;
  switch (tid) {
    case EE_T_EMB: *t = {2, c.vocab, d, m->emb, 0, 0, d, D}; return EE_OK;
    case EE_T_GFINAL: *t = {1, d, 1, m->gfinal, 0, 0, 0, D}; return EE_OK;
    case EE_T_HEAD: *t = {0, c.vocab, d, m->head.off, 0, 0, m->head.Kp, D}; return EE_OK;
    default: break;
  }
  const LayerLoc& L = m->L[layer];
  const int qi = m->bf16 ? 3 : 0;   // bf16 models keep the rotary halves of every head in adjacent tiles
  switch (tid) {
    case EE_T_G1: *t = {1, d, 1, L.g1, 0, 0, 0, D}; break;
    case EE_T_G2: *t = {1, d, 1, L.g2, 0, 0, 0, D}; break;
    case EE_T_WQ: *t = {0, c.n_q_heads * D, d, L.qkv.off, 0, qi, L.qkv.Kp, D}; break;
    case EE_T_WK: *t = {0, c.n_kv_heads * D, d, L.qkv.off, c.n_q_heads * D, qi, L.qkv.Kp, D}; break;
    case EE_T_WV: *t = {0, c.n_kv_heads * D, d, L.qkv.off, (c.n_q_heads + c.n_kv_heads) * D, qi, L.qkv.Kp, D}; break;
    case EE_T_WO: *t = {0, d, c.n_q_heads * D, L.o.off, 0, 0, L.o.Kp, D}; break;
    case EE_T_WGATE: *t = {0, c.d_ffn, d, L.gu.off, 0, 1, L.gu.Kp, D}; break;
    case EE_T_WUP: *t = {0, c.d_ffn, d, L.gu.off, 0, 2, L.gu.Kp, D}; break;
    case EE_T_WDOWN: *t = {0, d, c.d_ffn, L.down.off, 0, 0, L.down.Kp, D}; break;
    default: ee_set_error("unknown tensor id %d", tid); return EE_ERR_ARG;
  }
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// element access by logical index
// ---------------------------------------------------------------------------------------------
__device__ inline void store_elem(char* base, const TensorMap& t, int bf16, int r, int c, float v) {
  if (t.kind == 1) { ((float*)(base + t.off))[r] = bf16 ? bf16_to_f32(f32_to_bf16(v)) : v; return; }   // gains stay fp32 words
  if (t.kind == 2) {
    size_t i = (size_t)r * t.cols + c;
    if (bf16) ((bf16_t*)(base + t.off))[i] = f32_to_bf16(v); else ((float*)(base + t.off))[i] = v;
    return;
  }
  int pr = phys_row(r, t.row_off, t.interleave, t.hd);
  if (bf16) ((bf16_t*)(base + t.off))[frag_offset(pr, c, t.Kp >> 5)] = f32_to_bf16(v);
  else ((float*)(base + t.off))[(size_t)pr * t.Kp + c] = v;
}
__device__ inline float load_elem(const char* base, const TensorMap& t, int bf16, int r, int c) {
  if (t.kind == 1) return ((const float*)(base + t.off))[r];
  if (t.kind == 2) {
    size_t i = (size_t)r * t.cols + c;
    return bf16 ? bf16_to_f32(((const bf16_t*)(base + t.off))[i]) : ((const float*)(base + t.off))[i];
  }
  int pr = phys_row(r, t.row_off, t.interleave, t.hd);
  if (bf16) return bf16_to_f32(((const bf16_t*)(base + t.off))[frag_offset(pr, c, t.Kp >> 5)]);
  return ((const float*)(base + t.off))[(size_t)pr * t.Kp + c];
}

// ---------------------------------------------------------------------------------------------
// Counter-based synthetic weights (random-init stand-in for a trained EE checkpoint):
//   key   = mix64(mix64(seed) ^ ((tensor_id << 32) | layer))
//   w_j   = mix64(key + (3 e + j + 1) * GOLD), j = 0..2, e = row-major logical element index
//   value = float(sum of the twelve 16-bit lanes - 393210) * scale   (+ 1 for norm gains)
// Integer-exact up to one fp32 multiply (and one add), so host code can reproduce every bit.
// ---------------------------------------------------------------------------------------------
#define EE_GOLD 0x9E3779B97F4A7C15ull
__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__device__ inline int lanes16(uint64_t w) {
  return (int)(w & 0xFFFF) + (int)((w >> 16) & 0xFFFF) + (int)((w >> 32) & 0xFFFF) + (int)(w >> 48);
}

__global__ void gen_tensor_kernel(char* base, TensorMap t, int bf16, uint64_t key, float scale, int gain, size_t count) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
    uint64_t b = key + (3ull * e + 1ull) * EE_GOLD;
    int s = lanes16(mix64(b)) + lanes16(mix64(b + EE_GOLD)) + lanes16(mix64(b + 2ull * EE_GOLD));
    float v = (float)(s - 393210) * scale;
    // the product must be rounded on its own before the gain's +1: an empty asm keeps the
    // compiler from contracting the two into one fused multiply-add
    asm volatile("" : "+v"(v));
    if (gain) v = 1.0f + v;
    int r = (int)(e / (size_t)t.cols), c = (int)(e % (size_t)t.cols);
    store_elem(base, t, bf16, r, c, v);
  }
}

__global__ void import_tensor_kernel(char* base, TensorMap t, int bf16, const float* src, size_t count) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride)
    store_elem(base, t, bf16, (int)(e / (size_t)t.cols), (int)(e % (size_t)t.cols), src[e]);
}

__global__ void export_tensor_kernel(const char* base, TensorMap t, int bf16, int row0, float* dst, size_t count) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride)
    dst[e] = load_elem(base, t, bf16, row0 + (int)(e / (size_t)t.cols), (int)(e % (size_t)t.cols));
}

static int group_of_layer(const ee_config& c, int l) { return l < c.exit_draft ? 0 : (l < c.exit_inter ? 1 : 2); }

static int gen_one(ee_model* m, int tid, int layer) {
  TensorMap t;
  EE_TRY(ee_tensor_map(m, tid, layer, &t));
  const bool per_layer = tid >= EE_T_G1;
  uint64_t key = mix64(mix64(m->seed) ^ (((uint64_t)tid << 32) | (uint64_t)(per_layer ? layer : 0)));
  float gamma = (tid == EE_T_WO || tid == EE_T_WDOWN) ? m->cfg.gamma[group_of_layer(m->cfg, layer)] : 1.0f;
  if (tid == EE_T_AUX_B) gamma = m->cfg.gamma[layer < 2 ? layer : 2];     // `layer` is the exit index here
  volatile float s1 = m->cfg.sigma * gamma;        // one fp32 product, then an exact power-of-two scale
  float scale = s1 * 1.52587890625e-05f;           // 2^-16
  int gain = (tid == EE_T_GFINAL || tid == EE_T_G1 || tid == EE_T_G2 || tid == EE_T_AUX_G);
  size_t count = (size_t)t.rows * t.cols;
  int blocks = (int)((count + 255) / 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(gen_tensor_kernel, dim3(blocks), dim3(256), 0, m->stream, m->base, t, (int)m->bf16, key, scale, gain, count);
  HIP_TRY(hipGetLastError());
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI: model
// ---------------------------------------------------------------------------------------------
extern "C" size_t ee_model_bytes(const ee_config* cfg) {
  if (check_config(cfg) != EE_OK) return 0;
  ee_model tmp;
  tmp.cfg = *cfg;
  ee_layout_model(&tmp);
  return tmp.bytes;
}

extern "C" int ee_model_load(const ee_config* cfg, void* dev_arena, size_t arena_bytes, uint64_t seed,
                             void* stream, ee_model** out) {
  EE_TRY(check_config(cfg));
  if (!dev_arena || !out || ((uintptr_t)dev_arena & 255)) { ee_set_error("arena must be non-null and 256-byte aligned"); return EE_ERR_ARG; }
  ee_model* m = new ee_model();
  m->cfg = *cfg;
  m->base = (char*)dev_arena;
  m->stream = (hipStream_t)stream;
  m->seed = seed;
  ee_layout_model(m);
  if (arena_bytes < m->bytes) {
    ee_set_error("model arena too small: %zu < %zu", arena_bytes, m->bytes);
    delete m; return EE_ERR_CAPACITY;
  }
  hipError_t e = hipMemsetAsync(m->base, 0, m->bytes, m->stream);   // padding rows / columns must be zero
  if (e != hipSuccess) { ee_set_error("memset: %s", hipGetErrorString(e)); delete m; return EE_ERR_HIP; }
  int rc = EE_OK;
  for (int tid = EE_T_EMB; tid <= EE_T_GFINAL && rc == EE_OK; ++tid) rc = gen_one(m, tid, 0);
  for (int e = 0; e + 1 < (int)m->exits.size() && cfg->head_rank > 0; ++e)
    for (int tid = EE_T_AUX_G; tid <= EE_T_AUX_B && rc == EE_OK; ++tid) rc = gen_one(m, tid, e);
  for (int l = 0; l < cfg->n_layers && rc == EE_OK; ++l)
    for (int tid = EE_T_G1; tid <= EE_T_WDOWN && rc == EE_OK; ++tid) rc = gen_one(m, tid, l);
  if (rc == EE_OK) {
    const int half = cfg->head_dim / 2;
    std::vector<double> inv(half);
    for (int i = 0; i < half; ++i) inv[i] = std::pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
    e = hipMemcpyAsync(m->inv_freq, inv.data(), half * sizeof(double), hipMemcpyHostToDevice, m->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess) { ee_set_error("model init: %s", hipGetErrorString(e)); rc = EE_ERR_HIP; }
  }
  if (rc != EE_OK) { delete m; return rc; }
  *out = m;
  return EE_OK;
}

extern "C" int ee_model_set_tensor(ee_model* m, int tid, int layer, const float* host_values) {
  if (!m || !host_values) { ee_set_error("null argument"); return EE_ERR_ARG; }
  TensorMap t;
  EE_TRY(ee_tensor_map(m, tid, layer, &t));
  size_t count = (size_t)t.rows * t.cols;
  float* stage = nullptr;
  HIP_TRY(hipMalloc(&stage, count * sizeof(float)));
  hipError_t e = hipMemcpyAsync(stage, host_values, count * sizeof(float), hipMemcpyHostToDevice, m->stream);
  if (e == hipSuccess) {
    int blocks = (int)((count + 255) / 256);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(import_tensor_kernel, dim3(blocks), dim3(256), 0, m->stream, m->base, t, (int)m->bf16, (const float*)stage, count);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
  (void)hipFree(stage);
  if (e != hipSuccess) { ee_set_error("set_tensor: %s", hipGetErrorString(e)); return EE_ERR_HIP; }
  return EE_OK;
}

extern "C" int ee_model_get_tensor_rows(ee_model* m, int tid, int layer, int row0, int nrows, float* host_out) {
  if (!m || !host_out) { ee_set_error("null argument"); return EE_ERR_ARG; }
  TensorMap t;
  EE_TRY(ee_tensor_map(m, tid, layer, &t));
  if (row0 < 0 || nrows < 0 || row0 + nrows > t.rows) { ee_set_error("row range outside tensor"); return EE_ERR_ARG; }
  size_t count = (size_t)nrows * t.cols;
  if (!count) return EE_OK;
  float* stage = nullptr;
  HIP_TRY(hipMalloc(&stage, count * sizeof(float)));
  int blocks = (int)((count + 255) / 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(export_tensor_kernel, dim3(blocks), dim3(256), 0, m->stream, (const char*)m->base, t, (int)m->bf16, row0, stage, count);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(host_out, stage, count * sizeof(float), hipMemcpyDeviceToHost, m->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
  (void)hipFree(stage);
  if (e != hipSuccess) { ee_set_error("get_tensor_rows: %s", hipGetErrorString(e)); return EE_ERR_HIP; }
  return EE_OK;
}

extern "C" void ee_model_free(ee_model* m) { delete m; }
