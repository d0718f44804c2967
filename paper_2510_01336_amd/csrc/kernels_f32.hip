// Dtype-independent helper kernels and the plain fp32 path used by EE_F32 models.
// The fp32 kernels favour clarity over speed: EE_F32 exists for the small reference-precision
// configuration; the bandwidth-critical work is in kernels_bf16.hip.
#include "kernels.h"
#include <hip/hip_ext.h>
#include <algorithm>
#include <cmath>

// ---------------------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------------------
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

__global__ void embed_kernel(const void* emb, int bf16, const int* tok, float* X, int M, int d) {
  int r = blockIdx.x;
  size_t base = (size_t)tok[r] * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x)
    X[(size_t)r * d + c] = bf16 ? bf16_to_f32(((const bf16_t*)emb)[base + c]) : ((const float*)emb)[base + c];
}
void k_embed(hipStream_t st, bool bf16, const void* emb, const int* tok, float* X, int M, int d) {
  hipLaunchKernelGGL(embed_kernel, dim3(M), dim3(256), 0, st, emb, (int)bf16, tok, X, M, d);
}

__global__ void copy_rows_kernel(float* dst, const int* dst_idx, int dst_add, const float* src, const int* src_idx, int d) {
  int r = blockIdx.x;
  size_t so = (size_t)(src_idx ? src_idx[r] : r) * d, dof = (size_t)((dst_idx ? dst_idx[r] : r) + dst_add) * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) dst[dof + c] = src[so + c];
}
void k_copy_rows(hipStream_t st, float* dst, const int* dst_idx, int dst_add, const float* src, const int* src_idx, int M, int d) {
  hipLaunchKernelGGL(copy_rows_kernel, dim3(M), dim3(256), 0, st, dst, dst_idx, dst_add, src, src_idx, d);
}

// LeadingSubstringVerify (last function of Algorithms 1/2) given the verifier's arg-max tokens:
// one wavefront per sequence, ballot over mismatches, count of leading matches.
__global__ void accept_kernel(const int* v, const int* seq_row0, const int* seq_m, const int* cand, const int* n_cand,
                              int cand_stride, int* n_accept, int* next_tok) {
  int b = blockIdx.x, lane = threadIdx.x;
  int m = seq_m[b];
  if (m == 0) { if (lane == 0) { n_accept[b] = -1; next_tok[b] = -1; } return; }
  int nc = n_cand[b], row0 = seq_row0[b];
  int a = nc;
  for (int j0 = 0; j0 < nc; j0 += 64) {
    int j = j0 + lane;
    bool mism = j < nc && cand[b * cand_stride + j] != v[row0 + j];
    unsigned long long mask = __ballot(mism);
    if (mask) { a = j0 + __ffsll((long long)mask) - 1; break; }
  }
  if (lane == 0) {
    n_accept[b] = a;
    next_tok[b] = a < m ? v[row0 + a] : -1;
  }
}
void k_accept(hipStream_t st, const int* v, const CallMeta& meta, int cand_stride, int B, int* n_accept, int* next_tok) {
  hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, st, v, meta.seq_row0, meta.seq_m, meta.cand, meta.n_cand,
                     cand_stride, n_accept, next_tok);
}

__global__ void take_token_kernel(const int* v, const int* row_seq, int M, int* tok_next, int* draft_out, int stride, int j) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= M) return;
  tok_next[r] = v[r];
  draft_out[row_seq[r] * stride + j] = v[r];
}
void k_take_token(hipStream_t st, const int* v, const int* row_seq, int M, int* tok_next, int* draft_out, int stride, int j) {
  hipLaunchKernelGGL(take_token_kernel, dim3(ceil_div(M, 64)), dim3(64), 0, st, v, row_seq, M, tok_next, draft_out, stride, j);
}

// Rotary angles are formed in double: at position 32768 an fp32 product pos*freq is off by ~2e-3 rad.
// The thread of a row's first pair also resolves the row's lookups once for all layers of the call -- first q-tile of
// its sequence, row index inside the sequence, KV page and slot of its position -- so that the QKV epilogue of every
// layer finds them with one row-indexed load instead of a chain of dependent ones.
__global__ void rope_table_kernel(const int* row_pos, int pos_add, const double* inv_freq, float2* cs, int M, int half,
                                  const int* row_seq, const int* seq_row0, const int* seq_qt0, const int* block_table, int pps,
                                  int4* rowinfo) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M * half) return;
  int r = i / half, f = i % half;
  const int pos = row_pos[r] + pos_add;
  double ang = (double)pos * inv_freq[f];
  double s, c;
  sincos(ang, &s, &c);
  cs[i] = make_float2((float)c, (float)s);
  if (f == 0 && rowinfo) {
    const int sq = row_seq[r];
    rowinfo[r] = make_int4(seq_qt0[sq], r - seq_row0[sq], block_table[sq * pps + pos / EE_PAGE], pos % EE_PAGE);
  }
}
void k_rope_table(hipStream_t st, const CallMeta& mt, int pos_add, const double* inv_freq, float2* cs, int M, int half, int pps,
                  int4* rowinfo) {
  hipLaunchKernelGGL(rope_table_kernel, dim3(ceil_div(M * half, 256)), dim3(256), 0, st, mt.row_pos, pos_add, inv_freq, cs, M, half,
                     mt.row_seq, mt.seq_row0, mt.seq_qt0, mt.block_table, pps, rowinfo);
}

__global__ void fill_nan_dead_kv_kernel(void* kv, int bf16, const int* pages, int n_owned, int len, int layer0, int layer1,
                                        int n_pages, int n_kv, int D) {
  size_t per_layer = (size_t)n_owned * n_kv * EE_PAGE * D;
  size_t total = per_layer * (layer1 - layer0);
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    int d = i % D; size_t t = i / D;
    int pp = t % EE_PAGE; t /= EE_PAGE;
    int kvh = t % n_kv; t /= n_kv;
    int pi = t % n_owned; int layer = layer0 + (int)(t / n_owned);
    if (pi * EE_PAGE + pp < len) continue;
    size_t slab = kv_slab(layer, pages[pi], kvh, n_pages, n_kv, D);
    size_t ko = slab + k_page_off(pp, d, D), vo = slab + EE_PAGE * D + v_page_off(pp, d, D);
    if (bf16) { ((bf16_t*)kv)[ko] = 0x7fc0; ((bf16_t*)kv)[vo] = 0x7fc0; }
    else { ((float*)kv)[ko] = __builtin_nanf(""); ((float*)kv)[vo] = __builtin_nanf(""); }
  }
}
void k_fill_nan_dead_kv(hipStream_t st, bool bf16, void* kv, const int* pages, int n_owned_pages, int len,
                        int layer0, int layer1, int n_pages, int n_kv, int D) {
  if (n_owned_pages <= 0 || layer1 <= layer0) return;
  hipLaunchKernelGGL(fill_nan_dead_kv_kernel, dim3(1024), dim3(256), 0, st, kv, (int)bf16, pages, n_owned_pages, len,
                     layer0, layer1, n_pages, n_kv, D);
}

__global__ void read_kv_kernel(const void* kv, int bf16, const int* pages, int layer, int pos0, int n, int n_pages, int n_kv,
                               int D, float* k_out, float* v_out) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n * n_kv * D) return;
  int d = i % D, kvh = (i / D) % n_kv, p = pos0 + i / (D * n_kv);
  size_t slab = kv_slab(layer, pages[p / EE_PAGE], kvh, n_pages, n_kv, D);
  size_t ko = slab + k_page_off(p % EE_PAGE, d, D), vo = slab + EE_PAGE * D + v_page_off(p % EE_PAGE, d, D);
  k_out[i] = bf16 ? bf16_to_f32(((const bf16_t*)kv)[ko]) : ((const float*)kv)[ko];
  v_out[i] = bf16 ? bf16_to_f32(((const bf16_t*)kv)[vo]) : ((const float*)kv)[vo];
}
void k_read_kv(hipStream_t st, bool bf16, const void* kv, const int* pages, int layer, int pos0, int n,
               int n_pages, int n_kv, int D, float* k_out, float* v_out) {
  if (n <= 0) return;
  hipLaunchKernelGGL(read_kv_kernel, dim3(ceil_div(n * n_kv * D, 256)), dim3(256), 0, st, kv, (int)bf16, pages, layer, pos0, n,
                     n_pages, n_kv, D, k_out, v_out);
}

__global__ void write_kv_kernel(void* kv, int bf16, const int* pages, int layer, int pos0, int n, int n_pages, int n_kv, int D,
                                const float* k_in, const float* v_in) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n * n_kv * D) return;
  int d = i % D, kvh = (i / D) % n_kv, p = pos0 + i / (D * n_kv);
  size_t slab = kv_slab(layer, pages[p / EE_PAGE], kvh, n_pages, n_kv, D);
  size_t ko = slab + k_page_off(p % EE_PAGE, d, D), vo = slab + EE_PAGE * D + v_page_off(p % EE_PAGE, d, D);
  if (bf16) { ((bf16_t*)kv)[ko] = f32_to_bf16(k_in[i]); ((bf16_t*)kv)[vo] = f32_to_bf16(v_in[i]); }
  else { ((float*)kv)[ko] = k_in[i]; ((float*)kv)[vo] = v_in[i]; }
}
void k_write_kv(hipStream_t st, bool bf16, void* kv, const int* pages, int layer, int pos0, int n, int n_pages, int n_kv, int D,
                const float* k_in, const float* v_in) {
  if (n <= 0) return;
  hipLaunchKernelGGL(write_kv_kernel, dim3(ceil_div(n * n_kv * D, 256)), dim3(256), 0, st, kv, (int)bf16, pages, layer, pos0, n,
                     n_pages, n_kv, D, k_in, v_in);
}

// Plain streaming copy (16 bytes per lane, grid-stride): the known-size kernel against which hardware
// byte counters are calibrated when HBM traffic of the other kernels is measured.
__global__ __launch_bounds__(256) void stream_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
extern "C" int ee_debug_stream_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (!dst_dev || !src_dev || (bytes & 15) || ((uintptr_t)dst_dev & 15) || ((uintptr_t)src_dev & 15)) {
    ee_set_error("stream copy needs non-null 16-byte aligned pointers and a size that is a multiple of 16");
    return EE_ERR_ARG;
  }
  if (!bytes) return EE_OK;
  const size_t n16 = bytes / 16;
  const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst_dev, (const uint4*)src_dev, n16);
  HIP_TRY(hipGetLastError());
  return EE_OK;
}

// Plain streaming read (16 bytes per lane, four requests in flight per lane, streaming hint, grid-stride): what the
// chip delivers to a kernel that does nothing but fetch `bytes` once, launched after another kernel on the same
// stream.  The floor against which the weight-streaming projections are read: a dependent launch of a few tens of MB
// never reaches the peak rate, whatever its arithmetic.
__device__ unsigned g_read_sink;
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src0, size_t n16) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4* src = (const u32x4*)src0;
  const size_t stride = (size_t)gridDim.x * 1024;
  unsigned acc = 0;
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  for (; i + 768 < n16; i += stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + 256);
    const u32x4 c = __builtin_nontemporal_load(src + i + 512), d = __builtin_nontemporal_load(src + i + 768);
    acc ^= a.x ^ b.y ^ c.z ^ d.w;
  }
  for (; i < n16; i += 256) acc ^= __builtin_nontemporal_load(src + i).x;
  if (acc == 0x9e3779b9u) g_read_sink = acc;       // (keeps the loads alive; practically never taken)
}
extern "C" int ee_debug_read_floor(const void* buf_dev, const size_t* sizes, int n, int reps, float* us_out, void* stream) {
  if (!buf_dev || !sizes || !us_out || n < 1 || n > 16 || reps < 1 || ((uintptr_t)buf_dev & 15)) {
    ee_set_error("read floor needs a 16-byte aligned buffer, 1..16 sizes and at least one repetition");
    return EE_ERR_ARG;
  }
  for (int i = 0; i < n; ++i)
    if (!sizes[i] || (sizes[i] & 15)) { ee_set_error("read floor: every size must be a positive multiple of 16"); return EE_ERR_ARG; }
  hipStream_t st = (hipStream_t)stream;
  std::vector<hipEvent_t> ev(2 * n, nullptr);
  int rc = EE_OK;
  for (auto& e : ev)
    if (rc == EE_OK && hipEventCreate(&e) != hipSuccess) { ee_set_error("read floor: no event"); rc = EE_ERR_HIP; }
  std::vector<double> sum(n, 0.0);
  auto launch = [&](const char* p, size_t bytes, hipEvent_t a, hipEvent_t b) {
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 1023) / 1024, 2048);
    if (a) hipExtLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, st, a, b, 0, (const uint4*)p, n16);
    else hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, st, (const uint4*)p, n16);
  };
  // one round = the n reads back to back on the stream, behind an untimed one, as the projections of a layer follow
  // each other; the events are attached to the dispatches and hold each kernel's own start and end
  for (int r = 0; r < reps + 2 && rc == EE_OK; ++r) {           // (two untimed rounds first)
    const char* p = (const char*)buf_dev;
    launch(p, sizes[0], nullptr, nullptr);
    for (int i = 0; i < n; ++i) {
      launch(p, sizes[i], ev[2 * i], ev[2 * i + 1]);
      p += sizes[i];
    }
    if (hipStreamSynchronize(st) != hipSuccess) { ee_set_error("read floor: a launch failed"); rc = EE_ERR_HIP; break; }
    for (int i = 0; i < n && r >= 2; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess) { ee_set_error("read floor: timing a launch failed"); rc = EE_ERR_HIP; break; }
      sum[i] += 1e3 * ms;
    }
  }
  for (auto e : ev)
    if (e) (void)hipEventDestroy(e);
  if (rc != EE_OK) return rc;
  for (int i = 0; i < n; ++i) us_out[i] = (float)(sum[i] / reps);
  return EE_OK;
}

// ---------------------------------------------------------------------------------------------
// fp32 path
// ---------------------------------------------------------------------------------------------
__global__ void f32_rmsnorm_kernel(const float* X, const float* g, float eps, float* out, int d) {
  __shared__ float part[4];
  int r = blockIdx.x;
  const float* x = X + (size_t)r * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) ss += x[c] * x[c];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = part[0] + part[1] + part[2] + part[3];
  float inv = 1.0f / sqrtf(tot / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += blockDim.x) out[(size_t)r * d + c] = x[c] * inv * g[c];
}
void f32_rmsnorm(hipStream_t st, const float* X, const float* g, float eps, float* out, int M, int d) {
  hipLaunchKernelGGL(f32_rmsnorm_kernel, dim3(M), dim3(256), 0, st, X, g, eps, out, d);
}

// one wavefront per output element
__global__ void f32_gemm_kernel(const float* A, int lda, const float* W, float* Y, int ldy, int M, int N, int K, int add) {
  int lane = threadIdx.x & 63;
  long o = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (o >= (long)M * N) return;
  int m = (int)(o / N), n = (int)(o % N);
  const float* a = A + (size_t)m * lda;
  const float* w = W + (size_t)n * K;
  float acc = 0.f;
  for (int k = lane; k < K; k += 64) acc += a[k] * w[k];
  acc = wave_sum(acc);
  if (lane == 0) {
    size_t i = (size_t)m * ldy + n;
    Y[i] = add ? Y[i] + acc : acc;
  }
}
void f32_gemm(hipStream_t st, const float* A, int lda, const float* W, float* Y, int ldy, int M, int N, int K, bool add) {
  long outs = (long)M * N;
  hipLaunchKernelGGL(f32_gemm_kernel, dim3((unsigned)((outs + 3) / 4)), dim3(256), 0, st, A, lda, W, Y, ldy, M, N, K, (int)add);
}

__global__ void f32_rope_append_kernel(const float* QKV, int ldq, const float2* cs, const int* row_seq, const int* row_pos,
                                       const int* block_table, int pos_add, int M, int Hq, int Hkv, int D, int layer,
                                       int n_pages, int pps, float* Q, float* kv) {
  int half = D >> 1, heads = Hq + 2 * Hkv;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M * heads * half) return;
  int f = i % half, h = (i / half) % heads, r = i / (half * heads);
  const float* src = QKV + (size_t)r * ldq + (size_t)h * D;
  float a = src[f], b = src[f + half];
  float2 c = cs[r * half + f];
  if (h < Hq) {
    Q[(size_t)r * Hq * D + h * D + f] = a * c.x - b * c.y;
    Q[(size_t)r * Hq * D + h * D + f + half] = b * c.x + a * c.y;
    return;
  }
  int pos = row_pos[r] + pos_add;
  int page = block_table[row_seq[r] * pps + pos / EE_PAGE], pp = pos % EE_PAGE;
  if (h < Hq + Hkv) {
    size_t slab = kv_slab(layer, page, h - Hq, n_pages, Hkv, D);
    kv[slab + k_page_off(pp, f, D)] = a * c.x - b * c.y;
    kv[slab + k_page_off(pp, f + half, D)] = b * c.x + a * c.y;
  } else {
    size_t slab = kv_slab(layer, page, h - Hq - Hkv, n_pages, Hkv, D) + EE_PAGE * D;
    kv[slab + v_page_off(pp, f, D)] = a;
    kv[slab + v_page_off(pp, f + half, D)] = b;
  }
}
void f32_rope_append(hipStream_t st, const float* QKV, int ldq, const float2* cs, const CallMeta& meta, int pos_add, int M,
                     int Hq, int Hkv, int D, int layer, int n_pages, int pages_per_seq, float* Q, float* kv) {
  int total = M * (Hq + 2 * Hkv) * (D / 2);
  hipLaunchKernelGGL(f32_rope_append_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, QKV, ldq, cs, meta.row_seq,
                     meta.row_pos, meta.block_table, pos_add, M, Hq, Hkv, D, layer, n_pages, pages_per_seq, Q, kv);
}

// one workgroup per (row, query head): scores over positions 0..pos in LDS, two-pass softmax
__global__ void f32_attention_kernel(const float* Q, const float* kv, const int* row_seq, const int* row_pos,
                                     const int* block_table, int pos_add, int Hq, int Hkv, int D, int layer, int n_pages,
                                     int pps, float* out) {
  extern __shared__ float sm[];
  float* q = sm;            // [D]
  float* red = sm + D;      // [8]
  float* sc = sm + D + 8;   // [n]
  int r = blockIdx.x, h = blockIdx.y, kvh = h / (Hq / Hkv);
  int n = row_pos[r] + pos_add + 1;
  const int* bt = block_table + row_seq[r] * pps;
  for (int d = threadIdx.x; d < D; d += blockDim.x) q[d] = Q[(size_t)r * Hq * D + h * D + d];
  __syncthreads();
  float scale = 1.0f / sqrtf((float)D);
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < n; j += blockDim.x) {
    size_t slab = kv_slab(layer, bt[j / EE_PAGE], kvh, n_pages, Hkv, D);
    float s = 0.f;
    for (int d = 0; d < D; ++d) s += q[d] * kv[slab + k_page_off(j % EE_PAGE, d, D)];
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = threadIdx.x; j < n; j += blockDim.x) { float p = expf(sc[j] - mx); sc[j] = p; sum += p; }
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) red[4 + (threadIdx.x >> 6)] = sum;
  __syncthreads();
  sum = red[4] + red[5] + red[6] + red[7];
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) {
      size_t slab = kv_slab(layer, bt[j / EE_PAGE], kvh, n_pages, Hkv, D) + EE_PAGE * D;
      acc += sc[j] * kv[slab + v_page_off(j % EE_PAGE, d, D)];
    }
    out[(size_t)r * Hq * D + h * D + d] = acc / sum;
  }
}
void f32_attention(hipStream_t st, const float* Q, const float* kv, const CallMeta& meta, int pos_add, int M, int Hq, int Hkv,
                   int D, int layer, int n_pages, int pages_per_seq, int max_ctx, float* out) {
  size_t smem = (size_t)(D + 8 + max_ctx) * sizeof(float);
  hipLaunchKernelGGL(f32_attention_kernel, dim3(M, Hq), dim3(256), smem, st, Q, kv, meta.row_seq, meta.row_pos,
                     meta.block_table, pos_add, Hq, Hkv, D, layer, n_pages, pages_per_seq, out);
}

// GU columns follow the physical row order of the interleaved gate/up matrix
__global__ void f32_silu_mul_kernel(const float* GU, int ldg, float* H, int M, int F) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M * F) return;
  int m = i / F, f = i % F;
  int gc = ((f >> 4) * 2) * 16 + (f & 15);
  float g = GU[(size_t)m * ldg + gc], u = GU[(size_t)m * ldg + gc + 16];
  H[(size_t)m * F + f] = g / (1.0f + expf(-g)) * u;
}
void f32_silu_mul(hipStream_t st, const float* GU, int ldg, float* H, int M, int F) {
  hipLaunchKernelGGL(f32_silu_mul_kernel, dim3(ceil_div(M * F, 256)), dim3(256), 0, st, GU, ldg, H, M, F);
}

// arg max of each row; the lowest index wins ties
__global__ void f32_argmax_kernel(const float* logits, int V, int* v) {
  __shared__ float bv[256];
  __shared__ int bi[256];
  int r = blockIdx.x;
  const float* x = logits + (size_t)r * V;
  float best = -INFINITY; int idx = 0x7fffffff;
  for (int c = threadIdx.x; c < V; c += blockDim.x) {
    float t = x[c];
    if (t > best) { best = t; idx = c; }
  }
  bv[threadIdx.x] = best; bi[threadIdx.x] = idx;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) {
      float o = bv[threadIdx.x + s]; int oi = bi[threadIdx.x + s];
      if (o > bv[threadIdx.x] || (o == bv[threadIdx.x] && oi < bi[threadIdx.x])) { bv[threadIdx.x] = o; bi[threadIdx.x] = oi; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) v[r] = bi[0];
}
void f32_argmax(hipStream_t st, const float* logits, int M, int V, int* v) {
  hipLaunchKernelGGL(f32_argmax_kernel, dim3(M), dim3(256), 0, st, logits, V, v);
}
