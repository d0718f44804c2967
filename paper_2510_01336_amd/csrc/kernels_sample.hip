// Rejection-sampling acceptance (App. G): exit distributions, the accept test and the draws.
// All random numbers are inputs (uniform in [0, 1)); nothing here generates any.
#include "kernels.h"

#define EE_SAMPLE_THREADS 1024

__device__ inline float block_reduce_max(float v, float* sh) {
  for (int s = 1; s < 64; s <<= 1) v = fmaxf(v, __shfl_xor(v, s, 64));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < EE_SAMPLE_THREADS / 64; ++w) r = fmaxf(r, sh[w]);
  __syncthreads();
  return r;
}
// sum in a fixed order (lanes by butterfly, then the sixteen wave sums one after the other)
__device__ inline float block_reduce_sum(float v, float* sh) {
  for (int s = 1; s < 64; s <<= 1) v += __shfl_xor(v, s, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = 0.f;
  for (int w = 0; w < EE_SAMPLE_THREADS / 64; ++w) r += sh[w];
  __syncthreads();
  return r;
}

// p = softmax(logits) per row; row r of `in` (stride in_stride floats) -> row out_idx[r] (or r) + out_add of `out`
// (rows of `vocab` floats).  In place when in == out with the same row mapping.
__global__ __launch_bounds__(EE_SAMPLE_THREADS) void softmax_rows_kernel(const float* in, size_t in_stride, float* out,
                                                                        const int* out_idx, int out_add, int vocab) {
  __shared__ float sh[EE_SAMPLE_THREADS / 64];
  const int r = blockIdx.x;
  const float* x = in + (size_t)r * in_stride;
  float* y = out + (size_t)((out_idx ? out_idx[r] : r) + out_add) * vocab;
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < vocab; i += EE_SAMPLE_THREADS) mx = fmaxf(mx, x[i]);
  mx = block_reduce_max(mx, sh);
  float sum = 0.f;
  for (int i = threadIdx.x; i < vocab; i += EE_SAMPLE_THREADS) sum += __expf(x[i] - mx);
  sum = block_reduce_sum(sum, sh);
  const float inv = 1.0f / sum;
  for (int i = threadIdx.x; i < vocab; i += EE_SAMPLE_THREADS) y[i] = __expf(x[i] - mx) * inv;
}
void k_softmax_rows(hipStream_t st, const float* in, size_t in_stride, float* out, const int* out_idx, int out_add, int M, int vocab) {
  if (M <= 0) return;
  hipLaunchKernelGGL(softmax_rows_kernel, dim3(M), dim3(EE_SAMPLE_THREADS), 0, st, in, in_stride, out, out_idx, out_add, vocab);
}

// The accept tests of one block per sequence (one wavefront each): candidate j, drawn from row
// draft_row0 + j of the draft distributions, is accepted when u < min(1, p_target / p_draft) at that token;
// n_accept = number of leading accepted candidates.
__global__ void rs_accept_kernel(const float* __restrict__ Pt, const float* __restrict__ Pd, int pd_rows_per_seq, int vocab,
                                 const int* seq_row0, const int* seq_m, const int* cand, const int* n_cand, int cand_stride,
                                 const float* __restrict__ u_acc, int u_stride, int* n_accept) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int m = seq_m[b];
  if (m == 0) { if (lane == 0) n_accept[b] = -1; return; }
  const int nc = n_cand[b], row0 = seq_row0[b];
  int a = nc;
  for (int j0 = 0; j0 < nc; j0 += 64) {
    const int j = j0 + lane;
    bool rej = false;
    if (j < nc) {
      const int tok = cand[b * cand_stride + j];
      const float pt = Pt[(size_t)(row0 + j) * vocab + tok], pd = Pd[((size_t)b * pd_rows_per_seq + j) * vocab + tok];
      rej = !(u_acc[(size_t)b * u_stride + j] < fminf(1.0f, pt / pd));
    }
    const unsigned long long mask = __ballot(rej);
    if (mask) { a = j0 + __ffsll((long long)mask) - 1; break; }
  }
  if (lane == 0) n_accept[b] = a;
}
void k_rs_accept(hipStream_t st, const float* Pt, const float* Pd, int pd_rows_per_seq, int vocab, const CallMeta& meta,
                 int cand_stride, int B, const float* u_acc, int u_stride, int* n_accept) {
  hipLaunchKernelGGL(rs_accept_kernel, dim3(B), dim3(64), 0, st, Pt, Pd, pd_rows_per_seq, vocab, meta.seq_row0, meta.seq_m,
                     meta.cand, meta.n_cand, cand_stride, u_acc, u_stride, n_accept);
}

// One draw per workgroup by inverse CDF: the first token whose cumulative weight exceeds u * (sum of weights).
// Thread t owns the contiguous tokens [t*C, (t+1)*C); chunk sums meet in LDS, one thread walks them and the
// owner of the hit chunk walks its tokens.  weight(i) = max(0, A[i] - B[i]) with B optional.
__device__ inline int draw_token(const float* __restrict__ A, const float* __restrict__ B, int vocab, float u, float* chunk, int* hit) {
  const int t = threadIdx.x, C = (vocab + EE_SAMPLE_THREADS - 1) / EE_SAMPLE_THREADS;
  const int i0 = t * C, i1 = min(vocab, i0 + C);
  float local = 0.f;
  int last_pos = -1;
  for (int i = i0; i < i1; ++i) {
    const float w = B ? fmaxf(0.f, A[i] - B[i]) : A[i];
    local += w;
    if (w > 0.f) last_pos = i;
  }
  chunk[t] = local;
  if (t == 0) { hit[0] = -1; hit[1] = -1; }
  __syncthreads();
  atomicMax(&hit[1], last_pos);                 // last token with weight (integer maximum: order-free)
  __shared__ float s_target, s_prefix;
  if (t == 0) {
    float total = 0.f;
    for (int c = 0; c < EE_SAMPLE_THREADS; ++c) total += chunk[c];
    const float target = u * total;
    float pre = 0.f;
    int h = -1;
    for (int c = 0; c < EE_SAMPLE_THREADS; ++c) {
      if (pre + chunk[c] > target) { h = c; break; }
      pre += chunk[c];
    }
    hit[0] = h; s_target = target; s_prefix = pre;
  }
  __syncthreads();
  __shared__ int s_tok;
  if (t == 0) s_tok = -1;
  __syncthreads();
  if (t == hit[0]) {
    float run = s_prefix;
    int tok = -1;
    for (int i = i0; i < i1; ++i) {
      run += B ? fmaxf(0.f, A[i] - B[i]) : A[i];
      if (run > s_target) { tok = i; break; }
    }
    s_tok = tok;
  }
  __syncthreads();
  const int tok = s_tok >= 0 ? s_tok : hit[1];  // rounding at the very end of the interval: the last token with weight
  __syncthreads();
  return tok;
}

// drafting: token of sequence b ~ row b*rows_per_seq + j of P (the distribution just stored there)
__global__ __launch_bounds__(EE_SAMPLE_THREADS) void draw_rows_kernel(const float* __restrict__ P, int rows_per_seq, int j, int vocab,
                                                                      const float* __restrict__ u, int u_stride,
                                                                      const int* __restrict__ row_seq, int* tok_next,
                                                                      int* draft_out, int stride) {
  __shared__ float chunk[EE_SAMPLE_THREADS];
  __shared__ int hit[2];
  const int r = blockIdx.x, b = row_seq[r];            // one row per drafting sequence
  const int tok = draw_token(P + ((size_t)b * rows_per_seq + j) * vocab, nullptr, vocab, u[(size_t)b * u_stride + j], chunk, hit);
  if (threadIdx.x == 0) { tok_next[r] = tok; draft_out[b * stride + j] = tok; }
}
void k_draw_rows(hipStream_t st, const float* P, int rows_per_seq, int j, int vocab, const float* u, int u_stride,
                 const int* row_seq, int M, int* tok_next, int* draft_out, int stride) {
  hipLaunchKernelGGL(draw_rows_kernel, dim3(M), dim3(EE_SAMPLE_THREADS), 0, st, P, rows_per_seq, j, vocab, u, u_stride, row_seq,
                     tok_next, draft_out, stride);
}

// after the accept tests: the replacement from the residual distribution at the first rejected position, or,
// when every candidate was accepted and the block has one more row, the target's own next token
__global__ __launch_bounds__(EE_SAMPLE_THREADS) void rs_draw_kernel(const float* __restrict__ Pt, const float* __restrict__ Pd,
                                                                    int pd_rows_per_seq, int vocab, const int* seq_row0,
                                                                    const int* seq_m, const int* n_cand, const int* n_accept,
                                                                    const float* __restrict__ u_res, int* next_tok) {
  __shared__ float chunk[EE_SAMPLE_THREADS];
  __shared__ int hit[2];
  const int b = blockIdx.x;
  const int m = seq_m[b];
  if (m == 0) { if (threadIdx.x == 0) next_tok[b] = -1; return; }
  const int a = n_accept[b], nc = n_cand[b];
  if (a >= m) { if (threadIdx.x == 0) next_tok[b] = -1; return; }      // all accepted and no further row
  const float* A = Pt + (size_t)(seq_row0[b] + a) * vocab;
  const float* Bd = a < nc ? Pd + ((size_t)b * pd_rows_per_seq + a) * vocab : nullptr;
  const int tok = draw_token(A, Bd, vocab, u_res[b], chunk, hit);
  if (threadIdx.x == 0) next_tok[b] = tok;
}
void k_rs_draw(hipStream_t st, const float* Pt, const float* Pd, int pd_rows_per_seq, int vocab, const CallMeta& meta, int B,
               const int* n_accept, const float* u_res, int* next_tok) {
  hipLaunchKernelGGL(rs_draw_kernel, dim3(B), dim3(EE_SAMPLE_THREADS), 0, st, Pt, Pd, pd_rows_per_seq, vocab, meta.seq_row0,
                     meta.seq_m, meta.n_cand, n_accept, u_res, next_tok);
}
