// Launchers of the HIP kernels (internal).  All work is enqueued on `st`; nothing synchronises.
#pragma once
#include "common.h"

// ---- dtype-independent ---------------------------------------------------------------------
// X[r][:] = float(emb[tok[r]][:])
void k_embed(hipStream_t st, bool bf16, const void* emb, const int* tok, float* X, int M, int d);
// dst[dst_idx[r]][:] = src[src_idx[r]][:]   (null index = identity)
void k_copy_rows(hipStream_t st, float* dst, const int* dst_idx, int dst_add, const float* src, const int* src_idx, int M, int d);
// per sequence: a = number of leading j < n_cand[b] with cand[b][j] == v[row0[b]+j];
// next = v[row0+a] if a < m[b] else -1.  Sequences with m[b] == 0 report (-1, -1).
void k_accept(hipStream_t st, const int* v, const CallMeta& meta, int cand_stride, int B, int* n_accept, int* next_tok);
// sequential drafting, one row per sequence: tok_next[r] = v[r]; draft_out[row_seq[r]*stride + j] = v[r]
void k_take_token(hipStream_t st, const int* v, const int* row_seq, int M, int* tok_next, int* draft_out, int stride, int j);
// cos/sin table for the rows of this call: cs[r][i] = (cos, sin)(pos_r * inv_freq[i]), evaluated in double
void k_rope_table(hipStream_t st, const CallMeta& mt, int pos_add, const double* inv_freq, float2* cs, int M, int half, int pps,
                  int4* rowinfo);   // rowinfo[r] = (first q-tile of the row's sequence, row inside the sequence, KV page, slot in page)
void k_fill_nan_dead_kv(hipStream_t st, bool bf16, void* kv, const int* pages, int n_owned_pages, int len,
                        int layer0, int layer1, int n_pages, int n_kv, int D);
void k_read_kv(hipStream_t st, bool bf16, const void* kv, const int* pages, int layer, int pos0, int n,
               int n_pages, int n_kv, int D, float* k_out, float* v_out);
void k_write_kv(hipStream_t st, bool bf16, void* kv, const int* pages, int layer, int pos0, int n, int n_pages, int n_kv, int D,
                const float* k_in, const float* v_in);

// ---- fp32 reference-precision path (EE_F32 models) -----------------------------------------
void f32_rmsnorm(hipStream_t st, const float* X, const float* g, float eps, float* out, int M, int d);
// Y[m][n] (+)= sum_k A[m][k] W[n][k];  A row-major lda, W row-major [N][K], Y row-major ldy
void f32_gemm(hipStream_t st, const float* A, int lda, const float* W, float* Y, int ldy, int M, int N, int K, bool add);
void f32_rope_append(hipStream_t st, const float* QKV, int ldq, const float2* cs, const CallMeta& meta, int pos_add, int M,
                     int Hq, int Hkv, int D, int layer, int n_pages, int pages_per_seq, float* Q, float* kv);
void f32_attention(hipStream_t st, const float* Q, const float* kv, const CallMeta& meta, int pos_add, int M, int Hq, int Hkv,
                   int D, int layer, int n_pages, int pages_per_seq, int max_ctx, float* out);
void f32_silu_mul(hipStream_t st, const float* GU, int ldg, float* H, int M, int F);
void f32_argmax(hipStream_t st, const float* logits, int M, int V, int* v);

// ---- bf16 MFMA path (EE_BF16 models) ---------------------------------------------------------
enum { EPI_ADD = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2, EPI_ROPE = 3 };
// Deferred RMSNorm of a GEMM's activation operand: the rows hold bf16(x * gain) and the per-row factor
// rsqrt(mean(x^2) + eps) is applied to the fp32 accumulators in the epilogue (it commutes with the
// product).  ssq holds partial sums of squares [n_part][stride] left by the GEMM that produced x;
// null = the operand is already fully normalised.
struct NormIn {
  const float* ssq = nullptr; int n_part = 0, stride = 0; float inv_d = 0.f, eps = 0.f;
  const float* inv_rms = nullptr;   // row-tiled GEMM only: the factors themselves, reduced from ssq beforehand
};
// EPI_ADD extra output: the updated residual rows as the next GEMM's operand, bf16(x * g) in fragment
// layout, plus this tile's partial sums of squares ssq[tile][row].
struct NormOut {
  const float* g = nullptr; bf16_t* xn = nullptr; int ktiles = 0; float* ssq = nullptr; int stride = 0;
};
// EPI_ROPE (fused QKV projection): rotate Q and K, write Q tiles for the attention kernel and K/V into
// their cache pages.
struct RopeOut {
  const float2* cs = nullptr;   // [rows][D/2] (cos, sin) of every row's position
  const int4* rowinfo = nullptr;   // [rows] (first q-tile of the row's sequence, row inside the sequence, KV page, slot in page)
  int Hq = 0, Hkv = 0, D = 0, layer = 0, n_pages = 0, total_qt = 0;
  bf16_t *Q = nullptr, *kv = nullptr;
};
struct GemmOut {
  float* Y = nullptr; int ldy = 0;        // EPI_ADD: residual stream, Y += product (row-major fp32); EPI_ARGMAX: optional logits
  float* Y2 = nullptr; const int* y2_idx = nullptr; int y2_add = 0;   // EPI_ADD: the new rows also go to Y2[y2_idx[row] + y2_add] (kept hidden rows of an exit)
  bf16_t* H = nullptr; int h_ktiles = 0;  // EPI_SWIGLU target (fragment layout)
  float* pmax = nullptr; int* pidx = nullptr; int pstride = 0;   // EPI_ARGMAX partials [row][pstride >= ntiles]
  NormIn nin;
  NormOut nout;
  RopeOut rope;
};
// Y^T tile = W tile (A operand) x X^T (B operand); W, A in fragment layout.  Rows go in passes of 32.
void bf16_gemm(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N, const GemmOut& out);
void bf16_gemm_cfg(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N,
                   const GemmOut& out, int nw, int ksplit, int U);
// Row-tiled variant for 16 < M <= 512 rows (rows start at row 0 of the operand; the kernel reads whole row
// tiles up to the next of 64, 128, 192, 256, 384, 512 rows, which the operand buffer must hold).  scratch: bf16_gemm_rows_scratch_floats() floats for
// this shape (may be null when that is 0); inv_rms: M floats of scratch for the deferred RMSNorm factors.
// Launch timing: while this points to a pair of events, the next skinny-GEMM launch attaches them to the dispatch
// itself (hipExtLaunchKernelGGL), so that they hold the kernel's own start and end rather than the times at which
// two marker packets around it were processed; the launcher sets `used`.
struct LaunchEvents { hipEvent_t start, stop; bool used; };
extern LaunchEvents* g_launch_events;
extern int g_attn_pages_override;   // <= 0: pages per KV split chosen from the call's shape; else that many (test hook: batch and solo runs then cut their contexts alike)
extern int g_rows_wide;              // 1: gate/up and exit head at 257..512 rows run sixteen weight tiles per workgroup in two row blocks; 0: eight in one
extern int g_rows_blocks_override;   // -1: built-in choice between K shares and row blocks; else 0, or row tiles per block (+100: eight weight tiles per workgroup)
size_t bf16_gemm_rows_scratch_floats(int ntiles, int ktiles);
void bf16_gemm_rows(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N,
                    const GemmOut& out, float* scratch, float* inv_rms);
void bf16_rmsnorm(hipStream_t st, const float* X, const float* g, float eps, bf16_t* out, int ktiles, int M, int d);
// Opens a pass over layers in one launch: row r of X <- embedding of tok[r] (emb set), rows[row_idx[r]] (rows set) or
// itself; out <- its RMSNorm with gain g as a GEMM operand; cs / rowinfo as k_rope_table fills them.
void bf16_begin_pass(hipStream_t st, const bf16_t* emb, const int* tok, const float* rows, const int* row_idx, float* X,
                     const float* g, float eps, bf16_t* out, int ktiles, int M, int d, const CallMeta& mt, int pos_add,
                     const double* inv_freq, float2* cs, int half, int pps, int4* rowinfo);
struct AttnScratch { float* part_o; float* part_ml; int max_splits; };
// pages each KV split takes, chosen from the call's sequence ends (kv_end[b] = first position past the
// block, 0 for a sequence not taking part) so that a ragged batch is cut into equal workgroups
int bf16_attention_pages_per_split(const int* kv_end, const int* seq_m, int B, int Hq, int Hkv, int max_splits);
// per = pages per KV split (ceil(max pages / per) must not exceed scr.max_splits)
void bf16_attention(hipStream_t st, const bf16_t* Q, const bf16_t* kv, const CallMeta& meta, int pos_add, int B, int max_m,
                    int total_qt, int max_kv_end, int Hq, int Hkv, int D, int layer, int n_pages, int pages_per_seq,
                    const AttnScratch& scr, bf16_t* out, int out_ktiles, int per);
void bf16_argmax_reduce(hipStream_t st, const float* pmax, const int* pidx, int ntiles, int pstride, int M, int* v);

// ---- rejection-sampling acceptance (kernels_sample.hip) ----
void k_softmax_rows(hipStream_t st, const float* in, size_t in_stride, float* out, const int* out_idx, int out_add, int M, int vocab);
void k_rs_accept(hipStream_t st, const float* Pt, const float* Pd, int pd_rows_per_seq, int vocab, const CallMeta& meta,
                 int cand_stride, int B, const float* u_acc, int u_stride, int* n_accept);
void k_draw_rows(hipStream_t st, const float* P, int rows_per_seq, int j, int vocab, const float* u, int u_stride,
                 const int* row_seq, int M, int* tok_next, int* draft_out, int stride);
void k_rs_draw(hipStream_t st, const float* Pt, const float* Pd, int pd_rows_per_seq, int vocab, const CallMeta& meta, int B,
               const int* n_accept, const float* u_res, int* next_tok);
