// bf16 MFMA path for gfx950: weight-streaming skinny GEMM with fused epilogues, k-query
// causal-in-block GQA attention over the paged KV cache (split over the KV axis), RMSNorm and
// RoPE + KV append producing MFMA-ready operand layouts.
//
// Everything is built around v_mfma_f32_16x16x32_bf16 (D = A*B + C, 16x16 output, K = 32):
//   A operand: lane l holds A[l%16][8*(l/16) .. +7]      B operand: lane l holds B[8*(l/16)..+7][l%16]
//   C/D:       lane l holds D[4*(l/16) + v][l%16], v = 0..3
// All operands are stored in HBM already in that per-lane order ("fragment layout", common.h), so a
// wavefront fetches an operand tile as one fully coalesced 1 KiB load straight into registers; no
// LDS staging or transposition is needed anywhere on the streaming path.
#include "kernels.h"
#include <hip/hip_ext.h>
#include <cmath>
#include <type_traits>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ inline f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ inline f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
// two fp32 -> packed bf16 pair (lo in bits 0..15), round to nearest even: one v_cvt_pk_bf16_f32
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: fp32 row in, bf16 fragment-layout row out (the next GEMM's B operand)
// ---------------------------------------------------------------------------------------------
// One workgroup per row; the row is read once as float4 into registers (all loads issued before the
// first use), reduced, scaled, and written as 8-byte bf16 quads (4 consecutive k share a fragment lane).
template <int CH>   // float4 chunks per thread: d <= 4 * 256 * CH
__global__ __launch_bounds__(256) void bf16_rmsnorm_kernel(const float* __restrict__ X, const float* __restrict__ g, float eps,
                                                           bf16_t* __restrict__ out, int ktiles, int d) {
  __shared__ float part[4];
  const int r = blockIdx.x, nch = d >> 2;
  const float4* x4 = (const float4*)(X + (size_t)r * d);
  const float4* g4 = (const float4*)g;
  float4 xv[CH], gv[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = threadIdx.x + i * 256;
    xv[i] = c < nch ? x4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
    gv[i] = c < nch ? g4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < CH; ++i) ss += xv[i].x * xv[i].x + xv[i].y * xv[i].y + xv[i].z * xv[i].z + xv[i].w * xv[i].w;
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_down(ss, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = threadIdx.x + i * 256;
    if (c < nch) {
      uint2 pk = make_uint2(pack2(xv[i].x * inv * gv[i].x, xv[i].y * inv * gv[i].y),
                            pack2(xv[i].z * inv * gv[i].z, xv[i].w * inv * gv[i].w));
      *(uint2*)(out + frag_offset(r, c * 4, ktiles)) = pk;
    }
  }
}
void bf16_rmsnorm(hipStream_t st, const float* X, const float* g, float eps, bf16_t* out, int ktiles, int M, int d) {
  // d is a multiple of 16 for bf16 models (checked at model load), so float4 access is aligned
  if (d <= 1024) hipLaunchKernelGGL((bf16_rmsnorm_kernel<1>), dim3(M), dim3(256), 0, st, X, g, eps, out, ktiles, d);
  else if (d <= 4096) hipLaunchKernelGGL((bf16_rmsnorm_kernel<4>), dim3(M), dim3(256), 0, st, X, g, eps, out, ktiles, d);
  else hipLaunchKernelGGL((bf16_rmsnorm_kernel<16>), dim3(M), dim3(256), 0, st, X, g, eps, out, ktiles, d);
}

// The first kernel of a pass over layers, one workgroup per row: brings the row into the residual stream X -- from the
// embedding table by token, from a buffer of kept hidden rows by index, or leaves it where it is --, writes its
// RMSNorm as the first projection's operand, and fills the row's rotary table and epilogue lookups (what
// rope_table_kernel does) on the side.  One launch where the pass used to open with three.
template <int CH>
__global__ __launch_bounds__(256) void bf16_begin_pass_kernel(const bf16_t* __restrict__ emb, const int* __restrict__ tok,
                                                              const float* __restrict__ rows, const int* __restrict__ row_idx,
                                                              float* __restrict__ X, const float* __restrict__ g, float eps,
                                                              bf16_t* __restrict__ out, int ktiles, int d, const int* row_pos,
                                                              int pos_add, const double* inv_freq, float2* cs, int half,
                                                              const int* row_seq, const int* seq_row0, const int* seq_qt0,
                                                              const int* block_table, int pps, int4* rowinfo) {
  __shared__ float part[4];
  const int r = blockIdx.x, nch = d >> 2;
  const float4* g4 = (const float4*)g;
  float4 xv[CH], gv[CH];
  if (emb) {
    const uint2* e2 = (const uint2*)(emb + (size_t)tok[r] * d);          // four bf16 per chunk
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = threadIdx.x + i * 256;
      const uint2 e = c < nch ? e2[c] : make_uint2(0u, 0u);
      xv[i] = make_float4(__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xffff0000u), __uint_as_float(e.y << 16),
                          __uint_as_float(e.y & 0xffff0000u));
    }
  } else {
    const float4* x4 = (const float4*)((rows ? rows : X) + (size_t)(row_idx ? row_idx[r] : r) * d);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = threadIdx.x + i * 256;
      xv[i] = c < nch ? x4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = threadIdx.x + i * 256;
    gv[i] = c < nch ? g4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const int pos = row_pos[r] + pos_add;
  for (int f = threadIdx.x; f < half; f += 256) {     // rotary angles in double, as in rope_table_kernel
    double sn, cn;
    sincos((double)pos * inv_freq[f], &sn, &cn);
    cs[(size_t)r * half + f] = make_float2((float)cn, (float)sn);
  }
  if (threadIdx.x == 0) {
    const int sq = row_seq[r];
    rowinfo[r] = make_int4(seq_qt0[sq], r - seq_row0[sq], block_table[sq * pps + pos / EE_PAGE], pos % EE_PAGE);
  }
  if (emb || rows) {
    float4* xo = (float4*)(X + (size_t)r * d);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = threadIdx.x + i * 256;
      if (c < nch) xo[c] = xv[i];
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < CH; ++i) ss += xv[i].x * xv[i].x + xv[i].y * xv[i].y + xv[i].z * xv[i].z + xv[i].w * xv[i].w;
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_down(ss, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = threadIdx.x + i * 256;
    if (c < nch) {
      uint2 pk = make_uint2(pack2(xv[i].x * inv * gv[i].x, xv[i].y * inv * gv[i].y),
                            pack2(xv[i].z * inv * gv[i].z, xv[i].w * inv * gv[i].w));
      *(uint2*)(out + frag_offset(r, c * 4, ktiles)) = pk;
    }
  }
}
void bf16_begin_pass(hipStream_t st, const bf16_t* emb, const int* tok, const float* rows, const int* row_idx, float* X,
                     const float* g, float eps, bf16_t* out, int ktiles, int M, int d, const CallMeta& mt, int pos_add,
                     const double* inv_freq, float2* cs, int half, int pps, int4* rowinfo) {
#define BEGIN_PASS(CH_)                                                                                                       \
  hipLaunchKernelGGL((bf16_begin_pass_kernel<CH_>), dim3(M), dim3(256), 0, st, emb, tok, rows, row_idx, X, g, eps, out, ktiles, d,  \
                     mt.row_pos, pos_add, inv_freq, cs, half, mt.row_seq, mt.seq_row0, mt.seq_qt0, mt.block_table, pps, rowinfo)
  if (d <= 1024) BEGIN_PASS(1);
  else if (d <= 4096) BEGIN_PASS(4);
  else BEGIN_PASS(16);
#undef BEGIN_PASS
}

// ---------------------------------------------------------------------------------------------
// Skinny GEMM  Y[m][n] = sum_k X[m][k] W[n][k],  M <= 16*MT rows per launch, weights streamed once.
// A task is one 16-row weight tile strip over the whole K, or two adjacent strips (NB = 2) when the
// epilogue needs both at once: gate and up of the same features (SwiGLU), or the two rotary halves of
// a head (RoPE).  A workgroup of nw waves runs nw/ksplit tasks; the ksplit waves of a task split K
// into contiguous chunks, each wave streaming its chunk (1 KiB per MFMA step) through two register
// sets of U k-tiles that take turns (one in flight while the other is multiplied); the partial 16x16
// tiles are then summed through LDS in a fixed order (deterministic) and the task's first wave runs
// the epilogue.
// The MFMA computes Y^T = W X^T so that a lane ends up with 4 consecutive n of one row m.
//
// Epilogues (everything between two projections is fused here, so a layer is five launches, six when the attention is split over the KV axis and merged):
//   EPI_ADD     residual add into the fp32 stream; optionally emits the next projection's operand
//               bf16(x_new * gain) and this tile's partial sum of squares per row (deferred RMSNorm)
//   EPI_SWIGLU  silu(gate) * up  -> bf16 operand of the down projection
//   EPI_ROPE    rotary embedding of Q and K; Q tiles for the attention kernel; K, V into cache pages
//   EPI_ARGMAX  per-row (max, arg max) of the tile (+ optional fp32 logits)
// Every epilogue first applies the operand's deferred RMSNorm factor (NormIn).
// ---------------------------------------------------------------------------------------------
// ---- epilogue of one 16 x 16 output tile (or tile pair), shared by the skinny and the row-tiled GEMM ----
// A lane of the epilogue wave holds, for row m = mt*16 + lane%16, the four consecutive outputs
// n = 16*tile + 4*(lane/16) .. +3 (acc[0]); for the paired epilogues acc[1] is the same lane's slice of the
// partner tile (up for gate, the rotary partner half for Q/K/V).
struct EpiPre {            // operands of the epilogue that do not depend on the product
  float4 res, gnext;       // EPI_ADD: residual row slice, gains of the next operand
  float4 rc01, rc23;       // EPI_ROPE: (cos, sin) of the lane's four rotary pairs
  int r_a, r_b;            // EPI_ROPE: Q heads: (global q-tile, row in tile); K/V heads: (page, position in page)
                           // EPI_ADD: r_a = row of the second destination
};

template <int EPI>
__device__ inline void epi_prefetch(EpiPre& p, const GemmOut& out, int task, int row, bool ok, int lane) {
  const int g = lane >> 4;
  p.res = p.gnext = make_float4(0.f, 0.f, 0.f, 0.f);
  p.rc01 = p.rc23 = make_float4(1.f, 0.f, 1.f, 0.f);
  p.r_a = p.r_b = 0;
  if (EPI == EPI_ADD) {
    const int n = task * 16 + 4 * g;
    if (ok) p.res = *(const float4*)(out.Y + (size_t)row * out.ldy + n);
    if (out.nout.xn) p.gnext = *(const float4*)(out.nout.g + n);
    if (out.Y2 && ok) p.r_a = out.y2_idx[row] + out.y2_add;
  }
  if (EPI == EPI_ROPE && ok) {
    const RopeOut& R = out.rope;
    const int half = R.D >> 1, tph = R.D >> 5;
    const int h = task / tph, f = (task % tph) * 16 + 4 * g;
    const int4 ri = R.rowinfo[row];              // (every operand here is indexed by the row alone: no dependent loads)
    if (h < R.Hq + R.Hkv) {
      const float4* c4 = (const float4*)(R.cs + (size_t)row * half + f);
      p.rc01 = c4[0]; p.rc23 = c4[1];
    }
    if (h < R.Hq) {
      const int q = ri.y * (R.Hq / R.Hkv) + h % (R.Hq / R.Hkv);
      p.r_a = ri.x + (q >> 4); p.r_b = q & 15;
    } else {
      p.r_a = ri.z; p.r_b = ri.w;
    }
  }
}

// sc: the row's deferred RMSNorm factor (1 when the operand was already normalised)
template <int EPI>
__device__ inline void epi_apply(const f32x4& acc0, const f32x4& acc1, float sc, const EpiPre& p, const GemmOut& out, int task,
                                 int row, bool ok, int N, int lane) {
  const int g = lane >> 4;
  if (EPI == EPI_ADD) {
    const int n = task * 16 + 4 * g;
    float4 r = make_float4(acc0[0] * sc, acc0[1] * sc, acc0[2] * sc, acc0[3] * sc);
    r.x += p.res.x; r.y += p.res.y; r.z += p.res.z; r.w += p.res.w;
    if (ok) *(float4*)(out.Y + (size_t)row * out.ldy + n) = r;
    if (out.Y2 && ok) *(float4*)(out.Y2 + (size_t)p.r_a * out.ldy + n) = r;
    if (out.nout.xn) {
      const float4 gn = p.gnext;
      if (ok) *(uint2*)(out.nout.xn + frag_offset(row, n, out.nout.ktiles)) = make_uint2(pack2(r.x * gn.x, r.y * gn.y), pack2(r.z * gn.z, r.w * gn.w));
      float ss = ok ? (r.x * r.x + r.y * r.y) + (r.z * r.z + r.w * r.w) : 0.f;
      ss += __shfl_xor(ss, 16, 64);
      ss += __shfl_xor(ss, 32, 64);
      if (g == 0) out.nout.ssq[(size_t)task * out.nout.stride + row] = ss;
    }
  } else if (EPI == EPI_SWIGLU) {
    const int f = task * 16 + 4 * g;     // h[m][f..f+3] = silu(gate) * up
    if (ok) {
      float h[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float gt = acc0[v] * sc, up = acc1[v] * sc;
        h[v] = gt / (1.0f + __expf(-gt)) * up;
      }
      *(uint2*)(out.H + frag_offset(row, f, out.h_ktiles)) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
    }
  } else if (EPI == EPI_ROPE) {
    // task = (head h, 16 rotary pairs f0..f0+15): acc0 holds features f, acc1 their partners f + D/2
    const RopeOut& R = out.rope;
    const int D = R.D, half = D >> 1, tph = D >> 5;
    const int h = task / tph, f = (task % tph) * 16 + 4 * g;
    if (ok) {
      float lo[4], hi[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) { lo[v] = acc0[v] * sc; hi[v] = acc1[v] * sc; }
      if (h < R.Hq + R.Hkv) {
        const float cx[4] = {p.rc01.x, p.rc01.z, p.rc23.x, p.rc23.z}, sy[4] = {p.rc01.y, p.rc01.w, p.rc23.y, p.rc23.w};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float a = lo[v], b = hi[v];
          lo[v] = a * cx[v] - b * sy[v];
          hi[v] = b * cx[v] + a * sy[v];
        }
      }
      const uint2 plo = make_uint2(pack2(lo[0], lo[1]), pack2(lo[2], lo[3]));
      const uint2 phi = make_uint2(pack2(hi[0], hi[1]), pack2(hi[2], hi[3]));
      if (h < R.Hq) {
        const int kvh = h / (R.Hq / R.Hkv), q15 = p.r_b;
        const size_t tile = ((size_t)kvh * R.total_qt + p.r_a) * tph;
        const int d1 = f + half;
        *(uint2*)(R.Q + ((tile + (f >> 5)) * 64 + ((f & 31) >> 3) * 16 + q15) * 8 + (f & 7)) = plo;
        *(uint2*)(R.Q + ((tile + (d1 >> 5)) * 64 + ((d1 & 31) >> 3) * 16 + q15) * 8 + (d1 & 7)) = phi;
      } else {
        const int page = p.r_a, pp = p.r_b;
        if (h < R.Hq + R.Hkv) {
          bf16_t* slab = R.kv + kv_slab(R.layer, page, h - R.Hq, R.n_pages, R.Hkv, D);
          *(uint2*)(slab + k_page_off(pp, f, D)) = plo;
          *(uint2*)(slab + k_page_off(pp, f + half, D)) = phi;
        } else {
          bf16_t* slab = R.kv + kv_slab(R.layer, page, h - R.Hq - R.Hkv, R.n_pages, R.Hkv, D) + EE_PAGE * D;
          const uint32_t wl[2] = {plo.x, plo.y}, wh[2] = {phi.x, phi.y};
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            slab[v_page_off(pp, f + v, D)] = (bf16_t)(wl[v >> 1] >> (16 * (v & 1)));
            slab[v_page_off(pp, f + half + v, D)] = (bf16_t)(wh[v >> 1] >> (16 * (v & 1)));
          }
        }
      }
    }
  } else {   // EPI_ARGMAX: per-row (max, arg max) over this tile's 16 outputs; lowest index wins ties
    float best = -INFINITY; int bi = 0x7fffffff;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = task * 16 + 4 * g + v;
      const float t = acc0[v] * sc;
      if (n < N) {
        if (out.Y && ok) out.Y[(size_t)row * out.ldy + n] = t;
        if (t > best) { best = t; bi = n; }
      }
    }
#pragma unroll
    for (int sh = 16; sh <= 32; sh <<= 1) {
      const float ob = __shfl_xor(best, sh, 64); const int oi = __shfl_xor(bi, sh, 64);
      if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    if (g == 0 && ok) {
      out.pmax[(size_t)row * out.pstride + task] = best;
      out.pidx[(size_t)row * out.pstride + task] = bi;
    }
  }
}

template <int MT, int NB, int U>
struct Frags {
  u32x4 w[NB][U];
  u32x4 x[MT][U];
};

// Requests the fragments of k-tiles kt .. kt+U-1 (indices past `last` repeat the last k-tile: valid memory; the
// caller leaves those out of the product).  Nothing here touches a loaded value, so the wave does not wait.
template <int MT, int NB, int U>
__device__ inline void load_frags(Frags<MT, NB, U>& f, const u32x4* const (&wp)[NB], const u32x4* ap, int ktiles, int kt, int last) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int k = min(kt + u, last);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) f.w[nb][u] = __builtin_nontemporal_load(&wp[nb][(size_t)k * 64]);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) f.x[mt][u] = ap[((size_t)mt * ktiles + k) * 64];
  }
}
// acc += the product over the k-tiles kt .. kt+U-1 held in f; GUARD: only those below kt1 (kt and kt1 must be
// uniform in a way the compiler can see, see the kernel)
template <int MT, int NB, int U, bool GUARD>
__device__ inline void mma_frags(f32x4 (&acc)[NB][MT], const Frags<MT, NB, U>& f, int kt, int kt1) {
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (!GUARD || kt + u < kt1) {         // (uniform)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = mfma16(f.w[nb][u], f.x[mt][u], acc[nb][mt]);
    }
}

template <int MT, int EPI, int U>
__global__ __launch_bounds__(64 * EE_MAX_WAVES) void gemm_skinny_kernel(const uint4* __restrict__ W, int ktiles, int ntasks,
                                                                        const uint4* __restrict__ A, int row0, int M, int N,
                                                                        GemmOut out, int ksplit) {
  constexpr int NB = (EPI == EPI_SWIGLU || EPI == EPI_ROPE) ? 2 : 1;
  __shared__ float4 red[EE_MAX_WAVES - 1][NB * MT][64];
  __shared__ float ssq_red[EE_MAX_WAVES][MT * 16];
  // The wave's number is taken through a scalar register: the compiler then knows that everything derived from it (the
  // task, the K share and above all the conditions around the MFMAs of a short last group) is uniform and branches
  // on it.  A condition it takes for divergent it may turn into an EXEC mask without a branch -- and the matrix
  // instructions ignore EXEC, so a masked-off MFMA would still add its product.
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
  const int task = blockIdx.x * (nw / ksplit) + wave / ksplit, kpart = wave % ksplit;
  const bool active = task < ntasks;
  const int per = (ktiles + ksplit - 1) / ksplit;
  const int kt0 = kpart * per, kt1 = min(ktiles, kt0 + per);

  f32x4 acc[NB][MT];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const bool stream = active && kt0 < kt1;
  const u32x4* wp[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) wp[nb] = (const u32x4*)W + (size_t)(task * NB + nb) * ktiles * 64 + lane;
  const u32x4* ap = (const u32x4*)A + (size_t)(row0 >> 4) * ktiles * 64 + lane;
  Frags<MT, NB, U> cur;

  // Order of the requests: the partial sums of squares of the deferred RMSNorm (small, mostly L2), then the first
  // weight fragments, then the epilogue's operands; the sums are formed once their loads are back, which frees their
  // registers for the second set of fragments.  The load counter is in order, so nothing here waits for the weights.
  constexpr int SB = 16 / MT;   // 16-byte loads per lane and m-tile in one batch (64 registers in all)
  const bool normed = out.nin.ssq != nullptr && active;
  const int mc = lane & 15;
  const bool epi_wave = active && kpart == 0;
  EpiPre pre[MT];
  float ssl[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) ssl[mt] = 0.f;
  {
    // Deferred RMSNorm: sum of squares of row mt*16 + lane%16 from the producer's per-tile partials [partial][row], in
    // a fixed order.  The ksplit waves of a task each sum a contiguous share of the partials; a lane loads four rows
    // (lane % 4) of every 16th partial (lane / 4) at a time, the lanes' sums then meet in a butterfly.
    const int np = normed ? out.nin.n_part : 0, cp = (np + ksplit - 1) / ksplit;
    const int c0 = kpart * cp + (lane >> 2), c1 = min(np, (kpart + 1) * cp);
    const float* p = out.nin.ssq + row0 + 4 * (lane & 3);
    float4 t[MT][SB];
    if (normed) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < SB; ++j) t[mt][j] = *(const float4*)(p + (size_t)min(c0 + 16 * j, np - 1) * out.nin.stride + mt * 16);
    }
    if (stream) load_frags<MT, NB, U>(cur, wp, ap, ktiles, kt0, kt1 - 1);
    if (epi_wave) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) epi_prefetch<EPI>(pre[mt], out, task, row0 + mt * 16 + mc, mt * 16 + mc < M, lane);
    }
    if (normed) {
      float4 sv[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        sv[mt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < SB; ++j)
          if (c0 + 16 * j < c1) { sv[mt].x += t[mt][j].x; sv[mt].y += t[mt][j].y; sv[mt].z += t[mt][j].z; sv[mt].w += t[mt][j].w; }
      }
      for (int b0 = c0 + 16 * SB; b0 < c1; b0 += 16 * SB)      // (more partials than one batch: wide models, several row tiles)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
          for (int j = 0; j < SB; ++j) t[mt][j] = *(const float4*)(p + (size_t)min(b0 + 16 * j, np - 1) * out.nin.stride + mt * 16);
#pragma unroll
          for (int j = 0; j < SB; ++j)
            if (b0 + 16 * j < c1) { sv[mt].x += t[mt][j].x; sv[mt].y += t[mt][j].y; sv[mt].z += t[mt][j].z; sv[mt].w += t[mt][j].w; }
        }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int sh = 4; sh < 64; sh <<= 1) {
          sv[mt].x += __shfl_xor(sv[mt].x, sh, 64); sv[mt].y += __shfl_xor(sv[mt].y, sh, 64);
          sv[mt].z += __shfl_xor(sv[mt].z, sh, 64); sv[mt].w += __shfl_xor(sv[mt].w, sh, 64);
        }
        // lanes with lane % 4 == q now hold rows 4q .. 4q+3; this lane wants row mc
        const float a = __shfl(sv[mt].x, mc >> 2, 64), b = __shfl(sv[mt].y, mc >> 2, 64);
        const float c = __shfl(sv[mt].z, mc >> 2, 64), e = __shfl(sv[mt].w, mc >> 2, 64);
        ssl[mt] = (mc & 2) ? ((mc & 1) ? e : c) : ((mc & 1) ? b : a);
      }
    }
  }

  // Two register sets of fragments take turns: while one is multiplied the other is in flight, and the next request
  // for a set goes out as soon as its MFMAs are issued.
  if (stream) {
    // Groups of U k-tiles; only the last one can be short.  In the loop every fragment requested is multiplied, with
    // no condition in between -- a request whose data might go unused would make the compiler drain the load counter
    // before the registers are requested again, and with it the set in flight.
    Frags<MT, NB, U> oth;
    const int last = kt1 - 1;
    int kt = kt0;
    for (; kt + 2 * U < kt1; kt += 2 * U) {
      load_frags<MT, NB, U>(oth, wp, ap, ktiles, kt + U, last);
      mma_frags<MT, NB, U, false>(acc, cur, kt, kt1);
      load_frags<MT, NB, U>(cur, wp, ap, ktiles, kt + 2 * U, last);
      mma_frags<MT, NB, U, false>(acc, oth, kt + U, kt1);
    }
    if (kt + U < kt1) {                  // two groups left
      load_frags<MT, NB, U>(oth, wp, ap, ktiles, kt + U, last);
      mma_frags<MT, NB, U, false>(acc, cur, kt, kt1);
      mma_frags<MT, NB, U, true>(acc, oth, kt + U, kt1);
    } else {
      mma_frags<MT, NB, U, true>(acc, cur, kt, kt1);
    }
  }

  // fixed-order reduction over the K parts of a task (every wave reaches the barrier)
  if (ksplit > 1) {   // uniform branch
    if (normed && lane < 16) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) ssq_red[wave][mt * 16 + lane] = ssl[mt];
    }
    if (kpart > 0) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          red[wave - 1][nb * MT + mt][lane] = make_float4(acc[nb][mt][0], acc[nb][mt][1], acc[nb][mt][2], acc[nb][mt][3]);
    }
    __syncthreads();
  }
  if (kpart != 0 || !active) return;
  for (int w = 1; w < ksplit; ++w)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        float4 t = red[wave + w - 1][nb * MT + mt][lane];
        acc[nb][mt][0] += t.x; acc[nb][mt][1] += t.y; acc[nb][mt][2] += t.z; acc[nb][mt][3] += t.w;
      }

#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + mc;
    float sc = 1.0f;
    if (normed) {
      float ss = ssl[mt];
      for (int w = 1; w < ksplit; ++w) ss += ssq_red[wave + w][m];
      sc = 1.0f / sqrtf(ss * out.nin.inv_d + out.nin.eps);
    }
    epi_apply<EPI>(acc[0][mt], acc[NB - 1][mt], sc, pre[mt], out, task, row0 + m, m < M, N, lane);
  }
}

// ---------------------------------------------------------------------------------------------
// Row-tiled GEMM for a block of 16 < M <= 512 rows: weights cross HBM once per block, but every weight fragment now
// meets up to 32 row tiles, so the kernel sits near the machine's ridge (M flop per weight byte).
// Workgroup = 8 waves (two per SIMD: one wave alone does not keep a matrix pipe busy) on a group of
// 8 weight tiles (128 output features) and a share of K (grid.y); wave (rq, nh) owns 4 of the tiles and a
// quarter of the TMT row tiles (every fourth one): TMT accumulators.  Row tiles past the last row are neither
// requested nor multiplied.
// Both operands reach LDS by direct global->LDS loads (no staging registers, no LDS store
// instructions): a ring of S stages, one k-tile each (8 KiB of weights + TMT KiB of activations), as many
// as LDS holds, of which up to S-2 are in flight: that is what covers the HBM latency with one workgroup
// per compute unit.  Each wave requests one weight tile and one or two row tiles of every stage; per
// k-tile it waits until its own share of the next stage has landed (the load counter is in order), meets
// the other waves at a barrier -- which also says that everyone is past the MFMAs of the previous stage,
// whose slot the next request then overwrites -- reads the next stage's fragments (1 KiB, lane-linear,
// conflict-free) into the second register set and runs the TMT MFMAs of the current one under them.  The
// loop is unrolled over the ring so that every LDS address is a constant, and indices past the end are
// clamped (only the MFMAs are guarded).
// With grid.y == 1 the epilogue is fused; otherwise fp32 partial tiles go to scratch and
// gemm_rows_reduce_kernel sums the K shares in a fixed order and runs the same epilogue.
// ---------------------------------------------------------------------------------------------
#define EE_ROWS_TN 4
// s_waitcnt immediate: at most n vector-memory loads outstanding, all LDS reads done, export counter untouched
__host__ __device__ constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }

template <int TMT, int EPI, bool FULL, int TN>
__global__ __launch_bounds__(512) void gemm_rows_kernel(const uint4* __restrict__ W, int ktiles, int ntiles,
                                                        const uint4* __restrict__ A, int row0, int M_all, int N, GemmOut out,
                                                        int per, float* __restrict__ partial) {
  // rows row0 .. row0+M_all-1 of the operand (row0 a multiple of 16), of which this workgroup takes the block of
  // TMT*16 rows that blockIdx.z names; the deferred-norm factors and the K-share partials are indexed from row0,
  // everything the epilogue touches by the row itself
  constexpr int NB = (EPI == EPI_SWIGLU || EPI == EPI_ROPE) ? 2 : 1;
  static_assert(TN == 2 || TN == 4 || TN == 8, "weight tiles per wave");
  // TN = 8 (sixteen weight tiles per workgroup, rows in two blocks): the grid is one-dimensional and workgroups L and
  // L + 8 are the two row blocks of one column group -- dispatched together and on the same XCD (L mod 8), so the
  // weights cross HBM once and the second reader finds them in that XCD's L2
  const int bx = TN == 8 ? (int)(((blockIdx.x >> 4) << 3) | (blockIdx.x & 7)) : (int)blockIdx.x;
  const int bz = TN == 8 ? (int)((blockIdx.x >> 3) & 1) : (int)blockIdx.z;
  if (TN == 8 && (bx * (2 * TN) >= ntiles || bz * (TMT * 16) >= M_all)) return;       // whole workgroup
  const int rbase = bz * (TMT * 16), M = min(M_all - rbase, TMT * 16);
  constexpr int TMW = TMT / 4;                      // row tiles per wave
  static_assert(TMT % 4 == 0 && TMT >= 4 && TMT <= 32, "row tiles split four ways");
  constexpr int STAGE = (2 * TN + TMT) * 64;        // 16-byte units: weight tiles first, then row tiles
  constexpr int S = (160 / (2 * TN + TMT)) & ~1;    // stages in the ring: what 160 KiB of LDS holds (even: fragments alternate between two register sets)
  constexpr int XHI = (TMT + 7) / 8;                // row tiles a wave requests per stage at most: wave, wave+8, ...
  constexpr int WHI = TN == 8 ? 2 : 1;              // weight tiles a wave requests per stage: wave (and wave+8)
  constexpr int LHI = WHI + XHI;                    // requests per stage at most
  static_assert((S - 1) * LHI < 64, "the load counter has six bits");
  __shared__ u32x4 ring[S][STAGE];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);      // the same number, known to be uniform
  const int rq = wave_s >> 1, nh = wave_s & 1;
  const int rqv = wave >> 1, nhv = wave & 1;                    // the same again from the vector register: one address register
                                                                // serves all LDS reads, the slots being constant offsets from it
  const int nt0 = bx * (2 * TN) + nh * TN;                      // first weight tile of this wave
  // Row tiles of this wave: TMW in a row when all of them hold rows (FULL: the guards below fold away), else
  // rq, rq+4, ..., so that the tiles past the last row, which are neither requested nor multiplied, are spread
  // over the four wave pairs.  The launcher picks the smallest TMT that holds the rows, so the unused tiles are
  // among the last eight.
  constexpr int MT_STEP = FULL ? 1 : 4;                         // tile of accumulator mt: mt_first + mt * MT_STEP
  const int mt_first = FULL ? rq * TMW : rq;
  const int mt_used = FULL ? TMT : (M + 15) >> 4;
  const int kt0 = blockIdx.y * per, kt1 = min(ktiles, kt0 + per);
  if (kt0 >= kt1) return;                                       // whole workgroup (never with the launcher's shapes)
  const int last = kt1 - 1;

  f32x4 acc[TN][TMW];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int mt = 0; mt < TMW; ++mt) acc[tn][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // this wave's share of a stage: weight tile `wave` of the group and row tiles wave, wave+8, ... (every
  // wave requests both kinds with the same lead: a wave's load counter is in order, so it could not wait
  // for a recent request without draining all its older ones)
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  // this wave's last row tile holds rows: XHI requests per stage, else one less; with four weight tiles per
  // workgroup (TN = 2) only the first four waves request one
  const bool hi = (FULL && TMT % 8 == 0) || wave_s + 8 * (XHI - 1) < mt_used;
  const bool wreq = TN >= 4 || wave_s < 2 * TN;
  // LDS byte address of this wave's weight tile in stage 0 as a scalar: every request's LDS address is this plus a
  // constant, so none of them occupies a vector register (measured: 3-4 % at 24 and 32 row tiles)
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)&ring[0][0]) + 1024u * wave_s;
#define ROWS_LDS(slot_, tile_) ((lptr_t)(size_t)(lds0 + 16u * ((slot_) * STAGE + (tile_) * 64)))
  const u32x4* wsrc = (const u32x4*)W + (size_t)min(bx * (2 * TN) + wave, ntiles - 1) * ktiles * 64 + lane;
  const u32x4* wsrc2 = (const u32x4*)W + (size_t)min(bx * (2 * TN) + wave + 8, ntiles - 1) * ktiles * 64 + lane;   // (TN = 8)
  const u32x4* xsrc = (const u32x4*)A + (size_t)(((row0 + rbase) >> 4) + wave) * ktiles * 64 + lane;
  // (weights: streaming hint, except where a second workgroup is to find them in L2)
#define ROWS_REQUEST(slot_, kt_)                                                                              \
  do {                                                                                                        \
    const size_t k_ = (size_t)min(kt_, last) * 64;                                                            \
    if (wreq) __builtin_amdgcn_global_load_lds((gptr_t)(wsrc + k_), ROWS_LDS(slot_, 0), 16, 0, 2);                \
    if (TN == 8) __builtin_amdgcn_global_load_lds((gptr_t)(wsrc2 + k_), ROWS_LDS(slot_, 8), 16, 0, 2);        \
    _Pragma("unroll") for (int j = 0; j < XHI - 1; ++j)                                                       \
      __builtin_amdgcn_global_load_lds((gptr_t)(xsrc + (size_t)(8 * j) * ktiles * 64 + k_),                   \
                                       ROWS_LDS(slot_, 2 * TN + 8 * j), 16, 0, 0);                            \
    if (hi)                                                                                                   \
      __builtin_amdgcn_global_load_lds((gptr_t)(xsrc + (size_t)(8 * (XHI - 1)) * ktiles * 64 + k_),           \
                                       ROWS_LDS(slot_, 2 * TN + 8 * (XHI - 1)), 16, 0, 0);                    \
  } while (0)
#define ROWS_WAIT(stages_)                                                                                    \
  do {                                                                                                        \
    if (wreq && hi) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((stages_) * LHI));                            \
    else if (wreq) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((stages_) * (LHI - 1)));                       \
    else if (hi) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((stages_) * XHI));                               \
    else __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((stages_) * (XHI - 1)));                                 \
  } while (0)
#define ROWS_READ(buf_, slot_)                                                                               \
  do {                                                                                                        \
    const u32x4* wl_ = &ring[slot_][(nhv * TN) * 64 + lane];                                                  \
    const u32x4* xl_ = &ring[slot_][(2 * TN + (FULL ? rqv * TMW : rqv)) * 64 + lane];                         \
    _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) wf[buf_][tn] = wl_[tn * 64];                            \
    _Pragma("unroll") for (int mt = 0; mt < TMW; ++mt) xf[buf_][mt] = xl_[mt * MT_STEP * 64];                 \
  } while (0)
  u32x4 wf[2][TN], xf[2][TMW];      // fragments of the k-tile being multiplied and of the next one
#pragma unroll
  for (int s = 0; s < S - 1; ++s) ROWS_REQUEST(s, kt0 + s);
  ROWS_WAIT(S - 2);
  __builtin_amdgcn_s_barrier();
  ROWS_READ(0, 0);
  // One k-tile: own share of stage u+1 landed and own fragment reads done; then everybody's, and everybody
  // is past the MFMAs of stage u-1, whose slot the next request overwrites.  The requests and the reads of
  // the next fragments do not depend on this k-tile's MFMAs and ride along with them, one row tile's four
  // MFMAs at a time (the scheduling barriers pin that order): issued in one burst after the barrier, the
  // eight waves' LDS reads would queue up while the matrix pipes sit idle.
#define ROWS_STEP(u_, guard_)                                                                                 \
  do {                                                                                                        \
    ROWS_WAIT(S - 3);                                                                                         \
    __builtin_amdgcn_s_barrier();                                                                             \
    const int cb_ = (u_) & 1, nb_ = cb_ ^ 1, ns_ = ((u_) + 1) % S;                                            \
    ROWS_REQUEST(((u_) + S - 1) % S, kt + (u_) + S - 1);                                                      \
    const u32x4* wl_ = &ring[ns_][(nhv * TN) * 64 + lane];                                                    \
    const u32x4* xl_ = &ring[ns_][(2 * TN + (FULL ? rqv * TMW : rqv)) * 64 + lane];                           \
    const bool on_ = !(guard_) || kt + (u_) < kt1;                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                        \
    _Pragma("unroll") for (int mt = 0; mt < TMW; ++mt) {                                                      \
      _Pragma("unroll") for (int tn = mt * TN / TMW; tn < (mt + 1) * TN / TMW; ++tn) wf[nb_][tn] = wl_[tn * 64]; \
      xf[nb_][mt] = xl_[mt * MT_STEP * 64];                                                                   \
      if (on_ && (FULL || 4 * mt + 11 < TMT || rq + 4 * mt < mt_used)) {                                      \
        _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) acc[tn][mt] = mfma16(wf[cb_][tn], xf[cb_][mt], acc[tn][mt]); \
      }                                                                                                       \
      __builtin_amdgcn_sched_barrier(0);                                                                      \
    }                                                                                                         \
  } while (0)
  // of the two waves that share a SIMD the hardware favours the older one; the younger four get the higher
  // priority so that both reach the barrier closer together (measured: 1-3 % at 144 rows)
  if (wave_s >= 4) __builtin_amdgcn_s_setprio(2);
  int kt = kt0;
  for (; kt + S <= kt1; kt += S) {
#pragma unroll
    for (int u = 0; u < S; ++u) ROWS_STEP(u, false);
  }
  if (kt < kt1) {                                  // fewer than S k-tiles left: same steps, MFMAs guarded
#pragma unroll
    for (int u = 0; u < S; ++u) ROWS_STEP(u, true);
  }
#undef ROWS_STEP
#undef ROWS_READ
#undef ROWS_WAIT
#undef ROWS_REQUEST
#undef ROWS_LDS
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));              // requests past the end have landed before the wave moves on

  const int mc = lane & 15;
  if (gridDim.y > 1) {
    // K share: raw accumulator tiles [k share][weight tile][row tile][lane] for the reduce kernel
    f32x4* pp = (f32x4*)partial + (size_t)blockIdx.y * ntiles * TMT * 64 + lane;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      if (nt0 + tn >= ntiles) continue;
#pragma unroll
      for (int mt = 0; mt < TMW; ++mt)
        if (mt_first + mt * MT_STEP < mt_used)
          __builtin_nontemporal_store(acc[tn][mt], pp + ((size_t)(nt0 + tn) * TMT + mt_first + mt * MT_STEP) * 64);
    }
    return;
  }
#pragma unroll
  for (int t = 0; t < TN / NB; ++t) {
    const int nt = nt0 + t * NB;
    if (nt >= ntiles) continue;
    const int task = nt / NB;
#pragma unroll
    for (int mt = 0; mt < TMW; ++mt) {
      const int m = (mt_first + mt * MT_STEP) * 16 + mc;
      if (mt_first + mt * MT_STEP >= mt_used) continue;
      const float sc = out.nin.inv_rms ? out.nin.inv_rms[rbase + min(m, M - 1)] : 1.0f;
      EpiPre pre;
      epi_prefetch<EPI>(pre, out, task, row0 + rbase + m, m < M, lane);
      epi_apply<EPI>(acc[t * NB][mt], acc[t * NB + NB - 1][mt], sc, pre, out, task, row0 + rbase + m, m < M, N, lane);
    }
  }
}

// sums the K shares of one (task, row tile) in a fixed order and runs the epilogue; one wave per unit
template <int EPI>
__global__ __launch_bounds__(256) void gemm_rows_reduce_kernel(const float* __restrict__ partial, int ksplit, int ntiles, int TMT,
                                                               int row0, int M, int N, GemmOut out) {
  constexpr int NB = (EPI == EPI_SWIGLU || EPI == EPI_ROPE) ? 2 : 1;
  const int lane = threadIdx.x & 63, mc = lane & 15;
  const int mtiles = (M + 15) >> 4;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int task = unit / mtiles, mt = unit % mtiles;
  if (task * NB >= ntiles) return;
  const int m = mt * 16 + mc;
  EpiPre pre;
  epi_prefetch<EPI>(pre, out, task, row0 + m, m < M, lane);
  const float sc = out.nin.inv_rms ? out.nin.inv_rms[min(m, M - 1)] : 1.0f;
  f32x4 acc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const f32x4* pp = (const f32x4*)partial + ((size_t)(task * NB + nb) * TMT + mt) * 64 + lane;
    for (int s0 = 0; s0 < ksplit; s0 += 8) {
      f32x4 t[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = __builtin_nontemporal_load(pp + (size_t)min(s0 + i, ksplit - 1) * ntiles * TMT * 64);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (s0 + i < ksplit) acc[nb] += t[i];
    }
  }
  epi_apply<EPI>(acc[0], acc[NB - 1], sc, pre, out, task, row0 + m, m < M, N, lane);
}

// per-row factor rsqrt(mean(x^2) + eps) from the producer's per-tile partial sums of squares, in a fixed order:
// one wave per row, every lane taking each 64th partial with four loads in flight
__global__ __launch_bounds__(256) void norm_factor_kernel(const float* __restrict__ ssq, int n_part, int stride, float inv_d, float eps,
                                                          float* __restrict__ inv_rms, int M) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), t = threadIdx.x & 63;
  if (row >= M) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int i = t;
  for (; i + 192 < n_part; i += 256) {
    const float a = ssq[(size_t)i * stride + row], b = ssq[(size_t)(i + 64) * stride + row];
    const float c = ssq[(size_t)(i + 128) * stride + row], d = ssq[(size_t)(i + 192) * stride + row];
    s0 += a; s1 += b; s2 += c; s3 += d;
  }
  for (; i < n_part; i += 64) s0 += ssq[(size_t)i * stride + row];
  float ss = (s0 + s1) + (s2 + s3);
  for (int sh = 1; sh < 64; sh <<= 1) ss += __shfl_xor(ss, sh, 64);
  if (t == 0) inv_rms[row] = 1.0f / sqrtf(ss * inv_d + eps);
}

// number of K shares the row-tiled GEMM runs with: enough workgroups for the chip, at least 16 k-tiles each
static int rows_ksplit(int ntiles, int ktiles) {
  const int groups = ceil_div(ntiles, 2 * EE_ROWS_TN);
  int ks = groups >= 192 ? 1 : min(8, ceil_div(224, groups));
  while (ks > 1 && ktiles / ks < 16) --ks;
  return ks;
}
size_t bf16_gemm_rows_scratch_floats(int ntiles, int ktiles) {
  const int ks = rows_ksplit(ntiles, ktiles);
  return ks > 1 ? (size_t)ks * ntiles * 32 * 256 : 0;       // [k share][weight tile][up to 32 row tiles][64 lanes x 4]
}

// plain launch, or with the offered timing events attached to the dispatch
template <typename K, typename... Args>
static void launch_timed(LaunchEvents* ev, K kernel, dim3 grid, dim3 blk, hipStream_t st, Args... args) {
  if (ev) {
    hipExtLaunchKernelGGL(kernel, grid, blk, 0, st, ev->start, ev->stop, 0, args...);
    ev->used = true;
  } else {
    hipLaunchKernelGGL(kernel, grid, blk, 0, st, args...);
  }
}

template <int TMT>
static void launch_gemm_rows(hipStream_t st, int epi, const uint4* W, int ntiles, int ktiles, const uint4* A, int row0, int M, int N,
                             const GemmOut& out, float* scratch) {
  const int ks = rows_ksplit(ntiles, ktiles), per = ceil_div(ktiles, ks);
  dim3 grid(ceil_div(ntiles, 2 * EE_ROWS_TN), ceil_div(ktiles, per)), blk(512), rblk(256);
  const int ksr = grid.y;
  // every row tile holds rows; with 32 row tiles the kernel has no register to spare for the other variant
  const bool full = M > TMT * 16 - 16 || TMT == 32;
  // timing events are taken when this one kernel is the whole call (no K shares, hence no reduction pass)
  LaunchEvents* ev = ksr == 1 ? g_launch_events : nullptr;
  if (ev) g_launch_events = nullptr;
#define ROWS_LAUNCH(E_)                                                                                                          \
  do {                                                                                                                           \
    if (full) launch_timed(ev, gemm_rows_kernel<TMT, E_, true, EE_ROWS_TN>, grid, blk, st, W, ktiles, ntiles, A, row0, M, N, out, per, scratch); \
    else launch_timed(ev, gemm_rows_kernel<TMT, E_, TMT == 32, EE_ROWS_TN>, grid, blk, st, W, ktiles, ntiles, A, row0, M, N, out, per, scratch); \
  } while (0)
  switch (epi) {
    case EPI_ADD: ROWS_LAUNCH(EPI_ADD); break;
    case EPI_SWIGLU: ROWS_LAUNCH(EPI_SWIGLU); break;
    case EPI_ROPE: ROWS_LAUNCH(EPI_ROPE); break;
    default: ROWS_LAUNCH(EPI_ARGMAX); break;
  }
#undef ROWS_LAUNCH
  if (ksr > 1) {
    const int nb = (epi == EPI_SWIGLU || epi == EPI_ROPE) ? 2 : 1;
    const int units = (ntiles / nb) * ceil_div(M, 16);
    dim3 rgrid(ceil_div(units, 4));
    switch (epi) {
      case EPI_ADD: hipLaunchKernelGGL((gemm_rows_reduce_kernel<EPI_ADD>), rgrid, rblk, 0, st, scratch, ksr, ntiles, TMT, row0, M, N, out); break;
      case EPI_SWIGLU: hipLaunchKernelGGL((gemm_rows_reduce_kernel<EPI_SWIGLU>), rgrid, rblk, 0, st, scratch, ksr, ntiles, TMT, row0, M, N, out); break;
      case EPI_ROPE: hipLaunchKernelGGL((gemm_rows_reduce_kernel<EPI_ROPE>), rgrid, rblk, 0, st, scratch, ksr, ntiles, TMT, row0, M, N, out); break;
      default: hipLaunchKernelGGL((gemm_rows_reduce_kernel<EPI_ARGMAX>), rgrid, rblk, 0, st, scratch, ksr, ntiles, TMT, row0, M, N, out); break;
    }
  }
}

// Narrow matrices (few workgroup columns) without K shares: four weight tiles per workgroup and the rows cut into
// blocks of TMT*16 (grid.z), so that columns x blocks fill the chip and no partial tiles go through memory.
// Only the epilogues of the narrow projections are instantiated (O, down, adapters: residual add; QKV: RoPE).
template <int TMT, int TN>
static bool launch_gemm_rows_blocks(hipStream_t st, int epi, const uint4* W, int ntiles, int ktiles, const uint4* A, int row0, int M,
                                    int N, const GemmOut& out) {
  if (epi != EPI_ADD && epi != EPI_ROPE) return false;
  dim3 grid(ceil_div(ntiles, 2 * TN), 1, ceil_div(M, TMT * 16)), blk(512);
  const bool full = M % (TMT * 16) == 0;
  LaunchEvents* ev = g_launch_events;
  g_launch_events = nullptr;
#define ROWS_LAUNCH(E_)                                                                                                          \
  do {                                                                                                                           \
    if (full) launch_timed(ev, gemm_rows_kernel<TMT, E_, true, TN>, grid, blk, st, W, ktiles, ntiles, A, row0, M, N, out, ktiles, (float*)nullptr); \
    else launch_timed(ev, gemm_rows_kernel<TMT, E_, false, TN>, grid, blk, st, W, ktiles, ntiles, A, row0, M, N, out, ktiles, (float*)nullptr);    \
  } while (0)
  if (epi == EPI_ADD) ROWS_LAUNCH(EPI_ADD);
  else ROWS_LAUNCH(EPI_ROPE);
#undef ROWS_LAUNCH
  return true;
}

// Wide matrices (gate/up, exit head) at 257..512 rows: sixteen weight tiles per workgroup and the rows in two blocks of
// up to 256.  Per k-tile a workgroup then moves 16 + 16 KiB through its address path for 256 MFMAs where the
// one-block form (8 weight tiles x 32 row tiles) moves 8 + 32 KiB for the same 256: a fifth less request time per
// MFMA, which is what bounds these shapes.  The two blocks of a column group run side by side on one XCD (see the
// kernel), so the weights still cross HBM once.
template <int EPI>
static void launch_gemm_rows_wide(hipStream_t st, const uint4* W, int ntiles, int ktiles, const uint4* A, int row0, int M, int N,
                                  const GemmOut& out) {
  const int groups = ceil_div(ntiles, 16);
  dim3 grid(16 * ceil_div(groups, 8)), blk(512);
  LaunchEvents* ev = g_launch_events;
  g_launch_events = nullptr;
  if (M == 512) launch_timed(ev, gemm_rows_kernel<16, EPI, true, 8>, grid, blk, st, W, ktiles, ntiles, A, row0, M, N, out, ktiles, (float*)nullptr);
  else launch_timed(ev, gemm_rows_kernel<16, EPI, false, 8>, grid, blk, st, W, ktiles, ntiles, A, row0, M, N, out, ktiles, (float*)nullptr);
}
int g_rows_wide = 1;               // test and tuning hook: 0 keeps the one-block form for wide matrices

// Form of the launch above for a call of M rows: row tiles per block, plus 100 with eight weight tiles per workgroup
// (TN = 4) instead of four; 0: use the K-share kernel (wide matrices, and shapes where it measured faster).
LaunchEvents* g_launch_events = nullptr;
int g_rows_blocks_override = -1;   // test and tuning hook: >= 0 replaces the choice below
int g_attn_pages_override = 0;
static int rows_blocks_form(int ntiles, int ktiles, int M) {
  if (g_rows_blocks_override >= 0) return g_rows_blocks_override;
  // measured on the 8B shapes (N 4096 and 6144): the blocks win for K <= 4096 from about 200 rows when columns x
  // blocks fit one round of workgroups; with K 14336 the K shares win at every row count.  Among the forms that
  // fit, the one with the cheapest k-tile step per workgroup (request time + MFMA time, in clocks) is taken.
  if (rows_ksplit(ntiles, ktiles) == 1 || ktiles > 128 || M <= 192) return 0;
  static const int forms[5][3] = {{2, 4, 192}, {2, 8, 320}, {4, 4, 320}, {4, 8, 512}, {2, 16, 576}};   // TN, TMT, clocks
  for (const auto& f : forms)
    if (ceil_div(ntiles, 2 * f[0]) * ceil_div(M, 16 * f[1]) <= 256) return (f[0] == 4 ? 100 : 0) + f[1];
  return 0;
}

// more than 16 rows from row 0 of the operand; out.nin.ssq, if set, is first reduced to per-row factors (per block)
void bf16_gemm_rows(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N,
                    const GemmOut& out0, float* scratch, float* inv_rms) {
  const uint4* Wc = (const uint4*)W;
  const uint4* Ac = (const uint4*)A;
  // blocks of up to 512 rows, of equal size up to a row tile: calls beyond 512 rows stream the weights once per block
  const int blk = ceil_div(ceil_div(M, ceil_div(M, 512)), 16) * 16;
  if (M > blk) g_launch_events = nullptr;           // several launches: the caller's bracket times the call
  for (int m0 = 0; m0 < M; m0 += blk) {
    const int mc = min(blk, M - m0);
    GemmOut out = out0;
    if (out.nin.ssq) {
      hipLaunchKernelGGL(norm_factor_kernel, dim3(ceil_div(mc, 4)), dim3(256), 0, st, out.nin.ssq + m0, out.nin.n_part, out.nin.stride,
                         out.nin.inv_d, out.nin.eps, inv_rms, mc);
      out.nin.inv_rms = inv_rms;
    }
    if (g_rows_wide && mc > 256 && ntiles >= 1536 && (epi == EPI_SWIGLU || epi == EPI_ARGMAX)) {
      if (epi == EPI_SWIGLU) launch_gemm_rows_wide<EPI_SWIGLU>(st, Wc, ntiles, ktiles, Ac, m0, mc, N, out);
      else launch_gemm_rows_wide<EPI_ARGMAX>(st, Wc, ntiles, ktiles, Ac, m0, mc, N, out);
      continue;
    }
    const int bt = rows_blocks_form(ntiles, ktiles, mc);
    if (bt == 4 && launch_gemm_rows_blocks<4, 2>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out)) continue;
    if (bt == 8 && launch_gemm_rows_blocks<8, 2>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out)) continue;
    if (bt == 16 && launch_gemm_rows_blocks<16, 2>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out)) continue;
    if (bt == 104 && launch_gemm_rows_blocks<4, 4>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out)) continue;
    if (bt == 108 && launch_gemm_rows_blocks<8, 4>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out)) continue;
    if (mc <= 64) launch_gemm_rows<4>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, scratch);
    else if (mc <= 128) launch_gemm_rows<8>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, scratch);
    else if (mc <= 192) launch_gemm_rows<12>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, scratch);
    else if (mc <= 256) launch_gemm_rows<16>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, scratch);
    else if (mc <= 384) launch_gemm_rows<24>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, scratch);
    else launch_gemm_rows<32>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, scratch);
  }
}

template <int MT, int U>
static void launch_gemm_mt(hipStream_t st, int epi, const uint4* W, int ntiles, int ktiles, const uint4* A, int row0, int M, int N,
                           const GemmOut& out, int nw, int ksplit) {
  dim3 blk(64 * nw);
  const int tpw = nw / ksplit;
  const int ntasks = (epi == EPI_SWIGLU || epi == EPI_ROPE) ? ntiles / 2 : ntiles;
  dim3 grid(ceil_div(ntasks, tpw));
  LaunchEvents* ev = g_launch_events;
  g_launch_events = nullptr;                       // one launch per offer
#define SKINNY_LAUNCH(E_)                                                                                                        \
  do {                                                                                                                           \
    if (ev) {                                                                                                                    \
      hipExtLaunchKernelGGL((gemm_skinny_kernel<MT, E_, U>), grid, blk, 0, st, ev->start, ev->stop, 0, W, ktiles, ntasks, A, row0, M, N, \
                            out, ksplit);                                                                                        \
      ev->used = true;                                                                                                           \
    } else {                                                                                                                     \
      hipLaunchKernelGGL((gemm_skinny_kernel<MT, E_, U>), grid, blk, 0, st, W, ktiles, ntasks, A, row0, M, N, out, ksplit);      \
    }                                                                                                                            \
  } while (0)
  switch (epi) {
    case EPI_ADD: SKINNY_LAUNCH(EPI_ADD); break;
    case EPI_SWIGLU: SKINNY_LAUNCH(EPI_SWIGLU); break;
    case EPI_ROPE: SKINNY_LAUNCH(EPI_ROPE); break;
    default: SKINNY_LAUNCH(EPI_ARGMAX); break;
  }
#undef SKINNY_LAUNCH
}

// launch shape: nw waves per workgroup, ksplit of them per task, k-tiles per register set U (4 or 8; 4 at 17..32 rows)
void bf16_gemm_cfg(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N,
                   const GemmOut& out, int nw, int ksplit, int U) {
  const uint4* Wc = (const uint4*)W;
  const uint4* Ac = (const uint4*)A;
  // (the session sends calls of more than 32 rows to the row-tiled kernel; should one arrive here it goes in passes of 32)
  for (int m0 = 0; m0 < M; m0 += 32) {
    const int mc = min(32, M - m0);
    if (mc <= 16) {
      if (U >= 8) launch_gemm_mt<1, 8>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, nw, ksplit);
      else launch_gemm_mt<1, 4>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, nw, ksplit);
    } else {
      launch_gemm_mt<2, 4>(st, epi, Wc, ntiles, ktiles, Ac, m0, mc, N, out, nw, ksplit);
    }
  }
}

// Launch shape by task count (measured on MI355X at M <= 16): many tasks -> one wave streams a whole
// strip (no reduction, deepest pipeline); few tasks -> split K over the waves of a workgroup so that
// one to two thousand waves are in flight (the 70B projections with 320-512 tasks: two waves per task).  M may exceed 32: rows then go in passes of 32 (weights re-streamed).
void bf16_gemm(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N, const GemmOut& out) {
  const int ntasks = (epi == EPI_SWIGLU || epi == EPI_ROPE) ? ntiles / 2 : ntiles;
  // launch shape by task count, from sweeps over the 8B and 70B matrix shapes at 9 rows
  int ksplit = ntasks >= 768 ? 1 : (ntasks >= 320 ? 2 : (ntasks >= 200 ? 8 : 4));
  while (ksplit > 1 && ktiles / ksplit < 4) ksplit >>= 1;
  const int U = (ntasks >= 768 || ntasks < 200 || ktiles / ksplit >= 32) ? 8 : 4;
  const int nw = ksplit > 4 ? ksplit : 4;
  bf16_gemm_cfg(st, epi, W, ntiles, ktiles, A, M, N, out, nw, ksplit, U);
}

// one workgroup of 1024 threads per row; the row's partials lie side by side ([row][tile]), so a wave's load is one
// contiguous 256 bytes; eight independent partials per thread are requested at once
__global__ __launch_bounds__(1024) void bf16_argmax_reduce_kernel(const float* __restrict__ pmax, const int* __restrict__ pidx,
                                                                   int ntiles, int pstride, int* v) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const int m = blockIdx.x;
  float best = -INFINITY; int idx = 0x7fffffff;
  for (int t0 = threadIdx.x; t0 < ntiles; t0 += 8 * 1024) {
    float x[8]; int xi[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int t = min(t0 + j * 1024, ntiles - 1);
      x[j] = pmax[(size_t)m * pstride + t]; xi[j] = pidx[(size_t)m * pstride + t];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)      // a clamped duplicate carries the same (value, index): harmless
      if (x[j] > best || (x[j] == best && xi[j] < idx)) { best = x[j]; idx = xi[j]; }
  }
  // within the wave by shuffles, then the sixteen waves' results through LDS (one barrier)
  for (int sh = 32; sh > 0; sh >>= 1) {
    const float o = __shfl_xor(best, sh, 64); const int oi = __shfl_xor(idx, sh, 64);
    if (o > best || (o == best && oi < idx)) { best = o; idx = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
  __syncthreads();
  if (threadIdx.x < 64) {
    best = threadIdx.x < 16 ? bv[threadIdx.x] : -INFINITY; idx = threadIdx.x < 16 ? bi[threadIdx.x] : 0x7fffffff;
    for (int sh = 8; sh > 0; sh >>= 1) {
      const float o = __shfl_xor(best, sh, 64); const int oi = __shfl_xor(idx, sh, 64);
      if (o > best || (o == best && oi < idx)) { best = o; idx = oi; }
    }
    if (threadIdx.x == 0) v[m] = idx;
  }
}
void bf16_argmax_reduce(hipStream_t st, const float* pmax, const int* pidx, int ntiles, int pstride, int M, int* v) {
  hipLaunchKernelGGL(bf16_argmax_reduce_kernel, dim3(M), dim3(1024), 0, st, pmax, pidx, ntiles, pstride, v);
}

// ---------------------------------------------------------------------------------------------
// k-query causal-in-block GQA attention over the paged cache, split over the KV axis.
// A sequence's block of m rows times the `rep` query heads sharing one KV head forms nq = m*rep
// query rows, cut into 16-row q-tiles.  Workgroup = (KV split, KV head [x group of q-tiles],
// sequence), eight waves with fixed roles: six compute waves, each owning one q-tile, and two loader
// waves.  The split's pages stream HBM -> loader registers -> LDS: each loader fetches half of every
// page (1 KiB chunks) and keeps three pages in flight in its registers, which is what hides HBM latency;
// the compute waves read whole pages back from a three-slot LDS ring, so a page crosses HBM, L2 and the
// vector memory path once however many q-tiles consume it.  One barrier per page hands a slot over.  Per page (64 positions) and q-tile:
//   S^T[pos][q] = K[pos][:] . Q[q][:]        4 pos-tiles x D/32 MFMAs  (K page = A operand, Q^T = B)
//   online softmax per q column (= per lane%16; the 4 lane groups hold 16 positions each)
//   O^T[d][q] += V^T[d][pos] P^T[pos][q]     D/16 d-tiles x 2 MFMAs    (V page = A operand, P^T = B)
// The page's element order (common.h) makes the S^T accumulators, once exponentiated and packed to
// bf16, exactly the B operand of the second product: no shuffles beyond the row statistics.
// Row r of the block sits at position p0+r and may see cache positions 0..p0+r (its own block rows
// included, they were appended just before).  Dead cache entries (>= p0+m) are never trusted:
// scores are masked by select and V elements are zeroed, so NaN there cannot leak.
// With one split the normalised output goes straight to the O-projection operand; otherwise the
// partials (max, sum, unnormalised O) go to scratch and attn_merge_kernel combines them.
// ---------------------------------------------------------------------------------------------
// maximum over the four 16-lane rows of a wave, delivered to every lane: lane l ends up with
// max(x[l % 16 + 16 r], r = 0..3).  v_permlane16_swap exchanges the odd rows of its first operand with the
// even rows of its second, v_permlane32_swap the upper half of the first with the lower half of the second.
__device__ inline float colmax4(float x) {
  typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
  u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

#define EE_MAX_SPLITS 64
#define EE_ATTN_WAVES 8
#define EE_ATTN_COMPUTE 6   // compute waves = q-tiles per workgroup; the other waves load
#define EE_ATTN_AHEAD 3     // pages each loader wave keeps in flight

template <int D, int QPW>
__global__ __launch_bounds__(64 * EE_ATTN_WAVES) void attn_kernel(const uint4* __restrict__ Q, const bf16_t* __restrict__ kv,
                                                                  const int* seq_m, const int* seq_p0, const int* seq_qt0,
                                                                  const int* seq_row0, const int* block_table, int pos_add, int rep,
                                                                  int total_qt, int Hkv, int layer, int n_pages, int pps, int nsplit,
                                                                  int per, float* part_o, float* part_ml, bf16_t* __restrict__ out,
                                                                  int out_ktiles) {
  constexpr int DS = D / 32, DT = D / 16;
  constexpr int KCH = 4 * DS, CH = KCH + 2 * DT;       // 1 KiB chunks of a page: K first, then V
  constexpr int NL = EE_ATTN_WAVES - EE_ATTN_COMPUTE, PF = EE_ATTN_AHEAD;
  constexpr int CPL = CH / NL;                         // chunks each loader wave fetches per page
  static_assert(CH % NL == 0, "page chunks must divide among the loader waves");
  __shared__ u32x4 lds[3][CH * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, qc = lane & 15;
  const int b = blockIdx.z, kvh = blockIdx.y % Hkv, sp = blockIdx.x;
  const int pg0 = sp * per;                            // every split takes `per` pages: a short sequence has fewer splits
  const int* bt = block_table + b * pps;
  // every scalar the workgroup needs before its first KV fetch is requested ahead of the first branch,
  // so the prologue costs one memory round trip, not one per dependent step (indices clamped into the table)
  int m = seq_m[b], sp0 = seq_p0[b], sqt0 = seq_qt0[b];
  int bt0[EE_ATTN_AHEAD];
#pragma unroll
  for (int q = 0; q < EE_ATTN_AHEAD; ++q) bt0[q] = bt[min(pg0 + q, pps - 1)];
  static_assert(EE_ATTN_AHEAD == 3, "the statement below names the look-ahead entries one by one");
  // ties the values together ahead of the branches (not volatile and without a memory clobber, so later
  // table lookups stay scalar loads)
  asm("" : "+s"(m), "+s"(sp0), "+s"(sqt0), "+s"(bt0[0]), "+s"(bt0[1]), "+s"(bt0[2]));
  if (m == 0) return;                                  // whole workgroup
  const int nq = m * rep;
  const int qt0 = (blockIdx.y / Hkv) * (EE_ATTN_COMPUTE * QPW);
  if (qt0 * 16 >= nq) return;                          // whole workgroup
  const int p0 = sp0 + pos_add, kv_end = p0 + m;
  const int npages = (kv_end + EE_PAGE - 1) / EE_PAGE;
  const int pg1 = min(npages, pg0 + per);
  if (pg0 >= npages) return;                           // whole workgroup; the merge pass knows this sequence's split count

  const bool loader = wave >= EE_ATTN_COMPUTE;
  const int lw = wave - EE_ATTN_COMPUTE;
  int limit[QPW];
  bool has[QPW];
  u32x4 qf[QPW][DS];
  float mrun[QPW];
  f32x4 o[QPW][DT], lacc[QPW];   // lacc: running row sums (every element of a lane holds its column's sum)
#pragma unroll
  for (int i = 0; i < QPW; ++i) {
    const int qt = qt0 + wave * QPW + i;
    has[i] = !loader && qt * 16 < nq;
    const int qrow = qt * 16 + qc;
    limit[i] = (has[i] && qrow < nq) ? p0 + qrow / rep : -1;
    const int gqt = sqt0 + (has[i] ? qt : 0);
#pragma unroll
    for (int s = 0; s < DS; ++s) qf[i][s] = ((const u32x4*)Q)[(((size_t)kvh * total_qt + gqt) * DS + s) * 64 + lane];
    mrun[i] = -INFINITY; lacc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[i][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // loader side: st[q] holds this wave's chunks (lw, lw + NL, ...) of the page q pages ahead (mod PF)
  u32x4 st[PF][CPL];
#define ATTN_FETCH(q_, page_)                                                                                \
  do {                                                                                                       \
    const u32x4* src_ = (const u32x4*)(kv + kv_slab(layer, page_, kvh, n_pages, Hkv, D)) + lw * 64 + lane;   \
    _Pragma("unroll") for (int j = 0; j < CPL; ++j) st[q_][j] = __builtin_nontemporal_load(src_ + j * NL * 64); \
  } while (0)
#define ATTN_DEPOSIT(buf_, q_)                                                                               \
  do {                                                                                                       \
    u32x4* dst_ = lds[buf_] + lw * 64 + lane;                                                                \
    _Pragma("unroll") for (int j = 0; j < CPL; ++j) dst_[j * NL * 64] = st[q_][j];                           \
  } while (0)
  // Scores are kept in base-2 units (s * log2(e)/sqrt(D)) so that the exponential is a bare v_exp_f32;
  // the row sums of the bf16-rounded weights come from one more MFMA column block (an all-ones A
  // operand), not from the vector ALU.  One step handles the scores and softmax of page pg and the
  // P.V product of page pg-1, whose weights the previous step left in registers: the two are
  // independent, so the second's MFMAs run under the first's vector arithmetic.  TAIL steps (a page
  // reaching into the block or past the end) mask scores and zero dead V.
  const float sc2 = 1.4426950408889634f / sqrtf((float)D);
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  u32x4 Pp0 = {0u, 0u, 0u, 0u}, Pp1 = {0u, 0u, 0u, 0u};   // weights of the previous page (B operand of P.V)
  // LDS fragment reads are issued as whole groups ahead of the MFMAs that consume them, and scheduling
  // barriers keep the compiler from sinking them back next to their uses (which would expose the LDS
  // latency once per fragment).
  auto pv_mfma = [&](auto tail_c, const u32x4 (&vf)[2 * DT], int ppg) __attribute__((always_inline)) {
    constexpr bool TAIL = decltype(tail_c)::value;
    const int pbase = ppg * EE_PAGE + 16 * g;
    lacc[0] = mfma16(ones, Pp0, lacc[0]);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {     // the two MFMAs of a d-tile depend on each other: keep them 8 apart
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        u32x4 v = vf[dt * 2 + ks];
        if (TAIL) {   // zero V at dead positions: element j of the fragment is position pbase + 8*ks + j
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int pa = pbase + 8 * ks + 2 * j;
            v[j] &= pa + 1 < kv_end ? 0xffffffffu : (pa < kv_end ? 0xffffu : 0u);
          }
        }
        o[0][dt] = mfma16(v, ks == 0 ? Pp0 : Pp1, o[0][dt]);
      }
    }
    lacc[0] = mfma16(ones, Pp1, lacc[0]);
  };
  auto step = [&](auto tail_c, auto prev_c, int slot, int pslot, int pg) __attribute__((always_inline)) {
    constexpr bool TAIL = decltype(tail_c)::value, PREV = decltype(prev_c)::value;
    const u32x4* L = &lds[0][0] + slot * (CH * 64) + lane;     // the slot is a run-time value: one loop body serves the whole ring
    const u32x4* Lp = &lds[0][0] + pslot * (CH * 64) + lane;
    const int base = pg * EE_PAGE + 16 * g;          // this lane group holds positions base .. base+15
    u32x4 kf[4 * DS];
#pragma unroll
    for (int c = 0; c < 4 * DS; ++c) kf[c] = L[c * 64];
    __builtin_amdgcn_sched_barrier(0);
    f32x4 s4[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) s4[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < DS; ++s)
#pragma unroll
      for (int t = 0; t < 4; ++t) s4[t] = mfma16(kf[t * DS + s], qf[0][s], s4[t]);
    u32x4 vf[2 * DT];
    if (PREV) {
#pragma unroll
      for (int c = 0; c < 2 * DT; ++c) vf[c] = Lp[(KCH + c) * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
    if (PREV) pv_mfma(tail_c, vf, pg - 1);
    // raw scores; the maximum is taken before scaling (the scale is positive) and the scale is folded
    // into the exponent's argument as one fused multiply-add
    float tmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        if (TAIL && base + 4 * t + v > limit[0]) s4[t][v] = -INFINITY;
        tmax = fmaxf(tmax, s4[t][v]);
      }
    tmax *= sc2;
    // running maximum of the column, shared by the four lane groups that hold its positions (two
    // register swaps across lane rows, no LDS traffic).  Everything up to the packed weights is
    // straight-line code, so the exponentials can be scheduled under the MFMAs; only the rescaling of
    // the accumulators, which is rare once the maximum has settled, sits behind a branch at the end.
    tmax = colmax4(tmax);
    const float mnew = fmaxf(mrun[0], tmax);
    const float msafe = mnew == -INFINITY ? 0.f : mnew;
    const float alpha = __builtin_amdgcn_exp2f(mrun[0] - msafe);
    mrun[0] = mnew;
    const float nm = -msafe;
    uint32_t pk[8];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      pk[2 * t] = pack2(__builtin_amdgcn_exp2f(fmaf(s4[t][0], sc2, nm)), __builtin_amdgcn_exp2f(fmaf(s4[t][1], sc2, nm)));
      pk[2 * t + 1] = pack2(__builtin_amdgcn_exp2f(fmaf(s4[t][2], sc2, nm)), __builtin_amdgcn_exp2f(fmaf(s4[t][3], sc2, nm)));
    }
    // (the empty statement pins the weights ahead of the branch: otherwise the exponentials are sunk
    // below it, out of the block that holds the MFMAs)
    asm volatile("" : "+v"(pk[0]), "+v"(pk[1]), "+v"(pk[2]), "+v"(pk[3]), "+v"(pk[4]), "+v"(pk[5]), "+v"(pk[6]), "+v"(pk[7]));
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) { o[0][dt][0] *= alpha; o[0][dt][1] *= alpha; o[0][dt][2] *= alpha; o[0][dt][3] *= alpha; }
      lacc[0][0] *= alpha; lacc[0][1] *= alpha; lacc[0][2] *= alpha; lacc[0][3] *= alpha;
    }
    Pp0 = u32x4{pk[0], pk[1], pk[2], pk[3]};   // positions base+0..7  (pos-tiles 0, 1)
    Pp1 = u32x4{pk[4], pk[5], pk[6], pk[7]};   // positions base+8..15 (pos-tiles 2, 3)
  };
  auto pv_last = [&](auto tail_c, int pslot, int ppg) __attribute__((always_inline)) {
    const u32x4* Lp = &lds[0][0] + pslot * (CH * 64) + lane;
    u32x4 vf[2 * DT];
#pragma unroll
    for (int c = 0; c < 2 * DT; ++c) vf[c] = Lp[(KCH + c) * 64];
    pv_mfma(tail_c, vf, ppg);
  };
  // software pipeline over a ring of three LDS slots (slot = page offset mod 3): while the compute waves
  // work on page p (scores) and p-1 (P.V), the loaders drop page p+1 into the third slot and request
  // page p+1+PF; every wave passes one barrier per page
  // (the two roles run separate loops with the same number of barriers, so neither carries the other's
  // registers)
  if (loader) {
    // Loads return in order and the compiler places the waits from what it can prove about the order of
    // issue, so the long-split path is kept free of branches from the first fetch to the end of its
    // steady-state loop: one conditional fetch on the way in would make every deposit of the loop wait
    // for all outstanding loads.
    int pg = pg0;
    if (pg0 + 2 * PF < pg1) {
#pragma unroll
      for (int q = 0; q < PF; ++q) ATTN_FETCH(q, bt0[q]);
      ATTN_DEPOSIT(0, 0);
      ATTN_FETCH(0, bt[pg0 + PF]);
      __syncthreads();
      for (; pg + 2 * PF < pg1; pg += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
          ATTN_DEPOSIT((u + 1) % 3, (u + 1) % PF);
          ATTN_FETCH((u + 1) % PF, bt[pg + u + 1 + PF]);
          __syncthreads();
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < PF; ++q)
        if (pg0 + q < pg1) ATTN_FETCH(q, bt0[q]);
      if (pg0 < pg1) ATTN_DEPOSIT(0, 0);
      if (pg0 + PF < pg1) ATTN_FETCH(0, bt[pg0 + PF]);
      __syncthreads();
    }
    for (; pg < pg1; pg += PF) {     // guarded tail (and short splits): one barrier per remaining page
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        const int p = pg + u;
        if (p >= pg1) break;
        if (p + 1 < pg1) ATTN_DEPOSIT((u + 1) % 3, (u + 1) % PF);
        if (p + 1 + PF < pg1) ATTN_FETCH((u + 1) % PF, bt[p + 1 + PF]);
        __syncthreads();
      }
    }
    return;
  }
#undef ATTN_FETCH
#undef ATTN_DEPOSIT
  static_assert(PF == 3 && QPW == 1, "three ring slots, one q-tile per compute wave");
  // Compute side: 1 + (pg1 - pg0) barriers like the loaders.  The page loop is cut into three plain loops
  // (first page, pages wholly before the block, pages reaching into it) whose bodies are one step
  // variant each, so the accumulators stay in place: no variant merges inside the steady-state loop.
  __syncthreads();
  if (!has[0]) {
    for (int pg = pg0; pg < pg1; ++pg) __syncthreads();
    return;
  }
  {
    const int first_tail = p0 / EE_PAGE;       // pages from here on reach into the block or past the end
    int pg = pg0, slot = 0, pslot = 2;
    if (pg >= first_tail) step(std::true_type{}, std::false_type{}, slot, pslot, pg);
    else step(std::false_type{}, std::false_type{}, slot, pslot, pg);
    __syncthreads();
    pslot = 0; slot = 1; ++pg;
    const int pe = min(pg1, first_tail);
    for (; pg < pe; ++pg) {
      step(std::false_type{}, std::true_type{}, slot, pslot, pg);
      __syncthreads();
      pslot = slot; slot = slot == 2 ? 0 : slot + 1;
    }
    for (; pg < pg1; ++pg) {
      step(std::true_type{}, std::true_type{}, slot, pslot, pg);
      __syncthreads();
      pslot = slot; slot = slot == 2 ? 0 : slot + 1;
    }
    // P.V of the split's last page (its slot is not written again)
    if (pg1 > first_tail) pv_last(std::true_type{}, pslot, pg1 - 1);
    else pv_last(std::false_type{}, pslot, pg1 - 1);
  }

#pragma unroll
  for (int i = 0; i < QPW; ++i) {
    if (!has[i]) continue;
    const int qt = qt0 + wave * QPW + i, gqt = sqt0 + qt, qrow = qt * 16 + qc;
    const float l = lacc[i][0];
    if (nsplit == 1) {
      if (qrow < nq) {
        const float inv = 1.0f / l;
        const int row = seq_row0[b] + qrow / rep, col0 = (kvh * rep + qrow % rep) * D + 4 * g;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          *(uint2*)(out + frag_offset(row, col0 + dt * 16, out_ktiles)) =
              make_uint2(pack2(o[i][dt][0] * inv, o[i][dt][1] * inv), pack2(o[i][dt][2] * inv, o[i][dt][3] * inv));
      }
    } else {
      // partial O of a split: [d-tile][lane] float4, the accumulator registers as they are
      const size_t slot = ((size_t)gqt * Hkv + kvh) * nsplit + sp;
      if (g == 0) *(float2*)(part_ml + slot * 32 + qc * 2) = make_float2(mrun[i], l);
      float4* po = (float4*)part_o + slot * (DT * 64) + lane;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) po[dt * 64] = make_float4(o[i][dt][0], o[i][dt][1], o[i][dt][2], o[i][dt][3]);
    }
  }
}

// merge the KV splits of one (q-tile, KV head) and emit the bf16 attention output in fragment layout
// (O-projection operand).  Workgroup = (q-tile, KV head, pair of d-tiles); its four waves share out the
// splits (wave w takes w, w+4, ...), each folding its share with all loads of a batch of eight splits in
// flight at once, and the four wave results meet in LDS.  Every lane owns the accumulator elements the
// split kernel's lanes did, so partials are read as coalesced float4.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                         const int* qt_seq, const int* qt_local, const int* seq_m,
                                                         const int* seq_p0, const int* seq_row0, int pos_add, int rep, int Hkv,
                                                         int slot_stride, int per, bf16_t* __restrict__ out, int out_ktiles) {
  constexpr int DT = D / 16, DW = 2;         // d-tiles per workgroup; gridDim.z = DT / DW
  __shared__ float sm[4][64], sd[4][64];
  __shared__ f32x4 sacc[4][DW][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, qc = lane & 15;
  const int gqt = blockIdx.x, kvh = blockIdx.y, dq = blockIdx.z;
  const int b = qt_seq[gqt], qt = qt_local[gqt];
  const int nq = seq_m[b] * rep, qrow = qt * 16 + qc;
  const int npages = (seq_p0[b] + pos_add + seq_m[b] + EE_PAGE - 1) / EE_PAGE;
  const int nsplit = (npages + per - 1) / per;          // this sequence's split count
  const size_t slot0 = ((size_t)gqt * Hkv + kvh) * slot_stride;
  const float2* ml = (const float2*)(part_ml + slot0 * 32) + qc;
  const f32x4* pi = (const f32x4*)part_o + slot0 * (DT * 64) + (size_t)dq * DW * 64 + lane;
  float mw = -INFINITY, den = 0.f;
  f32x4 acc[DW];
#pragma unroll
  for (int j = 0; j < DW; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = wave; s0 < nsplit; s0 += 32) {
    float2 t[8];
    f32x4 ov[8][DW];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int sl = min(s0 + 4 * i, nsplit - 1);
      t[i] = ml[sl * 16];
#pragma unroll
      for (int j = 0; j < DW; ++j) ov[i][j] = __builtin_nontemporal_load(pi + ((size_t)sl * DT + j) * 64);
    }
    float bm = mw;
#pragma unroll
    for (int i = 0; i < 8; ++i) bm = fmaxf(bm, s0 + 4 * i < nsplit ? t[i].x : -INFINITY);
    const float safe = bm == -INFINITY ? 0.f : bm;
    const float sc = __builtin_amdgcn_exp2f(mw - safe);
    den *= sc;
#pragma unroll
    for (int j = 0; j < DW; ++j) { acc[j][0] *= sc; acc[j][1] *= sc; acc[j][2] *= sc; acc[j][3] *= sc; }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float w = s0 + 4 * i < nsplit ? __builtin_amdgcn_exp2f(t[i].x - safe) : 0.f;
      den += w * t[i].y;
#pragma unroll
      for (int j = 0; j < DW; ++j) { acc[j][0] += w * ov[i][j][0]; acc[j][1] += w * ov[i][j][1]; acc[j][2] += w * ov[i][j][2]; acc[j][3] += w * ov[i][j][3]; }
    }
    mw = bm;
  }
  sm[wave][lane] = mw; sd[wave][lane] = den;
#pragma unroll
  for (int j = 0; j < DW; ++j) sacc[wave][j][lane] = acc[j];
  __syncthreads();
  if (wave != 0) return;
  float mall = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) mall = fmaxf(mall, sm[w][lane]);
  const float msafe = mall == -INFINITY ? 0.f : mall;
  den = 0.f;
#pragma unroll
  for (int j = 0; j < DW; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < 4; ++w) {        // fixed order: the result does not depend on timing
    const float f = __builtin_amdgcn_exp2f(sm[w][lane] - msafe);
    den += f * sd[w][lane];
#pragma unroll
    for (int j = 0; j < DW; ++j) {
      const f32x4 a = sacc[w][j][lane];
      acc[j][0] += f * a[0]; acc[j][1] += f * a[1]; acc[j][2] += f * a[2]; acc[j][3] += f * a[3];
    }
  }
  if (qrow < nq) {
    const float inv = 1.0f / den;
    const int row = seq_row0[b] + qrow / rep, col0 = (kvh * rep + qrow % rep) * D + dq * DW * 16 + 4 * g;
#pragma unroll
    for (int j = 0; j < DW; ++j)
      *(uint2*)(out + frag_offset(row, col0 + j * 16, out_ktiles)) =
          make_uint2(pack2(acc[j][0] * inv, acc[j][1] * inv), pack2(acc[j][2] * inv, acc[j][3] * inv));
  }
}

// Pages per KV split.  Every split of every sequence takes the same number of pages, so that a ragged
// batch is cut into workgroups of equal length; the count is the smallest one (>= 4, the software
// pipeline's depth) that keeps the launch within one workgroup per compute unit (the LDS ring admits
// one resident workgroup, so a second round would start cold).  kv_end[b] = 0: sequence not taking part.
int bf16_attention_pages_per_split(const int* kv_end, const int* seq_m, int B, int Hq, int Hkv, int max_splits) {
  const int rep = Hq / Hkv;
  int max_pages = 1;
  for (int b = 0; b < B; ++b) max_pages = max(max_pages, ceil_div(kv_end[b], EE_PAGE));
  int per = max(2, ceil_div(max_pages, max(1, min(max_splits, EE_MAX_SPLITS))));
  if (g_attn_pages_override > 0) return min(max(per, g_attn_pages_override), max_pages);   // (never more splits than the scratch holds)
  for (; per < max_pages; ++per) {
    long wgs = 0;
    for (int b = 0; b < B; ++b)
      if (kv_end[b] > 0)
        wgs += (long)ceil_div(ceil_div(kv_end[b], EE_PAGE), per) * Hkv * ceil_div(ceil_div(seq_m[b] * rep, 16), EE_ATTN_COMPUTE);
    if (wgs <= 256) break;
  }
  return min(per, max_pages);
}

template <int D, int QPW>
static void launch_attn(hipStream_t st, dim3 grid, const bf16_t* Q, const bf16_t* kv, const CallMeta& meta, int pos_add, int rep,
                        int total_qt, int Hkv, int layer, int n_pages, int pps, int nsplit, int per, const AttnScratch& scr,
                        bf16_t* out, int out_ktiles) {
  hipLaunchKernelGGL((attn_kernel<D, QPW>), grid, dim3(64 * EE_ATTN_WAVES), 0, st, (const uint4*)Q, kv, meta.seq_m, meta.seq_p0,
                     meta.seq_qt0, meta.seq_row0, meta.block_table, pos_add, rep, total_qt, Hkv, layer, n_pages, pps, nsplit, per,
                     scr.part_o, scr.part_ml, out, out_ktiles);
}

void bf16_attention(hipStream_t st, const bf16_t* Q, const bf16_t* kv, const CallMeta& meta, int pos_add, int B, int max_m,
                    int total_qt, int max_kv_end, int Hq, int Hkv, int D, int layer, int n_pages, int pages_per_seq,
                    const AttnScratch& scr, bf16_t* out, int out_ktiles, int per) {
  const int rep = Hq / Hkv;
  const int max_qt = ceil_div(max_m * rep, 16);
  const int qt_groups = ceil_div(max_qt, EE_ATTN_COMPUTE);
  const int max_pages = ceil_div(max_kv_end, EE_PAGE);
  per = max(1, min(per, max_pages));
  const int nsplit = ceil_div(max_pages, per);       // grid width and stride of the partial slots
  dim3 grid(nsplit, Hkv * qt_groups, B);
  if (D == 128) launch_attn<128, 1>(st, grid, Q, kv, meta, pos_add, rep, total_qt, Hkv, layer, n_pages, pages_per_seq, nsplit, per, scr, out, out_ktiles);
  else launch_attn<64, 1>(st, grid, Q, kv, meta, pos_add, rep, total_qt, Hkv, layer, n_pages, pages_per_seq, nsplit, per, scr, out, out_ktiles);
  if (nsplit > 1) {
    if (D == 128)
      hipLaunchKernelGGL((attn_merge_kernel<128>), dim3(total_qt, Hkv, 4), dim3(256), 0, st, scr.part_o, scr.part_ml, meta.qt_seq,
                         meta.qt_local, meta.seq_m, meta.seq_p0, meta.seq_row0, pos_add, rep, Hkv, nsplit, per, out, out_ktiles);
    else
      hipLaunchKernelGGL((attn_merge_kernel<64>), dim3(total_qt, Hkv, 2), dim3(256), 0, st, scr.part_o, scr.part_ml, meta.qt_seq,
                         meta.qt_local, meta.seq_m, meta.seq_p0, meta.seq_row0, pos_add, rep, Hkv, nsplit, per, out, out_ktiles);
  }
}
