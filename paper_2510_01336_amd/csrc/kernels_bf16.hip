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
#include <cmath>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ inline f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ inline f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ inline uint32_t pack2(float lo, float hi) { return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16); }

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

// ---------------------------------------------------------------------------------------------
// Skinny GEMM  Y[m][n] = sum_k X[m][k] W[n][k],  M <= 16*MT rows, weights streamed once.
// A task is one 16-row weight tile strip over the whole K (two strips for SwiGLU: the gate tile and
// its up tile).  A workgroup of nw waves runs nw/ksplit tasks; the ksplit waves of a task split K
// into contiguous chunks, each wave streaming its chunk (1 KiB per MFMA step) through a two-stage
// register pipeline of depth U; the partial 16x16 tiles are then summed through LDS in a fixed
// order (deterministic) and the task's first wave runs the epilogue.
// The MFMA computes Y^T = W X^T so that a lane ends up with 4 consecutive n of one row m.
// ---------------------------------------------------------------------------------------------
template <int MT, int NB, int U>
struct Frags {
  u32x4 w[NB][U];
  u32x4 x[MT][U];
};

template <int MT, int NB, int U>
__device__ inline void load_frags(Frags<MT, NB, U>& f, const u32x4* const (&wp)[NB], const u32x4* ap, int ktiles, int kt, int kt1) {
  const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int u = 0; u < U; ++u) {
    bool ok = kt + u < kt1;
    int k = ok ? kt + u : kt1 - 1;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { u32x4 t = __builtin_nontemporal_load(&wp[nb][(size_t)k * 64]); f.w[nb][u] = ok ? t : z; }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) f.x[mt][u] = ap[((size_t)mt * ktiles + k) * 64];
  }
}

template <int MT, int EPI, int U>
__global__ __launch_bounds__(64 * EE_MAX_WAVES) void gemm_skinny_kernel(const uint4* __restrict__ W, int ktiles, int ntasks,
                                                                        const uint4* __restrict__ A, int M, int N, GemmOut out,
                                                                        int ksplit) {
  constexpr int NB = EPI == EPI_SWIGLU ? 2 : 1;
  __shared__ float4 red[EE_MAX_WAVES][NB * MT][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int task = blockIdx.x * (nw / ksplit) + wave / ksplit, kpart = wave % ksplit;
  const bool active = task < ntasks;
  const int per = (ktiles + ksplit - 1) / ksplit;
  const int kt0 = kpart * per, kt1 = min(ktiles, kt0 + per);

  f32x4 acc[NB][MT];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (active && kt0 < kt1) {
    const u32x4* wp[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wp[nb] = (const u32x4*)W + (size_t)(task * NB + nb) * ktiles * 64 + lane;
    const u32x4* ap = (const u32x4*)A + lane;
    Frags<MT, NB, U> cur, nxt;
    load_frags<MT, NB, U>(cur, wp, ap, ktiles, kt0, kt1);
    for (int kt = kt0; kt < kt1; kt += U) {
      const bool more = kt + U < kt1;
      if (more) load_frags<MT, NB, U>(nxt, wp, ap, ktiles, kt + U, kt1);
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = mfma16(cur.w[nb][u], cur.x[mt][u], acc[nb][mt]);
      if (more) cur = nxt;
    }
  }

  if (ksplit > 1) {   // fixed-order reduction over the K parts of a task (uniform branch: no wave left before it)
    if (kpart > 0) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          red[wave][nb * MT + mt][lane] = make_float4(acc[nb][mt][0], acc[nb][mt][1], acc[nb][mt][2], acc[nb][mt][3]);
    }
    __syncthreads();
    if (kpart == 0) {
      for (int w = 1; w < ksplit; ++w)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            float4 t = red[wave + w][nb * MT + mt][lane];
            acc[nb][mt][0] += t.x; acc[nb][mt][1] += t.y; acc[nb][mt][2] += t.z; acc[nb][mt][3] += t.w;
          }
    }
  }
  if (kpart != 0 || !active) return;

  const int g = lane >> 4, mc = lane & 15;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + mc;
    if (EPI == EPI_STORE || EPI == EPI_ADD) {
      const int n = task * 16 + 4 * g;
      if (m < M) {
        float4* p = (float4*)(out.Y + (size_t)m * out.ldy + n);
        float4 r = make_float4(acc[0][mt][0], acc[0][mt][1], acc[0][mt][2], acc[0][mt][3]);
        if (EPI == EPI_ADD) { float4 o = *p; r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w; }
        *p = r;
      }
    } else if (EPI == EPI_SWIGLU) {
      const int f = task * 16 + 4 * g;     // h[m][f..f+3] = silu(gate) * up
      if (m < M) {
        float h[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float gt = acc[0][mt][v], up = acc[NB - 1][mt][v];
          h[v] = gt / (1.0f + __expf(-gt)) * up;
        }
        uint2 pk = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
        *(uint2*)(out.H + frag_offset(m, f, out.h_ktiles)) = pk;
      }
    } else {   // EPI_ARGMAX: per-row (max, arg max) over this tile's 16 outputs; lowest index wins ties
      float best = -INFINITY; int bi = 0x7fffffff;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int n = task * 16 + 4 * g + v;
        float t = acc[0][mt][v];
        if (n < N) {
          if (out.Y && m < M) out.Y[(size_t)m * out.ldy + n] = t;
          if (t > best) { best = t; bi = n; }
        }
      }
#pragma unroll
      for (int sh = 16; sh <= 32; sh <<= 1) {
        float ob = __shfl_xor(best, sh, 64); int oi = __shfl_xor(bi, sh, 64);
        if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
      }
      if (g == 0 && m < M) {
        out.pmax[(size_t)task * out.pstride + m] = best;
        out.pidx[(size_t)task * out.pstride + m] = bi;
      }
    }
  }
}

template <int MT, int U>
static void launch_gemm_mt(hipStream_t st, int epi, const uint4* W, int ntiles, int ktiles, const uint4* A, int M, int N,
                           const GemmOut& out, int nw, int ksplit) {
  dim3 blk(64 * nw);
  const int tpw = nw / ksplit;
  const int ntasks = epi == EPI_SWIGLU ? ntiles / 2 : ntiles;
  dim3 grid(ceil_div(ntasks, tpw));
  switch (epi) {
    case EPI_STORE: hipLaunchKernelGGL((gemm_skinny_kernel<MT, EPI_STORE, U>), grid, blk, 0, st, W, ktiles, ntasks, A, M, N, out, ksplit); break;
    case EPI_ADD: hipLaunchKernelGGL((gemm_skinny_kernel<MT, EPI_ADD, U>), grid, blk, 0, st, W, ktiles, ntasks, A, M, N, out, ksplit); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((gemm_skinny_kernel<MT, EPI_SWIGLU, U>), grid, blk, 0, st, W, ktiles, ntasks, A, M, N, out, ksplit); break;
    default: hipLaunchKernelGGL((gemm_skinny_kernel<MT, EPI_ARGMAX, U>), grid, blk, 0, st, W, ktiles, ntasks, A, M, N, out, ksplit); break;
  }
}

// launch shape: nw waves per workgroup, ksplit of them per task, register pipeline depth U (2, 4 or 8)
void bf16_gemm_cfg(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N,
                   const GemmOut& out0, int nw, int ksplit, int U) {
  for (int m0 = 0; m0 < M; m0 += 64) {
    int mc = min(64, M - m0);
    GemmOut out = out0;
    if (out.Y) out.Y += (size_t)m0 * out.ldy;
    if (out.H) out.H += (size_t)(m0 / 16) * out.h_ktiles * 512;
    if (out.pmax) { out.pmax += m0; out.pidx += m0; }
    const uint4* Ac = (const uint4*)A + (size_t)(m0 / 16) * ktiles * 64;
    const uint4* Wc = (const uint4*)W;
    if (mc <= 16) {
      if (U >= 8) launch_gemm_mt<1, 8>(st, epi, Wc, ntiles, ktiles, Ac, mc, N, out, nw, ksplit);
      else if (U >= 4) launch_gemm_mt<1, 4>(st, epi, Wc, ntiles, ktiles, Ac, mc, N, out, nw, ksplit);
      else launch_gemm_mt<1, 2>(st, epi, Wc, ntiles, ktiles, Ac, mc, N, out, nw, ksplit);
    } else if (mc <= 32) {
      if (U >= 4) launch_gemm_mt<2, 4>(st, epi, Wc, ntiles, ktiles, Ac, mc, N, out, nw, ksplit);
      else launch_gemm_mt<2, 2>(st, epi, Wc, ntiles, ktiles, Ac, mc, N, out, nw, ksplit);
    } else {
      launch_gemm_mt<4, 2>(st, epi, Wc, ntiles, ktiles, Ac, mc, N, out, nw, ksplit);
    }
  }
}

// Launch shape by task count (measured on MI355X at M <= 16): many tasks -> one wave streams a whole
// strip (no reduction, deepest pipeline); few tasks -> split K over the waves of a workgroup so that
// about two thousand waves are in flight.  M may exceed 64: rows go in chunks of 64 (weights re-streamed).
void bf16_gemm(hipStream_t st, int epi, const bf16_t* W, int ntiles, int ktiles, const bf16_t* A, int M, int N, const GemmOut& out) {
  const int ntasks = epi == EPI_SWIGLU ? ntiles / 2 : ntiles;
  int ksplit = ntasks >= 768 ? 1 : (ntasks >= 320 ? 4 : 8);
  while (ksplit > 1 && ktiles / ksplit < 4) ksplit >>= 1;
  const int nw = ksplit > 4 ? ksplit : 4;
  bf16_gemm_cfg(st, epi, W, ntiles, ktiles, A, M, N, out, nw, ksplit, ksplit == 1 ? 8 : 4);
}

__global__ void bf16_argmax_reduce_kernel(const float* pmax, const int* pidx, int ntiles, int pstride, int* v) {
  __shared__ float bv[256];
  __shared__ int bi[256];
  int m = blockIdx.x;
  float best = -INFINITY; int idx = 0x7fffffff;
  for (int t = threadIdx.x; t < ntiles; t += blockDim.x) {
    float x = pmax[(size_t)t * pstride + m]; int xi = pidx[(size_t)t * pstride + m];
    if (x > best || (x == best && xi < idx)) { best = x; idx = xi; }
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
  if (threadIdx.x == 0) v[m] = bi[0];
}
void bf16_argmax_reduce(hipStream_t st, const float* pmax, const int* pidx, int ntiles, int pstride, int M, int* v) {
  hipLaunchKernelGGL(bf16_argmax_reduce_kernel, dim3(M), dim3(256), 0, st, pmax, pidx, ntiles, pstride, v);
}

// ---------------------------------------------------------------------------------------------
// RoPE + KV append.  Q goes to the attention kernel's B-operand layout
//   Q[kv head][global q-tile][s = D/32][lane][8],  lane = 16*((d%32)/8) + q%16, q = row_in_seq*rep + head_in_group
// K and V go to their cache page in fragment order (common.h).  Rotation in fp32, then bf16.
// ---------------------------------------------------------------------------------------------
__global__ void bf16_rope_append_kernel(const float* QKV, int ldq, const float2* cs, const int* row_seq, const int* row_pos,
                                        const int* seq_row0, const int* seq_qt0, const int* block_table, int pos_add, int M,
                                        int Hq, int Hkv, int D, int layer, int n_pages, int pps, int total_qt, bf16_t* Q,
                                        bf16_t* kv) {
  int half = D >> 1, heads = Hq + 2 * Hkv;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M * heads * half) return;
  int f = i % half, h = (i / half) % heads, r = i / (half * heads);
  const float* src = QKV + (size_t)r * ldq + (size_t)h * D;
  float a = src[f], b = src[f + half];
  float2 c = cs[r * half + f];
  int sq = row_seq[r];
  if (h < Hq) {
    int rep = Hq / Hkv, kvh = h / rep, hh = h % rep;
    int q = (r - seq_row0[sq]) * rep + hh;
    size_t tile = ((size_t)kvh * total_qt + seq_qt0[sq] + (q >> 4)) * (D >> 5);
    int d0 = f, d1 = f + half;
    Q[((tile + (d0 >> 5)) * 64 + ((d0 & 31) >> 3) * 16 + (q & 15)) * 8 + (d0 & 7)] = f32_to_bf16(a * c.x - b * c.y);
    Q[((tile + (d1 >> 5)) * 64 + ((d1 & 31) >> 3) * 16 + (q & 15)) * 8 + (d1 & 7)] = f32_to_bf16(b * c.x + a * c.y);
    return;
  }
  int pos = row_pos[r] + pos_add;
  int page = block_table[sq * pps + pos / EE_PAGE], pp = pos % EE_PAGE;
  if (h < Hq + Hkv) {
    size_t slab = kv_slab(layer, page, h - Hq, n_pages, Hkv, D);
    kv[slab + k_page_off(pp, f, D)] = f32_to_bf16(a * c.x - b * c.y);
    kv[slab + k_page_off(pp, f + half, D)] = f32_to_bf16(b * c.x + a * c.y);
  } else {
    size_t slab = kv_slab(layer, page, h - Hq - Hkv, n_pages, Hkv, D) + EE_PAGE * D;
    kv[slab + v_page_off(pp, f, D)] = f32_to_bf16(a);
    kv[slab + v_page_off(pp, f + half, D)] = f32_to_bf16(b);
  }
}
void bf16_rope_append(hipStream_t st, const float* QKV, int ldq, const float2* cs, const CallMeta& meta, int pos_add, int M,
                      int Hq, int Hkv, int D, int layer, int n_pages, int pages_per_seq, int total_qt, bf16_t* Q, bf16_t* kv) {
  int total = M * (Hq + 2 * Hkv) * (D / 2);
  hipLaunchKernelGGL(bf16_rope_append_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, QKV, ldq, cs, meta.row_seq,
                     meta.row_pos, meta.seq_row0, meta.seq_qt0, meta.block_table, pos_add, M, Hq, Hkv, D, layer, n_pages,
                     pages_per_seq, total_qt, Q, kv);
}

// ---------------------------------------------------------------------------------------------
// k-query causal-in-block GQA attention over the paged cache, split over the KV axis.
// A sequence's block of m rows times the `rep` query heads sharing one KV head forms nq = m*rep
// query rows, cut into 16-row q-tiles.  Workgroup = (KV split, KV head [x q-tile group], sequence);
// each wave owns one q-tile and walks the split's pages.  Per page (64 positions):
//   S^T[pos][q] = K[pos][:] . Q[q][:]        4 pos-tiles x D/32 MFMAs  (K page = A operand, Q^T = B)
//   online softmax per q column (= per lane%16; the 4 lane groups hold 16 positions each)
//   O^T[d][q] += V^T[d][pos] P^T[pos][q]     D/16 d-tiles x 2 MFMAs    (V page = A operand, P^T = B)
// The page's element order (common.h) makes the S^T accumulators, once exponentiated and packed to
// bf16, exactly the B operand of the second product: no LDS, no shuffles beyond the row statistics.
// Row r of the block sits at position p0+r and may see cache positions 0..p0+r (its own block rows
// included, they were appended just before).  Dead cache entries (>= p0+m) are never trusted:
// scores are masked by select and V elements are zeroed, so NaN there cannot leak.
// Partials (max, sum, unnormalised O) go to scratch; attn_combine merges the splits.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512) void attn_split_kernel(const uint4* __restrict__ Q, const bf16_t* __restrict__ kv,
                                                         const int* seq_m, const int* seq_p0, const int* seq_qt0,
                                                         const int* block_table, int pos_add, int rep, int total_qt, int Hkv,
                                                         int layer, int n_pages, int pps, int nsplit, float* part_o,
                                                         float* part_ml) {
  constexpr int DS = D / 32, DT = D / 16;
  const int lane = threadIdx.x & 63, g = lane >> 4, qc = lane & 15;
  const int b = blockIdx.z, kvh = blockIdx.y % Hkv, sp = blockIdx.x;
  const int qt = (blockIdx.y / Hkv) * 8 + (threadIdx.x >> 6);
  const int m = seq_m[b];
  if (m == 0) return;
  const int nq = m * rep;
  if (qt * 16 >= nq) return;
  const int p0 = seq_p0[b] + pos_add, kv_end = p0 + m;
  const int npages = (kv_end + EE_PAGE - 1) / EE_PAGE;
  const int per = (npages + nsplit - 1) / nsplit;
  const int pg0 = sp * per, pg1 = min(npages, pg0 + per);
  const int gqt = seq_qt0[b] + qt;
  const int qrow = qt * 16 + qc;
  const int limit = qrow < nq ? p0 + qrow / rep : -1;

  uint4 qf[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s) qf[s] = Q[(((size_t)kvh * total_qt + gqt) * DS + s) * 64 + lane];

  const float scale = 1.0f / sqrtf((float)D);
  float mrun = -INFINITY, lrun = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int pg = pg0; pg < pg1; ++pg) {
    const int page = block_table[b * pps + pg];
    const uint4* Kp = (const uint4*)(kv + kv_slab(layer, page, kvh, n_pages, Hkv, D)) + lane;
    const uint4* Vp = Kp + (EE_PAGE * D / 8);
    uint4 kf[4][DS];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int s = 0; s < DS; ++s) kf[t][s] = Kp[(t * DS + s) * 64];
    uint4 vf[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) { vf[dt][0] = Vp[(dt * 2) * 64]; vf[dt][1] = Vp[(dt * 2 + 1) * 64]; }

    f32x4 s4[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      s4[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < DS; ++s) s4[t] = mfma16(kf[t][s], qf[s], s4[t]);
    }
    const int base = pg * EE_PAGE + 16 * g;          // this lane group holds positions base .. base+15
    const bool tail = pg * EE_PAGE + EE_PAGE > p0;   // page reaches into the block (or past the end)
    float tmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float x = s4[t][v] * scale;
        if (tail && base + 4 * t + v > limit) x = -INFINITY;
        s4[t][v] = x;
        tmax = fmaxf(tmax, x);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float mnew = fmaxf(mrun, tmax);
    const float msafe = mnew == -INFINITY ? 0.f : mnew;
    const float alpha = __expf(mrun - msafe);
    float psum = 0.f;
    uint32_t pk[8];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float e0 = __expf(s4[t][0] - msafe), e1 = __expf(s4[t][1] - msafe);
      float e2 = __expf(s4[t][2] - msafe), e3 = __expf(s4[t][3] - msafe);
      bf16_t b0 = f32_to_bf16(e0), b1 = f32_to_bf16(e1), b2 = f32_to_bf16(e2), b3 = f32_to_bf16(e3);
      psum += (bf16_to_f32(b0) + bf16_to_f32(b1)) + (bf16_to_f32(b2) + bf16_to_f32(b3));
      pk[2 * t] = (uint32_t)b0 | ((uint32_t)b1 << 16);
      pk[2 * t + 1] = (uint32_t)b2 | ((uint32_t)b3 << 16);
    }
    lrun = lrun * alpha + psum;
    mrun = mnew;
    const uint4 P0 = make_uint4(pk[0], pk[1], pk[2], pk[3]);   // positions base+0..7  (pos-tiles 0, 1)
    const uint4 P1 = make_uint4(pk[4], pk[5], pk[6], pk[7]);   // positions base+8..15 (pos-tiles 2, 3)
    if (tail) {
      // zero V at dead positions: element j of vf[.][ks] is position base + 8*ks + j
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          uint32_t w[4] = {vf[dt][ks].x, vf[dt][ks].y, vf[dt][ks].z, vf[dt][ks].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            int pa = base + 8 * ks + 2 * j;
            if (pa >= kv_end) w[j] = 0;
            else if (pa + 1 >= kv_end) w[j] &= 0xffffu;
          }
          vf[dt][ks] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      f32x4 acc = o[dt];
      acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
      acc = mfma16(vf[dt][0], P0, acc);
      acc = mfma16(vf[dt][1], P1, acc);
      o[dt] = acc;
    }
  }

  lrun += __shfl_xor(lrun, 16, 64);
  lrun += __shfl_xor(lrun, 32, 64);
  const size_t slot = ((size_t)gqt * Hkv + kvh) * nsplit + sp;
  if (g == 0) { part_ml[slot * 32 + qc * 2] = mrun; part_ml[slot * 32 + qc * 2 + 1] = lrun; }
  float* po = part_o + (slot * 16 + qc) * D;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) *(float4*)(po + dt * 16 + 4 * g) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
}

// merge the KV splits and emit the bf16 attention output in fragment layout (O-projection operand):
// first the normalised weight of every (query row, split) pair goes to LDS, then each thread sums
// four output dims over the splits with coalesced float4 reads.
#define EE_MAX_SPLITS 64
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                           const int* qt_seq, const int* qt_local, const int* seq_m,
                                                           const int* seq_row0, int rep, int Hkv, int D, int nsplit,
                                                           bf16_t* out, int out_ktiles) {
  __shared__ float w[16][EE_MAX_SPLITS];
  const int gqt = blockIdx.x, kvh = blockIdx.y;
  const int b = qt_seq[gqt], qt = qt_local[gqt];
  const int nq = seq_m[b] * rep;
  const size_t slot0 = ((size_t)gqt * Hkv + kvh) * nsplit;
  {
    // 16 threads per query row: each takes splits s = t, t+16, ...
    const int qc = threadIdx.x >> 4, t = threadIdx.x & 15;
    float mloc = -INFINITY;
    for (int s = t; s < nsplit; s += 16) mloc = fmaxf(mloc, part_ml[(slot0 + s) * 32 + qc * 2]);
    for (int sh = 1; sh < 16; sh <<= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, sh, 64));
    float den = 0.f;
    for (int s = t; s < nsplit; s += 16) {
      float ms = part_ml[(slot0 + s) * 32 + qc * 2];
      float e = ms == -INFINITY ? 0.f : __expf(ms - mloc);
      w[qc][s] = e;
      den += e * part_ml[(slot0 + s) * 32 + qc * 2 + 1];
    }
    for (int sh = 1; sh < 16; sh <<= 1) den += __shfl_xor(den, sh, 64);
    const float inv = 1.0f / den;
    for (int s = t; s < nsplit; s += 16) w[qc][s] *= inv;
  }
  __syncthreads();
  const int d4n = D >> 2;
  for (int i = threadIdx.x; i < 16 * d4n; i += blockDim.x) {
    const int qc = i / d4n, d = (i % d4n) * 4;
    const int qrow = qt * 16 + qc;
    if (qrow >= nq) continue;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < nsplit; ++s) {
      const float ws = w[qc][s];
      const float4 o = *(const float4*)(part_o + ((slot0 + s) * 16 + qc) * D + d);
      acc.x += ws * o.x; acc.y += ws * o.y; acc.z += ws * o.z; acc.w += ws * o.w;
    }
    const int row = seq_row0[b] + qrow / rep, col = (kvh * rep + qrow % rep) * D + d;
    *(uint2*)(out + frag_offset(row, col, out_ktiles)) = make_uint2(pack2(acc.x, acc.y), pack2(acc.z, acc.w));
  }
}

void bf16_attention(hipStream_t st, const bf16_t* Q, const bf16_t* kv, const CallMeta& meta, int pos_add, int B, int max_m,
                    int total_qt, int max_kv_end, int Hq, int Hkv, int D, int layer, int n_pages, int pages_per_seq,
                    const AttnScratch& scr, bf16_t* out, int out_ktiles) {
  const int rep = Hq / Hkv;
  const int max_qt = ceil_div(max_m * rep, 16);
  const int qt_groups = ceil_div(max_qt, 8), waves = min(max_qt, 8);
  const int max_pages = ceil_div(max_kv_end, EE_PAGE);
  // enough (split, head, q-tile) waves to cover the chip, but at least two pages per wave when possible
  int nsplit = ceil_div(768, max(1, B * Hkv * max_qt));
  nsplit = max(1, min(nsplit, min(ceil_div(max_pages, 2), min(scr.max_splits, EE_MAX_SPLITS))));
  dim3 grid(nsplit, Hkv * qt_groups, B), blk(64 * waves);
  if (D == 128)
    hipLaunchKernelGGL((attn_split_kernel<128>), grid, blk, 0, st, (const uint4*)Q, kv, meta.seq_m, meta.seq_p0, meta.seq_qt0,
                       meta.block_table, pos_add, rep, total_qt, Hkv, layer, n_pages, pages_per_seq, nsplit, scr.part_o, scr.part_ml);
  else
    hipLaunchKernelGGL((attn_split_kernel<64>), grid, blk, 0, st, (const uint4*)Q, kv, meta.seq_m, meta.seq_p0, meta.seq_qt0,
                       meta.block_table, pos_add, rep, total_qt, Hkv, layer, n_pages, pages_per_seq, nsplit, scr.part_o, scr.part_ml);
  hipLaunchKernelGGL(attn_combine_kernel, dim3(total_qt, Hkv), dim3(256), 0, st, scr.part_o, scr.part_ml, meta.qt_seq,
                     meta.qt_local, meta.seq_m, meta.seq_row0, rep, Hkv, D, nsplit, out, out_ktiles);
}
