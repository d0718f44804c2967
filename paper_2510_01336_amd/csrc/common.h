// Internal declarations shared by the HIP sources of libhispec (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include <string>
#include "../../include/hispec.h"

#define EE_PAGE 64          // positions per KV page
#define EE_MAX_WAVES 8      // waves per workgroup in the skinny GEMM

void ee_set_error(const char* fmt, ...);

#define HIP_TRY(x)                                                            \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      ee_set_error("%s failed: %s", #x, hipGetErrorString(e_));               \
      return EE_ERR_HIP;                                                      \
    }                                                                         \
  } while (0)

#define EE_TRY(x)                   \
  do {                              \
    int r_ = (x);                   \
    if (r_ != EE_OK) return r_;     \
  } while (0)

typedef uint16_t bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)b << 16;
  return c.f;
}
// round to nearest even; NaN stays NaN
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40);
  uint32_t bias = ((c.u >> 16) & 1u) + 0x7fffu;
  return (bf16_t)((c.u + bias) >> 16);
}

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------
// Fragment-tiled bf16 matrix: rows r (padded to 16) x cols k (padded to 32), stored as
// [r/16][k/32][64 lanes][8 elements] so that one wavefront reads one 16x32 MFMA operand
// (v_mfma_f32_16x16x32_bf16: lane l holds row l%16, k = 8*(l/16)..+7) as 1 KiB of contiguous
// memory, 16 B per lane.  Used for weights (row = output feature) and activations (row = token).
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline size_t frag_offset(int r, int k, int ktiles) {
  return ((size_t)(r >> 4) * ktiles + (k >> 5)) * 512 + (size_t)((((k & 31) >> 3) << 4) + (r & 15)) * 8 + (k & 7);
}

// ---------------------------------------------------------------------------------------------
// KV page (64 positions of one layer and one KV head), element order chosen so that the attention
// kernel's MFMA operands are contiguous 1 KiB reads:
//   K part: [t=4][s=D/32][lane][8]  with pos%64 -> t = (pos%16)/4, lane row r = 4*(pos/16) + pos%4,
//                                          d  -> s = d/32, lane group = (d%32)/8, element d%8
//   V part: [dt=D/16][ks=2][lane][8] with d -> dt = d/16, lane row r = d%16,
//                                          pos%64 -> lane group pos/16, ks = (pos%16)/8, element pos%8
// (K serves as the A operand of S^T = K Q^T; V as the A operand of O^T = V^T P^T.)
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline int k_page_off(int pos, int d, int D) {
  int t = (pos & 15) >> 2, r = ((pos >> 4) << 2) | (pos & 3);
  int s = d >> 5, g = (d & 31) >> 3, e = d & 7;
  return ((t * (D >> 5) + s) * 64 + g * 16 + r) * 8 + e;
}
__host__ __device__ inline int v_page_off(int pos, int d, int D) {
  int dt = d >> 4, r = d & 15;
  int g = pos >> 4, ks = (pos & 15) >> 3, j = pos & 7;
  return ((dt * 2 + ks) * 64 + g * 16 + r) * 8 + j;
}
// element offset of the (layer, page, kv head) slab inside the KV arena; K first, then V
__host__ __device__ inline size_t kv_slab(int layer, int page, int kvh, int n_pages, int n_kv, int D) {
  return (((size_t)layer * n_pages + page) * n_kv + kvh) * (size_t)(2 * EE_PAGE * D);
}

// ---------------------------------------------------------------------------------------------
// model
// ---------------------------------------------------------------------------------------------
struct MatLoc {          // one (possibly fused) weight matrix inside the model arena
  size_t off = 0;        // byte offset
  int N = 0, K = 0;      // logical rows (output features, fused/interleaved), cols
  int Np = 0, Kp = 0;    // padded to 16 / 32 (bf16 fragment layout); == N, K for fp32 row-major
  int ntiles() const { return Np / 16; }
  int ktiles() const { return Kp / 32; }
};

struct LayerLoc {
  size_t g1 = 0, g2 = 0;     // fp32 gains [d]
  MatLoc qkv, o, gu, down;   // gu: gate/up interleaved in 16-row tiles (gate tile j, up tile j, ...)
};

#define EE_MAX_GROUPS 7        // L_d, L_i, up to four further verifier exits, L_f: at most seven layer groups
struct ee_model {
  ee_config cfg;
  std::vector<int> exits;    // verifier exits in layers: L_d, L_i, the extra ones, L_f; group g = layers [exits[g-1], exits[g])
  char* base = nullptr;
  size_t bytes = 0;
  hipStream_t stream = nullptr;
  uint64_t seed = 0;
  bool bf16 = false;
  int Fp = 0;                // d_ffn padded to 16
  size_t emb = 0;            // [vocab][d] row-major, bf16 or fp32
  size_t gfinal = 0;         // fp32 [d]
  MatLoc head;
  size_t auxg[EE_MAX_GROUPS - 1] = {0, 0, 0, 0, 0, 0};   // auxiliary exit heads (cfg.head_rank > 0), per early exit: fp32 gain [d],
  MatLoc auxA[EE_MAX_GROUPS - 1], auxB[EE_MAX_GROUPS - 1];   // down projection [r, d] and up projection [d, r]
  std::vector<LayerLoc> L;
  double* inv_freq = nullptr;  // device [head_dim/2] rotary frequencies (inside the arena)
};

// where a logical tensor lives
struct TensorMap {
  int kind;        // 0 matrix, 1 fp32 vector (gain), 2 embedding (row-major)
  int rows, cols;
  size_t off;      // byte offset of matrix / vector / embedding
  int row_off;     // first physical row (fused QKV)
  int interleave;  // 0 none, 1 gate (tiles 2j), 2 up (tiles 2j+1), 3 rotary halves of a head (see phys_row)
  int Kp;          // padded K of the matrix
  int hd;          // head_dim (interleave 3 only)
};
int ee_tensor_map(const ee_model* m, int tensor_id, int layer, TensorMap* out);
int ee_layout_model(ee_model* m);   // fills offsets, returns total bytes in m->bytes

// physical row of logical row n.
// interleave 1/2: gate and up tiles alternate, so one GEMM task (two adjacent 16-row tiles) holds gate and
// up of the same 16 features.  interleave 3 (fused QKV of bf16 models): inside every head the 16-row tiles
// of the two rotary halves alternate -- tile 2j holds features 16j..16j+15, tile 2j+1 their partners
// D/2 + 16j.. -- so one GEMM task holds both elements of 16 rotary pairs.
__host__ __device__ inline int phys_row(int n, int row_off, int interleave, int hd) {
  if (interleave == 0) return row_off + n;
  if (interleave == 3) {
    const int r = row_off + n, h = r / hd, f = r % hd, half = hd >> 1;
    const int hi = f >= half ? 1 : 0, fj = (f - hi * half) >> 4;
    return h * hd + ((2 * fj + hi) << 4) + (f & 15);
  }
  return (((n >> 4) * 2 + (interleave - 1)) << 4) | (n & 15);
}

// ---------------------------------------------------------------------------------------------
// per-call metadata, built on the host and uploaded in one copy
// ---------------------------------------------------------------------------------------------
struct CallMeta {          // device pointers into the session's metadata block
  const int* row_seq;      // [M] sequence of row r
  const int* row_pos;      // [M] position of row r
  const int* row_tok;      // [M] input token of row r (embedding lookups)
  const int* row_src;      // [M] source row index for gathers
  const int* row_dst;      // [M] destination row index for scatters
  const int* seq_row0;     // [B] first packed row of sequence b
  const int* seq_m;        // [B] rows of sequence b in this call (0 = not taking part)
  const int* seq_p0;       // [B] position of its first row
  const int* seq_qt0;      // [B] first global q-tile of sequence b
  const int* qt_seq;       // [QT] sequence of global q-tile
  const int* qt_local;     // [QT] q-tile index inside its sequence
  const int* cand;         // [B][cand_stride] tokens to compare against the verifier's arg max
  const int* n_cand;       // [B]
  const int* block_table;  // [B][pages_per_seq]
};

// kernel-family ids for launch accounting
enum { KF_EMBED = 0, KF_NORM, KF_GEMM_QKV, KF_ROPE, KF_ATTN, KF_ATTN_COMBINE, KF_GEMM_O, KF_GEMM_GU,
       KF_GEMM_DOWN, KF_GEMM_HEAD, KF_ARGMAX, KF_ACCEPT, KF_COPY, KF_MISC, KF_COUNT };
