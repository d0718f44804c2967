/*
 * hispec.h -- C ABI of the MI355X (gfx950) implementation of HiSpec's k-token
 * verification path: hierarchical speculative decoding on an early-exit (EE)
 * transformer (paper: "HiSpec: Hierarchical Speculative Decoding for LLMs").
 *
 * One EE model with L_f layers is cut into three contiguous layer groups by its
 * draft exit L_d and its intermediate exit L_i (paper Sec. 3.1, "Early-Exit
 * Model"):  G1 = layers 1..L_d,  G2 = L_d+1..L_i,  G3 = L_i+1..L_f.
 * Every exit reads the hidden state through one shared final RMSNorm and one
 * shared LM head and takes the arg max (greedy rule of Sec. 3.1; ties go to the
 * lowest token id).
 *
 * Conventions
 *  - Every call returns EE_OK (0) or a negative EE_ERR_* code; ee_last_error()
 *    gives a message for the most recent failure on the calling thread.  A call
 *    that fails leaves the session as it was.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host
 *    memory.  The two arenas are allocated and owned by the caller and must stay
 *    alive until the matching *_free call; the library carves them up and never
 *    allocates device memory inside the draft / verify / rollback calls.
 *  - `stream` is a hipStream_t passed as void*; all device work of an object is
 *    enqueued on the stream given at creation.  Calls that return tokens or accept
 *    lengths synchronise that stream once before returning, so host outputs are
 *    valid on return.
 *  - Token ids, lengths and counts are int32.  Positions are 0-based.
 *  - Not thread safe per object; distinct sessions may be used from distinct threads.
 *
 * Per-sequence state (paper Algorithm 2 and Sec. 3.2).  C = committed tokens,
 * V = tokens tentatively accepted by L_i, T = C||V.  The last token of T is
 * "pending": it has no KV entry yet.  Between calls
 *      len(G1) = len(G2) = |T|-1,   len(G3) = |C|-1,
 * and the session buffers the L_i hidden rows of positions |C|-1 .. |T|-2 (H_i).
 * KV entries past a group's length are dead: pruning only lowers the length.
 */
#ifndef HISPEC_H
#define HISPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { EE_OK = 0, EE_ERR_ARG = -1, EE_ERR_STATE = -2, EE_ERR_CAPACITY = -3, EE_ERR_HIP = -4 };
enum { EE_F32 = 0, EE_BF16 = 1 };

/* tensor ids (also the stream ids of the synthetic weight generator) */
enum {
  EE_T_EMB = 0, EE_T_HEAD = 1, EE_T_GFINAL = 2, EE_T_G1 = 3, EE_T_WQ = 4, EE_T_WK = 5,
  EE_T_WV = 6, EE_T_WO = 7, EE_T_G2 = 8, EE_T_WGATE = 9, EE_T_WUP = 10, EE_T_WDOWN = 11,
  /* auxiliary low-rank exit heads (head_rank > 0): the `layer` argument is the exit, 0 = L_d, 1 = L_i, 2.. = extra exits */
  EE_T_AUX_G = 12,   /* gain of the adapter's RMSNorm        [d_model]            */
  EE_T_AUX_A = 13,   /* down projection                      [head_rank, d_model] */
  EE_T_AUX_B = 14    /* up projection (synthetic init: damped by gamma[exit])  [d_model, head_rank] */
};

typedef struct ee_config {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t exit_draft;   /* L_d, 1 <= L_d < L_i                        (Sec. 3.1) */
  int32_t exit_inter;   /* L_i, L_i < n_layers = L_f                             */
  float rope_theta;     /* rotary base; half-split pairing (i, i + head_dim/2)   */
  float rms_eps;
  int32_t dtype;        /* EE_F32: fp32 weights/activations/KV.  EE_BF16: bf16 weights,
                           bf16 matrix operands and KV, fp32 accumulation, fp32 residual */
  int32_t bonus_inter;  /* 1: verify k+1 rows at L_i so a fully matching block also yields
                           L_i's next token (LeadingSubstringVerify as printed); 0: k rows   */
  int32_t bonus_full;   /* 1: before the L_f pass run the pending token through G1+G2 so a
                           fully accepted V also yields L_f's next token; 0: |V| rows        */
  float sigma;          /* std of the synthetic weights (used by seeded init only)           */
  float gamma[3];       /* synthetic damping of the residual-writing matrices (Wo, Wdown) of
                           G1, G2, G3; 1 = plain random init                                 */
  int32_t head_rank;    /* 0: every exit uses the shared final norm + LM head (Sec. 3.1).  r > 0: every early
                           exit (L_d, L_i, the extra verifier exits) first passes the hidden state through its own rank-r adapter,
                           z = h + B (A RMSNorm(h; g)), and feed z to the shared norm and head -- the
                           low-rank prediction heads of the post-training conversion (App. I).  The final
                           exit is unchanged.  EE_BF16 models need a multiple of 32.                       */
  int32_t n_extra_exits;   /* 0..4 further intermediate verifiers L_{i,2} < L_{i,3} < ... between L_i and L_f
                              (the hierarchy of the paper's Future Work section); 0 = Alg. 2 as printed       */
  int32_t extra_exits[4];  /* their layers, strictly increasing, L_i < . < n_layers                          */
} ee_config;

typedef struct ee_model ee_model;
typedef struct ee_session ee_session;

/* ---- model ------------------------------------------------------------------------------- */

/* Bytes of device memory a model of this shape needs (weights in the library's own layout). */
size_t ee_model_bytes(const ee_config* cfg);

/* Build a model inside the caller's device arena (256-byte aligned, >= ee_model_bytes()).
 * Weights are filled ON DEVICE from `seed` with the counter-based generator documented in
 * ee_model_set_tensor's counterpart below (an EE checkpoint of the paper's kind would instead be
 * streamed in tensor by tensor with ee_model_set_tensor).  Synchronises `stream`.
 * Errors: EE_ERR_ARG (bad shape / null / misaligned), EE_ERR_CAPACITY (arena too small),
 * EE_ERR_HIP. */
int ee_model_load(const ee_config* cfg, void* dev_arena, size_t arena_bytes, uint64_t seed,
                  void* stream, ee_model** out);

/* Replace one tensor from host fp32 values in logical row-major [out_features, in_features]
 * layout (1-D for gains).  `layer` is 0-based and ignored for EMB/HEAD/GFINAL.  Values are
 * rounded to bf16 (nearest even) for EE_BF16 models.  Allocates a temporary staging buffer. */
int ee_model_set_tensor(ee_model* m, int tensor_id, int layer, const float* host_values);

/* Read rows [row0, row0+nrows) of a tensor back to host fp32 in logical layout (for gains:
 * elements).  Used to check the device generator against the host generator bit for bit. */
int ee_model_get_tensor_rows(ee_model* m, int tensor_id, int layer, int row0, int nrows,
                             float* host_out);

void ee_model_free(ee_model* m);   /* frees host bookkeeping only; the arena is the caller's */

/* ---- session ----------------------------------------------------------------------------- */

/* A session holds, for `batch` independent sequences: the paged KV cache shared by the three
 * layer groups (Sec. 3.2; pages of 64 positions, one block table per sequence, as in the
 * batched-inference section), the buffered exit hidden states H_d / H_i, the tentative buffer V
 * and the work buffers of one forward pass.
 *   max_ctx  : largest number of positions any one sequence may hold (incl. speculative rows)
 *   max_rows : largest number of rows one sequence contributes to one call, also the capacity
 *              of H_d / H_i / V per sequence (>= rounds_between_full_verifies*(k+1) + 1)
 *   total_pages : size of the shared page pool, 0 = batch * ceil(max_ctx/64)               */
size_t ee_session_bytes(const ee_model* m, int batch, int max_ctx, int max_rows, int total_pages);
int ee_session_create(ee_model* m, int batch, int max_ctx, int max_rows, int total_pages,
                      void* dev_arena, size_t arena_bytes, void* stream, ee_session** out);
void ee_session_free(ee_session* s);

/* Context build.  tokens: host, the prompts packed back to back; lens: host [batch], each >= 1.
 * Runs all L_f layers over every prompt in passes of up to 512 rows (64 for EE_F32 models): a long prompt fills
 * passes by itself, short prompts share one; leaves all group lengths at
 * lens[b], and commits first_token[b] = arg max at L_f of the last prompt position
 * (the "Vanilla generation" step of Sec. 3.1).  first_token: host [batch]. */
int ee_prefill(ee_session* s, const int32_t* tokens, const int32_t* lens, int32_t* first_token);

/* The same for one sequence while the others keep their state (a finished request leaves, a new one takes its
 * slot): the sequence's pages return to the shared pool, then its new prompt (host, len >= 1 tokens) is built.
 * EE_ERR_CAPACITY if the pool cannot hold it; the session is unchanged then. */
int ee_prefill_seq(ee_session* s, int seq, const int32_t* tokens, int len, int32_t* first_token);

/* A finished request leaves its slot: the sequence's KV pages return to the shared pool (Sec. 3.2: only the
 * block table changes) and its tokens, lengths and pending blocks are dropped.  The slot is idle until
 * ee_prefill / ee_prefill_seq starts it again: the batch-wide calls (ee_draft*, ee_verify_*, ee_decode_ar)
 * step the started sequences only and report -1 (tokens and accept counts) for an idle slot; they fail with
 * EE_ERR_STATE when no sequence is started.  EE_ERR_ARG for a bad index. */
int ee_seq_release(ee_session* s, int seq);

/* Pages of the shared KV pool that no sequence holds (64 positions of every layer each). */
int ee_free_pages(const ee_session* s);

/* Vanilla generation of Sec. 3.1 (the baseline the method is measured against and whose output it must
 * reproduce): n greedy single-token steps through all L_f layers per sequence, each committing
 * arg max at L_f.  Requires every started sequence to have an empty tentative buffer and no pending
 * draft block (EE_ERR_STATE otherwise); 1 <= n <= max_rows; EE_ERR_CAPACITY if positions would overflow.
 * All three group lengths advance by n.  out: host [batch, n], the committed tokens. */
int ee_decode_ar(ee_session* s, int n, int32_t* out);

/* Generate(L_d, x||V, k) of Algorithm 2: k sequential single-row passes through G1 + exit head +
 * arg max per sequence, each appending one KV row per G1 layer and one H_d row (Sec. 3.2,
 * "expanding during draft generation").  With bonus_inter one more G1-only row is run for the
 * last draft token.  draft: host [batch, k] out.  Errors: EE_ERR_STATE if a draft block is
 * already pending, EE_ERR_CAPACITY if positions or rows would overflow. */
int ee_draft(ee_session* s, int k, int32_t* draft);

/* Same state transition for an externally supplied draft block (host [batch, k]): G1 runs
 * block-parallel on the rows [pending token, S_1 .. S_k] (k+1 rows, k without bonus_inter). */
int ee_draft_inject(ee_session* s, int k, const int32_t* draft);

/* LeadingSubstringVerify(S, L_i, x||V) of Algorithm 2 for every sequence with a pending draft
 * block: the buffered H_d rows run through G2 block-causally against the shared KV cache, the
 * exit head + arg max gives v_1..v_rows, a = number of leading draft tokens equal to v.  Appends
 * [S_1..S_a, v_{a+1}] to V (only S when all k matched and no bonus row exists), keeps the L_i
 * hidden rows of the surviving positions in H_i, prunes G1/G2 KV to the surviving length, drops
 * H_d.  n_accept: host [batch] (0..k); next_token: host [batch] (v_{a+1}, or -1 if none). */
int ee_verify_intermediate(ee_session* s, int32_t* n_accept, int32_t* next_token);

/* For callers that cannot allocate device memory or hand over more of it -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: ee_verify_intermediate with every scratch buffer of the call (the
 * attention's KV-split partials, the exit head's per-tile (max, arg max) partials, the deferred-RMSNorm partial sums
 * and factors, the K-share partials of the row-tiled GEMM) taken from a static device array inside the library
 * instead of the session arena.  Arguments, results, state transition and errors as ee_verify_intermediate, and
 * bit-identical results (same kernels, same split plan).  The array holds 32 MiB per GPU from the first such call on
 * that GPU until the process ends; a call that needs more (about: more than 16 block rows in total on an 8B-sized
 * model, or a very long context) returns EE_ERR_CAPACITY before any device work and leaves the session unchanged.
 * The call allocates nothing (no hipMalloc / hipFree / event or stream creation; EE_ERR_STATE while kernel timing
 * is enabled, which creates events).  Every such call on a GPU uses that GPU's one array, which keeps the previous
 * call's contents (nothing in it needs clearing: each call writes what it reads), so calls on the same GPU that
 * overlap in time -- from two sessions or two streams -- race and must be serialised by the caller. */
int ee_verify_intermediate_static(ee_session* s, int32_t* n_accept, int32_t* next_token);

/* LeadingSubstringVerify(V, L_f, x) of Algorithm 2 for every sequence with active[b] != 0
 * (null = all) and a non-empty V: the buffered H_i rows (after the pending token's catch-up
 * through G1+G2 when bonus_full) run through G3, exit head + arg max, f = leading matches with V.
 * Commits [V_1..V_f, w_{f+1}] (only V when all matched and no bonus row), prunes all three
 * groups to |C|-1 and empties V and H_i (Sec. 3.2, last sentence).
 * n_accept, next_token, n_committed: host [batch]; committed: host [batch, max_rows+1], the newly
 * committed tokens of each sequence.  Inactive sequences report n_accept = -1, n_committed = 0. */
int ee_verify_full(ee_session* s, const uint8_t* active, int32_t* n_accept, int32_t* next_token,
                   int32_t* committed, int32_t* n_committed);

/* Several intermediate verifiers (the extension the paper's Future Work section sketches; models with
 * n_extra_exits > 0).  The verifier exits after L_d are levels 1..n = ee_n_levels(): level 1 is L_i
 * (ee_verify_intermediate), level n is L_f.  Level j in 2..n treats the tokens that exit j-1 accepted and that
 * still wait for exit j as its draft block, exactly as L_i treats S in Alg. 2: their buffered hidden rows of
 * exit j-1 (plus, in bonus_full mode, one row for the buffer's last token, run through the groups below first)
 * pass through the layers between the two exits, LeadingSubstringVerify against exit j's arg max keeps the
 * matching prefix and exit j's own next token, everything below is dropped and the KV lengths of the groups up
 * to j are pruned to what was kept (Sec. 3.2).  The kept tokens wait for exit j+1; at level n they are committed
 * and the call is ee_verify_full.  Every buffer below the one being checked must be empty (EE_ERR_STATE), so the
 * levels run bottom-up: 1, then 2 when enough tokens wait there, and so on.  Arguments as ee_verify_full
 * (`moved`: host [batch, max_rows+1], the kept tokens).  EE_ERR_ARG for a level outside 2..n; EE_ERR_CAPACITY when
 * the buffer of a level below L_f would exceed max_rows - bonus_full tokens (the next level's catch-up row shares its
 * max_rows slots); the session is unchanged then. */
int ee_verify_level(ee_session* s, int level, const uint8_t* active, int32_t* n_accept, int32_t* next_token,
                    int32_t* moved, int32_t* n_moved);

/* In-place KV length rollback of one sequence (Sec. 3.2 "pruning"): keep `new_len` positions.
 * group_mask bit0 = G1, bit1 = G2, bit2 = G3.  G1 and G2 move together: T is cut to new_len+1
 * tokens (the last becomes pending), V / H_i follow; if the cut reaches committed tokens V is
 * emptied and bit2 must be set (G3 is cut to new_len as well).  A pending draft block is dropped.
 * Only integers and the block-table tail change; no KV bytes move.  Shrink only:
 * EE_ERR_ARG if new_len exceeds the current length or the mask is inconsistent. */
int kv_rollback(ee_session* s, int seq, int group_mask, int new_len);

/* ---- rejection-sampling acceptance (App. G) --------------------------------------------------
 * The same three steps with the stochastic acceptance rule in place of arg max comparison: draft tokens
 * are drawn from p_{L_d}; a token S_j is accepted at a verifier with distribution p when
 * u < min(1, p(S_j) / q(S_j)), q being the distribution it was drawn from; at the first rejection the block
 * is cut and a replacement is drawn from max(0, p - q) normalised; after a fully accepted block the verifier's
 * extra row (if the block has one) supplies the next token, drawn from p.  The full verification applies the
 * rule again with V as the draft and its stored p_{L_i} rows as q.  All uniform numbers are inputs: host
 * arrays of floats in [0, 1) (EE_ERR_ARG otherwise).  Draws are by inverse CDF over the token ids in order.
 * The distributions are kept in a caller-owned device arena of ee_sampling_bytes() bytes (one store of batch *
 * max_rows * vocab floats per exit below L_f -- two for Alg. 2 -- and the uniform numbers), attached once per session;
 * 256-byte aligned.
 * The sampling calls and the arg max calls may not be mixed within one round (EE_ERR_STATE). */
size_t ee_sampling_bytes(const ee_session* s);
int ee_sampling_attach(ee_session* s, void* dev_arena, size_t arena_bytes);
/* u: host [batch, k], one number per drafted token.  Otherwise as ee_draft. */
int ee_draft_sample(ee_session* s, int k, const float* u, int32_t* draft);
/* u_acc: host [batch, u_stride], number j tests draft token j (u_stride >= k, EE_ERR_ARG otherwise); u_res: host
 * [batch], the replacement / next-token draw.  The entries of sequences that take no part are ignored.  Outputs
 * and state transition as ee_verify_intermediate. */
int ee_verify_intermediate_rs(ee_session* s, const float* u_acc, int u_stride, const float* u_res,
                              int32_t* n_accept, int32_t* next_token);
/* u_acc: host [batch, u_stride] (u_stride >= the longest tentative buffer taking part, EE_ERR_ARG otherwise).
 * Otherwise as ee_verify_full. */
int ee_verify_full_rs(ee_session* s, const uint8_t* active, const float* u_acc, int u_stride, const float* u_res,
                      int32_t* n_accept, int32_t* next_token, int32_t* committed, int32_t* n_committed);
/* The same rule at a further verifier exit (models with n_extra_exits > 0; level in 2..ee_n_levels(), the last being
 * ee_verify_full_rs): the tokens waiting below the level, distributed as the exit below it (their stored
 * distributions), are the draft, exit `level`'s distribution the target; what is kept follows exit `level`'s
 * distribution and waits for the next level with that law stored.  By the appendix's lemma applied level by level the
 * committed tokens follow p_{L_f}.  u_acc: host [batch, u_stride] (u_stride >= the longest buffer taking part), u_res:
 * host [batch].  EE_ERR_STATE if the waiting tokens were not produced by the sampling calls.  Otherwise as
 * ee_verify_level. */
int ee_verify_level_rs(ee_session* s, int level, const uint8_t* active, const float* u_acc, int u_stride, const float* u_res,
                       int32_t* n_accept, int32_t* next_token, int32_t* moved, int32_t* n_moved);
/* Test support: n rows from row0 of one sequence's stored distributions (which = 0: the draft distributions of
 * the pending block, 1: the L_i distributions of the tentative tokens), host out [n, vocab].  After a sampling
 * verify call ee_debug_last_logits returns that call's target distributions instead of logits. */
int ee_debug_read_dist(ee_session* s, int which, int seq, int row0, int n, float* host_out);

/* ---- introspection (parity tests; not part of the timed path) ---------------------------- */
int ee_get_lengths(const ee_session* s, int32_t* len_by_batch);   /* host [batch, ee_n_levels()+1]: KV length of every layer group (3 for Alg. 2) */
int ee_n_levels(const ee_session* s);   /* verifier exits after L_d: 2 (L_i, L_f) plus the model's extra exits */
int ee_get_counts(const ee_session* s, int32_t* n_committed, int32_t* n_tentative); /* [batch] each */
int ee_get_tokens(const ee_session* s, int seq, int32_t* out, int cap, int32_t* n_out); /* T = C||V */
/* When enabled, every exit-head call also stores full fp32 logits for its rows. */
int ee_debug_enable_logits(ee_session* s, int on);
int ee_debug_last_logits(ee_session* s, float* host_out, int max_rows, int32_t* n_rows);  /* [rows, vocab] */
int ee_debug_last_hidden(ee_session* s, float* host_out, int max_rows, int32_t* n_rows);  /* [rows, d]     */
/* K and V of `n` positions from pos0 of one layer, logical layout [n, n_kv_heads, head_dim]. */
int ee_debug_read_kv(ee_session* s, int seq, int layer, int pos0, int n, float* k_out, float* v_out);
/* The reverse, for tests that plant a KV context instead of building it (same layout, host in; values are
 * rounded to the cache's element type; the range must lie in pages the sequence owns). */
int ee_debug_write_kv(ee_session* s, int seq, int layer, int pos0, int n, const float* k_in, const float* v_in);
/* Overwrite every dead KV entry (position >= the group's length, in owned pages) of a sequence
 * with NaN: a test that pruned entries can never leak into a later result. */
int ee_debug_poison_dead_kv(ee_session* s, int seq);
/* Per-kernel launch accounting of the most recent draft/verify call: number of kernel launches
 * and, when enabled with ee_debug_time_kernels, HIP-event time (ms) per kernel family.        */
int ee_debug_time_kernels(ee_session* s, int on);
int ee_debug_kernel_times(ee_session* s, int32_t* n_families, const char** names /*[16]*/,
                          float* ms /*[16]*/, int32_t* launches /*[16]*/);

/* Test and tuning support, process-wide: the row-tiled GEMM (calls of more than 16 rows) serves the narrow
 * projections (O, down, QKV, adapters) either with K shares and a reduction pass or with blocks of row_tiles*16
 * rows and no K shares; row_tiles = 4, 8 or 16 forces the second form for every such call (104 and 108: blocks of 4
 * and 8 row tiles with eight instead of four weight tiles per workgroup), 0 the first, -1 restores the built-in
 * choice.  Two more values choose the form of the wide projections (gate/up, exit head) at 257..512 rows: 1016 (the
 * default) sixteen weight tiles per workgroup with the rows in two blocks, 1000 eight weight tiles and one block;
 * these two give bit-identical results.  Results of the forms of the narrow projections agree to rounding order.
 * EE_ERR_ARG for any other value. */
int ee_debug_gemm_row_blocks(int row_tiles);

/* Test support, process-wide: the attention kernel cuts every sequence's cached context into KV splits of equal
 * length, by default the shortest one that keeps the whole call within one workgroup per compute unit -- so the cut,
 * and with it the order in which a row's softmax partials are summed, follows the shape of the batch.  pages > 0
 * fixes the split length to that many 64-position pages for every call (raised where the split scratch would not
 * hold the count), so that a sequence is cut alike whether it runs alone or in a batch and the batched-inference
 * claim (a sequence's results do not depend on its neighbours) can be checked bit for bit; 0 restores the built-in
 * choice.  EE_ERR_ARG for a negative value. */
int ee_debug_attention_split_pages(int pages);

/* Plain device-to-device streaming copy on `stream` (pointers and size multiples of 16 bytes; not
 * synchronised).  A kernel of exactly known traffic -- `bytes` read, `bytes` written -- used to
 * calibrate hardware byte counters when the HBM traffic of the other kernels is measured. */
int ee_debug_stream_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

/* Plain streaming reads of known size, timed: buf_dev holds sum(sizes) bytes (16-byte aligned, sizes multiples of
 * 16, 1 <= n <= 16); per round the n regions are read back to back on `stream` by a kernel that only fetches them
 * (behind one untimed read), each launch timed by events attached to its dispatch; us_out[i] (host) = mean
 * microseconds of region i over `reps` rounds after two untimed ones.  Blocks until done.  This is the measured
 * floor for a weight-streaming projection of that size launched behind another kernel -- the rate a dependent launch
 * of tens of MB can reach on the chip, which is below the peak rate -- and is what the measurement script prints
 * beside each projection's own time.  EE_ERR_ARG for bad arguments, EE_ERR_HIP if a launch or an event fails. */
int ee_debug_read_floor(const void* buf_dev, const size_t* sizes, int n, int reps, float* us_out, void* stream);

const char* ee_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HISPEC_H */
