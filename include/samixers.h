/* samixers.h -- C ABI of the MI355X (gfx950) decode-step library for the four token mixers of
 * "Super Apriel: One Checkpoint, Many Speeds": Gated DeltaNet (GDN), Kimi Delta Attention (KDA),
 * full GQA attention (FA) and sliding-window GQA attention (SWA), plus the per-request placement
 * dispatcher over a stack of mixer layers.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a parameter says "host".  The caller owns every
 *     buffer; no hot call allocates or frees device memory.
 *   - `stream` is a hipStream_t (NULL = the null stream).  Calls only enqueue work on it and never
 *     synchronise; buffers must stay alive until that work has run.
 *   - bf16 tensors are passed as `const void*` (16-bit patterns, round-to-nearest-even of fp32).
 *   - Every entry returns a status.  Host-checkable violations (null or misaligned pointers, bad
 *     shapes, unsupported sizes) are reported BEFORE anything is enqueued and leave outputs
 *     untouched.  Values that live in device memory (seq_lens, page tables, index lists) are not
 *     validated.  sa_last_error() gives a message for the last failing call of the calling thread.
 *   - Pointers must be 16-byte aligned (4-byte for int32 lists and per-head gate scalars).
 */
#ifndef SAMIXERS_H
#define SAMIXERS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int sa_status;
enum {
  SA_OK = 0,
  SA_EINVAL = -1,       /* null/misaligned pointer, inconsistent shape, bad placement string */
  SA_EUNSUPPORTED = -2, /* a size outside what the kernels are built for                      */
  SA_EHIP = -3,         /* a HIP call or launch failed                                        */
  SA_EWORKSPACE = -4,   /* workspace too small                                                */
  SA_ENOMEM = -5        /* the page pool has too few free pages                               */
};

/* Message of the last failure on this thread; static storage, never freed by the caller. */
const char* sa_last_error(void);
int sa_version(void);

/* ---------------------------------------------------------------------------------------------
 * Recurrent mixers (Appendix B, "Gated DeltaNet (GDN)" and "Kimi Delta Attention (KDA)").
 *
 * For every processed batch row b, state head h and t = 0..T-1 in order, with S the dk x dv state:
 *     GDN:  Sbar = alpha[b,t,h] * S                 KDA:  Sbar[i,:] = alpha[b,t,h,i] * S[i,:]
 *     u = Sbar^T k;   S = Sbar + beta[b,t,h] * k (v - u)^T;   out[b,t,h,:] = scale * S^T q
 * which is the paper's S_t = alpha_t (I - beta_t k k^T) S_{t-1} + beta_t k v^T (GDN) and
 * S_t = (I - beta_t k k^T) diag(alpha_t) S_{t-1} + beta_t k v^T (KDA).  The read-out uses the state
 * after the write of step t (the paper prints no read-out; this is the reading taken).
 *
 *   q, k      bf16 [B,T,Hk,dk]   state head h reads q/k head h / (H/Hk); H % Hk == 0
 *   v         bf16 [B,T,H,dv]
 *   alpha     fp32 [B,T,H] (gdn) or [B,T,H,dk] (kda), each in (0,1]
 *   beta      fp32 [B,T,H]
 *   state_in  fp32 tiles, tile (slot,h) at ((slot*H)+h)*dk*dv, row-major [dk][dv]
 *   state_out same layout; may equal state_in (in place).  It receives the state after n_commit
 *             steps (0 <= n_commit <= T; n_commit = 0 copies the tile), so a verify pass over T
 *             drafted tokens can keep state_in intact and commit only the accepted prefix.
 *   out       fp32 [B,T,H,dv]
 *   slot_idx  int32 [B] or NULL: batch row -> state slot (NULL = identity)
 *   req_idx   int32 [n_req] or NULL: the batch rows to process (NULL = rows 0..B-1, n_req ignored);
 *             rows not listed are not touched.  A row must not be listed twice.
 * Supported: (dk,dv) in {(64,64),(128,128)}, 1 <= T <= 16.  B = 0 or n_req = 0 is a no-op.
 * At (128,128) calls of 7 (gdn) / 8 (kda) and more tokens are evaluated in the chunk-parallel form (see
 * gdn_chunk_steps): same arguments and results, outputs and states about 1e-5 instead of 1e-6 from the fp64 recurrence.
 */
sa_status gdn_decode_step(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                          const float* state_in, float* state_out, float* out,
                          const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                          int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, void* stream);
sa_status kda_decode_step(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                          const float* state_in, float* state_out, float* out,
                          const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                          int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, void* stream);
/* The same steps with the committed prefix chosen per request (Appendix "Speculative Decoding": every request of a
 * batch accepts its own number of drafted tokens): n_commit_rows is a device array int32 [B], indexed by batch row
 * like q; row b's state_out tile receives the state after n_commit_rows[b] steps, values outside [0,T] are clamped
 * to that range.  Everything else as above; SA_EINVAL if n_commit_rows is NULL or not 4-byte aligned. */
sa_status gdn_decode_step_var(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                              const float* state_in, float* state_out, float* out,
                              const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                              int B, int T, int H, int Hk, int dk, int dv, float scale,
                              const int32_t* n_commit_rows, void* stream);
sa_status kda_decode_step_var(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                              const float* state_in, float* state_out, float* out,
                              const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                              int B, int T, int H, int Hk, int dk, int dv, float scale,
                              const int32_t* n_commit_rows, void* stream);

/* State tiles.  A recurrent state is dk*dv fp32 values per (slot, head); callers that do not want to depend on the
 * order inside a tile convert with these (Appendix B: one dk x dv state matrix per head).  In this library a
 * tile is plain row-major [dk][dv] (key channel major), so both conversions are copies; they exist so that the order
 * can change without breaking callers.  rowmajor and tiles: device pointers, n_tiles * dk * dv floats each, 16-byte
 * aligned, not overlapping.  (dk,dv) as for the decode steps. */
size_t    sa_state_tile_bytes(int dk, int dv);   /* dk * dv * 4, or 0 for an unsupported shape */
sa_status sa_state_pack(const float* rowmajor, float* tiles, int n_tiles, int dk, int dv, void* stream);
sa_status sa_state_unpack(const float* tiles, float* rowmajor, int n_tiles, int dk, int dv, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Many tokens per state pass: the same recurrences and read-out as gdn_decode_step / kda_decode_step,
 * evaluated in their chunk-parallel form (Appendix B: GDN is evaluated chunk by chunk on a WY representation, KDA on
 * DPLR transitions; Section 6: such kernels serve prefill).  Tokens are processed 16 at a time as matrix
 * products on the matrix cores with the state held in registers across the whole call.  Results equal T
 * chained single steps up to rounding: every fp32 operand of a product enters as two bf16 terms (relative
 * error 2^-18), which leaves outputs and states about 1e-5 from the fp64 recurrence.  Arguments as for the
 * decode steps (n_commit included: all T outputs are produced, the state written is the one after n_commit
 * tokens); any T >= 1.  The decode steps themselves run on these kernels from 7 (GDN) or 8 (KDA) tokens per call at
 * (dk,dv) = (128,128), where they are as fast or faster (8 tokens: 51 / 61 us against 54 / 61 us at batch 64).  Gates below 2^-100 act as 2^-100 in kda_chunk_steps and below the smallest
 * normal fp32 number as that number in gdn_chunk_steps.  Supported: (dk,dv) = (128,128).
 */
sa_status gdn_chunk_steps(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                          const float* state_in, float* state_out, float* out,
                          const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                          int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, void* stream);
sa_status kda_chunk_steps(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                          const float* state_in, float* state_out, float* out,
                          const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                          int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Whole-block decode step of a recurrent mixer: the state update above with the block's own pre- and
 * post-processing fused around it in one launch (Appendix B: a short causal 1-D convolution with SiLU on
 * Q, K and V, L2-normalised q and k, beta = sigmoid(beta_raw), log-decay
 * g = -exp(A_log) * softplus(alpha_raw + dt_bias), gated RMS normalisation of the read-out with z; Section 6:
 * the decode step updates the recurrent state and the convolution histories in place).  One new token per row.
 *
 * Per processed row b (slot s = slot_idx ? slot_idx[b] : b), with C the channel count of a stream
 * (Hk*dk for q and k, H*dv for v) and Kc = conv_taps:
 *     y[c]   = SiLU( sum_{j<Kc-1} w[j][c] * conv_in[s][j][c] + w[Kc-1][c] * x[b][c] )
 *     conv_out[s] = (conv_in[s][1..Kc-2], x[b])                      (the Kc-1 most recent inputs, oldest first)
 *     q, k   = y / sqrt(sum_head(y^2) + 1e-6) per head;   v = y
 *     beta   = sigmoid(beta_raw[b,h]);   alpha = exp(-exp(A_log[h]) * softplus(alpha_raw + dt_bias))
 *              gdn: alpha_raw [B,H], dt_bias [H];   kda: alpha_raw [B,H,dk], dt_bias [H,dk] (one gate per key channel)
 *     (o, S) = the gdn / kda step above with these q, k, v, alpha, beta
 *     out[b,h,:] = norm_weight * o / sqrt(mean(o^2) + norm_eps) * act(z[b,h,:]),  act = SiLU (gate_act 0) or sigmoid (1)
 * The paper names these operations but prints no formula for the two normalisations, for KDA's gate or for the
 * output gate; the forms above are this library's reading.
 *
 *   xq, xk   bf16 [B,Hk,dk]     xv, z  bf16 [B,H,dv]       wq, wk fp32 [Kc][Hk*dk]    wv fp32 [Kc][H*dv]
 *   conv_*   bf16 [slots][Kc-1][C]; *_out may equal *_in when Hk == H (each channel then has one reader);
 *            with Hk < H the q and k buffers must be distinct from their inputs
 *   beta_raw, alpha_raw, A_log, dt_bias, norm_weight fp32;  state and out as for the plain step
 * Supported: (dk,dv) in {(64,64),(128,128)}, 2 <= conv_taps <= 4.
 */
typedef struct {
  const void *xq, *xk, *xv;
  const float *wq, *wk, *wv;
  const void *conv_q_in, *conv_k_in, *conv_v_in;
  void *conv_q_out, *conv_k_out, *conv_v_out;
  int conv_taps;
  const float *beta_raw, *alpha_raw, *A_log, *dt_bias;
  const void* z;
  const float* norm_weight;
  float norm_eps;
  int gate_act;
} sa_block_io;

sa_status gdn_block_decode(const sa_block_io* io, const float* state_in, float* state_out, float* out,
                           const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                           int B, int H, int Hk, int dk, int dv, float scale, void* stream);
sa_status kda_block_decode(const sa_block_io* io, const float* state_in, float* state_out, float* out,
                           const int32_t* slot_idx, const int32_t* req_idx, int n_req,
                           int B, int H, int Hk, int dk, int dv, float scale, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Paged KV cache (Section 6, "Heterogeneous state": KV caches grow with the sequence for FA and are
 * bounded at the window for SWA; the paper fixes no in-page order, the one below is this library's).
 *
 * Pages hold 16 tokens.  A pool is [n_pages][Hkv] blocks of 16*D bf16 (4 KiB at D = 128):
 *   K block  [D/8][16 tokens][8 dims]              element (token j, dim d) at ((d/8)*16 + j)*8 + d%8
 *   V block  [D/16][4 token groups][16 dims][4]    element (j, d) at (((d/16)*4 + j/4)*16 + d%16)*4 + j%4
 * page_table int32 [B,max_pages]: logical page -> physical page; entries for pages no live token
 * falls in may be -1 and are never read.
 *
 * n_pages is the pool size; a table entry outside [0,n_pages) that attn_decode does meet is clamped
 * into the pool (the result is then meaningless, but no access leaves the pool).  Slots of a page
 * that hold no live token may contain any bit pattern, NaN included.
 *
 * kv_append writes T new tokens per sequence: token i of row b goes to position positions[b] + i;
 * a token whose position is at or beyond max_pages*16, or whose page is unmapped, is skipped.
 *   k_new, v_new  bf16 [B,T,Hkv,D] (token-major, as a projection produces them)
 */
sa_status kv_append(const void* k_new, const void* v_new, void* kpool, void* vpool, int n_pages,
                    const int32_t* page_table, int max_pages, const int32_t* positions, int B, int T, int Hkv, int D,
                    int page_size, void* stream);

/* ---------------------------------------------------------------------------------------------
 * GQA decode attention (Appendix B, "Full Attention (FA)" and "Sliding Window Attention (SWA)").
 *
 * For every processed row b with L = seq_lens[b] (the count includes the T newest tokens, whose K/V
 * are already in the cache), new token i in [0,T) and query head h (KV head h / (Hq/Hkv)):
 *     hi = L - T + i + 1,  lo = window > 0 ? max(0, hi - window) : 0
 *     out[b,i,h,:] = sum_j softmax_j(scale * q[b,i,h,:] . K_j) V_j   over cached positions j in [lo,hi)
 * i.e. window <= 0 is full attention, window = w attends to the w most recent positions including
 * the token itself.  Rows with hi <= 0 give zeros.  seq_lens above max_seq_len are treated as
 * max_seq_len (max_seq_len is the host-side bound used to plan the split over pages).
 *
 *   q          bf16 [B,T,Hq,D]            out  fp32 [B,T,Hq,D]
 *   seq_lens   int32 [B]                  req_idx as for the recurrent mixers
 *   workspace  at least attn_decode_workspace_bytes(...) bytes (0 when the plan has a single page range per
 *              (request, KV head); workspace may then be NULL), 16-byte aligned; holds the per-split
 *              partial results (running maximum, normaliser, unnormalised output) that a second
 *              kernel merges in a fixed order, so results are run-to-run deterministic.
 * Supported: D = 128, page_size = 16, T * (Hq/Hkv) <= 32 (e.g. 8 new tokens at 4 query heads per KV head).
 */
size_t attn_decode_workspace_bytes(int n_req, int T, int Hq, int Hkv, int D, int max_seq_len, int window);
sa_status attn_decode(const void* q, const void* kpool, const void* vpool, int n_pages,
                      const int32_t* page_table, int max_pages, const int32_t* seq_lens, const int32_t* req_idx, int n_req, float* out,
                      int B, int T, int Hq, int Hkv, int D, int page_size, int max_seq_len, int window, float scale,
                      void* workspace, size_t workspace_bytes, void* stream);

/* attn_decode for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and results (bit for bit) as
 * attn_decode, without the workspace: the per-range partial results live in a fixed device array of
 * attn_decode_static_max_bytes() = 16 MiB that is part of the library's image (every GPU the library runs on holds
 * its copy until the process ends).  The call allocates and frees nothing.  SA_EWORKSPACE, with nothing enqueued, if
 * attn_decode_workspace_bytes() of the call exceeds that size (batch 64 at 32768 tokens needs 8.1 MiB).
 * All calls on one GPU share the array: it keeps the last call's partial results (every value a call reads it has
 * written itself first, so nothing needs clearing), and two calls that overlap in time on one GPU (different
 * streams) race; calls on one stream are ordered and safe. */
size_t attn_decode_static_max_bytes(void);
sa_status attn_decode_static(const void* q, const void* kpool, const void* vpool, int n_pages,
                             const int32_t* page_table, int max_pages, const int32_t* seq_lens, const int32_t* req_idx, int n_req,
                             float* out, int B, int T, int Hq, int Hkv, int D, int page_size, int max_seq_len, int window,
                             float scale, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Placement decode (Section 6, "Per-request placement switching": each request names a placement,
 * a placement names one mixer per layer, and the layer dispatches on it with no global state).
 *
 * A placement is a NUL-terminated string with one character per layer: F (full attention),
 * S (sliding window), K (KDA), G (GDN).  A plan groups the B requests of a batch per (layer, mixer)
 * and keeps the index lists in device memory; it is the only object the library allocates.
 */
typedef struct sa_plan sa_plan;

typedef struct {
  int H, Hk, dk, dv;             /* recurrent mixers                      */
  int Hq, Hkv, D, page_size;     /* attention mixers                      */
} sa_shapes;

typedef struct {                 /* one per layer; every pointer is a device pointer indexed by request */
  const void* q;                 /* recurrent: bf16 [B,T,Hk,dk]           */
  const void* k;                 /*            bf16 [B,T,Hk,dk]           */
  const void* v;                 /*            bf16 [B,T,H,dv]            */
  const float* alpha_scalar;     /* GDN gate   fp32 [B,T,H]               */
  const float* alpha_vec;        /* KDA gate   fp32 [B,T,H,dk]            */
  const float* beta;             /*            fp32 [B,T,H]               */
  float* state;                  /* recurrent tiles of this layer, updated in place */
  const int32_t* slot_idx;       /* request -> state slot, or NULL        */
  const void* q_attn;            /* attention: bf16 [B,T,Hq,D]            */
  const void* kpool;             /* this layer's K pool (new tokens already appended) */
  const void* vpool;
  int n_pages;                   /* pages in each pool                    */
  const int32_t* page_table;     /* int32 [B,max_pages]                   */
  const int32_t* seq_lens;       /* int32 [B]                             */
  int max_pages;
  int max_seq_len;
  float* out;                    /* fp32 [B,T,H,dv] == [B,T,Hq,D] (needs H*dv == Hq*D) */
  const int32_t* n_commit_rows;  /* recurrent: int32 [B], how many of the T steps each request's state keeps
                                    (as in gdn_decode_step_var), or NULL = all T: a verify pass runs with zeros
                                    and leaves the states alone, the pass after acceptance with the accepted counts */
} sa_layer_io;

/* placements: host array of n_placements strings, each of length L.  placement_id: host int32 [B],
 * values in [0,n_placements).  Errors: SA_EINVAL for a wrong length, an unknown character or an id
 * out of range. */
sa_status placement_plan_create(const char* const* placements, int n_placements, int L,
                                const int32_t* placement_id, int B, sa_plan** plan_out);
void placement_plan_destroy(sa_plan* plan);
/* Number of requests that run mixer `mixer` ('F','S','K','G') at layer `layer`; -1 on bad arguments. */
int placement_plan_count(const sa_plan* plan, int layer, char mixer);
/* Bytes of device workspace placement_decode needs for this plan (0 if no layer splits its contexts into page
 * ranges): twice the largest sum over a layer of its full-attention and its sliding-window partial results.  A
 * fused layer launch keeps the two side by side, and alternate layers use alternate halves of the workspace,
 * because a fused layer's partial results are merged by the launch of the layer after it. */
size_t placement_workspace_bytes(const sa_plan* plan, const sa_shapes* shapes, int T, int max_seq_len, int window);
/* io: host array of L descriptors.  Checks the arguments of every launch of the stack first (nothing is
 * enqueued if any is bad), then enqueues layer by layer.  A step of T <= 4 tokens at 128x128 states with at most
 * 16 query rows (T * Hq/Hkv) per KV head runs every layer as one fused launch over the request lists of all mixers
 * present; if one of its attention calls has several page ranges, their partial results are merged at the head of
 * the next layer's launch (a small merge launch of its own follows the last layer).  Any other step runs one launch
 * (attention: plus a merge) per mixer present.  Either way the attention rows
 * come out bit for bit as from attn_decode over the same request list; recurrent rows agree with the stand-alone
 * steps to the rounding order of their sums (a tile's rows are added in an order that depends on the workgroup's place
 * in the grid; a given launch is run-to-run deterministic).  Every layer's output is complete in stream order when
 * the call's last launch has run.
 * Layers may share one output buffer or use one each: where the outputs of two consecutive layers overlap, the
 * earlier layer's partial results are merged by a launch of their own instead of riding on the later layer's launch.
 * Recurrent layers update their states in place, by all T steps or by each request's n_commit_rows.
 * workspace: device memory, 256-byte aligned, at least placement_workspace_bytes(); SA_EWORKSPACE if too small. */
sa_status placement_decode(const sa_plan* plan, const sa_layer_io* io, const sa_shapes* shapes, int T, int window,
                           float attn_scale, float rec_scale, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Unified page pool (Section 6, "Heterogeneous state": FA caches grow with the sequence, SWA caches are
 * bounded at the window, GDN / KDA keep a fixed-size state, and a unified page size lets one paged memory
 * manager serve all layer kinds).  Host-side bookkeeping only: the caller allocates one device arena of
 * n_pages * sa_pool_page_bytes() bytes and the pool hands out page numbers.
 *
 * One unified page is the recurrent state of one (sequence, layer): H*dk*dv*4 bytes.  For an attention
 * layer the same page holds the K and V blocks of sa_pool_tokens_per_page() tokens: first the K blocks of
 * its 16-token pages, then, from the middle of the page, their V blocks.  With
 *     kpool = arena,  vpool = arena + page_bytes/2,  n_pages(kernel) = sa_pool_kernel_pages()
 * the 16-token page i of unified page u has the kernel page id u * sa_pool_kv_id_stride() + i, and the
 * attention and append entry points above work on the arena unchanged.  sa_pool_kernel_pages() is
 * n_pages * sa_pool_kv_id_stride() - sa_pool_kv_id_stride()/2, one past the last id whose K and V blocks both
 * lie inside the arena (the V block of an id sits half a unified page behind its K block), so that the kernels'
 * clamp of a bad table entry stays inside the arena for V as well.  For a recurrent layer
 *     state = (float*)arena,  slot = u
 * (convolution histories, if used, live in caller arrays indexed by the same slot).
 * Requires page_bytes to be a multiple of 2 * Hkv*16*D*2 (SA_EUNSUPPORTED otherwise).
 *
 * A sequence names a placement (one of F,S,K,G per layer).  sa_pool_seq_create gives every K/G layer its
 * state page; sa_pool_seq_reserve(len) makes tokens [0,len) addressable on F layers and the last
 * `window` + `slack` tokens on S layers, returning pages that fell out of the window to the pool; it
 * either succeeds completely or changes nothing (SA_ENOMEM).  Not thread-safe.
 */
typedef struct sa_pool sa_pool;
sa_status sa_pool_create(int n_pages, const sa_shapes* shapes, int n_layers, sa_pool** pool_out);
void sa_pool_destroy(sa_pool* pool);
size_t sa_pool_page_bytes(const sa_pool* pool);
int sa_pool_tokens_per_page(const sa_pool* pool);
int sa_pool_kv_id_stride(const sa_pool* pool);
int sa_pool_kernel_pages(const sa_pool* pool);
int sa_pool_free_pages(const sa_pool* pool);
sa_status sa_pool_seq_create(sa_pool* pool, const char* placement, int* seq_id_out);
sa_status sa_pool_seq_reserve(sa_pool* pool, int seq_id, int len, int window, int slack);
sa_status sa_pool_seq_free(sa_pool* pool, int seq_id);
int sa_pool_seq_pages(const sa_pool* pool, int seq_id);      /* pages the sequence holds now; -1 if unknown */
/* Host tables of one layer for a batch of sequences: page_table [B,max_pages] in kernel page ids (-1 where
 * nothing is mapped or the layer is not an attention layer for that sequence), slot [B] = state page of a
 * recurrent layer (-1 otherwise).  Either output may be NULL. */
sa_status sa_pool_layer_tables(const sa_pool* pool, const int32_t* seq_ids, int B, int layer, int32_t* page_table,
                               int max_pages, int32_t* slot);

/* ---------------------------------------------------------------------------------------------
 * Measurement helpers (not part of the method).
 */
enum { SA_K_GDN = 0, SA_K_KDA = 1, SA_K_ATTN_SPLIT = 2, SA_K_ATTN_MERGE = 3, SA_K_KV_APPEND = 4, SA_K_COPY = 5,
       SA_K_GDN_BLOCK = 6, SA_K_KDA_BLOCK = 7, SA_K_GDN_CHUNK = 8, SA_K_KDA_CHUNK = 9, SA_K_STREAM = 10, SA_K_LAYER = 11, SA_K_COUNT = 12 };
/* While enabled, every launch of the kernels above carries HIP start/stop events on its stream that
 * are stamped with the begin and end of the kernel itself. */
void sa_prof_enable(int on);
/* Waits for the recorded events of `kernel`, returns their count and summed duration, and forgets them.
 * If ms_each is not NULL (host array of `capacity` floats) the first `capacity` durations are
 * also stored there in launch order. */
sa_status sa_prof_read(int kernel, int* n_launches, float* total_ms, float* ms_each, int capacity);
/* Plain streaming copy of n_bytes (multiple of 16) used to calibrate bandwidth counters. */
sa_status sa_copy_bytes(const void* src, void* dst, size_t n_bytes, void* stream);
/* The memory traffic of a recurrent decode step at 128x128 without its arithmetic, to measure what the access
 * pattern itself can reach: one workgroup per 64 KiB tile of `tiles` (device, n_tiles * 16384 floats, 16-byte
 * aligned), lane pattern and cache hints of the step kernel.  kind 0 reads every tile, 1 overwrites every tile
 * with a constant, 2 reads each tile, scales it by 0.999 and writes it back.  SA_EINVAL on another kind, a
 * negative count, a null or misaligned pointer. */
sa_status sa_stream_tiles(int kind, float* tiles, int n_tiles, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SAMIXERS_H */
