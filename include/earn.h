/*
 * libearn — the attention hot path of EARN's register-token inference scheme on one MI355X (gfx950).
 *
 * EARN places register tokens at the head and tail of every prompt, runs the first k layers over the whole
 * sequence, gathers the register rows at the input of layer k, and from then on (later layers of the prefill and
 * every decode step) attends over registers plus generated tokens only (paper Section 3.2, "Inference").
 *
 * Conventions for every entry point
 *   - plain C ABI; every pointer is DEVICE memory owned by the caller unless marked "host";
 *   - the library owns no memory, never allocates and never synchronises: a call validates its scalar arguments
 *     on the host, enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the null stream) and returns;
 *   - tensors are row-major, packed ragged over the batch: [tokens, heads, head_dim], element type bf16 or fp32
 *     (earn_attn_desc.dtype); softmax statistics and accumulators are fp32; lengths and indices are int32;
 *   - scalars the host needs for grid sizing (batch, total_tokens, max_seqlen, ...) are passed by value so that no
 *     device-to-host read is needed.  Conditions that live in device memory (cu_seqlens starting at 0 and
 *     non-decreasing, n_s >= h+t, 0 <= gen_len < gen_cap, stream_to_seq in [0, batch), positions >= 0) are
 *     PRECONDITIONS and are NOT checked by a normal call.  What the kernels do guard: gen_len is clamped into
 *     [0, gen_cap) before the cache append and the walk over the generated rows, stream_to_seq is clamped into
 *     [0, batch), the compaction clamps a source row into its sequence (an empty sequence yields zero rows), and the
 *     prefill entry points, which are told total_tokens, hold every sequence's bounds inside [0, total_tokens], its
 *     length within max_seqlen and (earn_prefill_register_rows) every row_pos inside its sequence: wrong values
 *     there give wrong results, no stray access.  The same holds for the decode entry points (shared_cu against
 *     shared_total and max_shared_len), the compaction, the statistics and the backward (cu_seqlens against
 *     total_tokens): wrong VALUES in these arrays give wrong results, never an access outside the tensors.
 *     earn_set_validation(1) switches on a debug mode in which every call first copies these arrays to the host,
 *     checks them and returns EARN_ERR_INVALID_ARG before any kernel is launched;
 *   - return value: EARN_OK or a negative error code; earn_last_error() returns a thread-local message.
 *
 * The split layer k and the layer count N are not kernel arguments: the caller expresses them by which cache and
 * which cu_seqlens it hands to which call (first k layers: the full-length tensors; remaining N-k layers: the
 * compacted ones).
 */
#ifndef EARN_H
#define EARN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EARN_OK 0
#define EARN_ERR_INVALID_ARG (-1)
#define EARN_ERR_UNSUPPORTED (-2)
#define EARN_ERR_WORKSPACE_TOO_SMALL (-3)
#define EARN_ERR_HIP (-4)

#define EARN_F32 0
#define EARN_BF16 1

/* Largest number of tensors one earn_compact_registers call gathers. */
#define EARN_MAX_COMPACT_TENSORS 112

/* Attention description shared by prefill and decode (host struct, read during the call only). */
typedef struct {
  int32_t dtype;          /* EARN_F32 | EARN_BF16: element type of q, k, v, out and the caches */
  int32_t n_q_heads;      /* Hq */
  int32_t n_kv_heads;     /* Hkv; Hq % Hkv == 0 */
  int32_t head_dim;       /* d: 64 or 128 */
  const int32_t* q_to_kv; /* HOST array [Hq] or NULL: kv head that query head a reads (grouped-query attention).
                             NULL means a / (Hq/Hkv).  An explicit map may permute the heads but must give every kv
                             head exactly Hq/Hkv query heads, and Hq <= 128; anything else -> EARN_ERR_UNSUPPORTED
                             (the kernels serve the query heads of a kv head together, in groups of equal size) */
  float softmax_scale;    /* <= 0 means 1/sqrt(head_dim) (Eq. 3) */
  float rope_base;        /* rotary base (10000); <= 0 disables the rotation */
} earn_attn_desc;

/* Message of the last error on the calling thread ("" if none). Never NULL. */
const char* earn_last_error(void);

/* Library version string and the GPU architecture the kernels were built for. */
const char* earn_version(void);

/*
 * Debug validation of the preconditions that live in device memory (process-wide switch, off by default; returns the
 * previous setting).  While it is on, every entry point copies cu_seqlens / positions / gen_len / stream_to_seq /
 * q_pos / row_pos to the host on `stream`, WAITS for the stream, checks them (cu_seqlens[0] == 0, non-decreasing,
 * cu_seqlens[batch] == total_tokens, lengths <= max_seqlen / max_shared_len, n_s >= h + t, 0 <= gen_len < gen_cap,
 * stream_to_seq in [0, batch) with at most 1024 streams per sequence, positions and q_pos in [0, 2^24), row_pos
 * ascending and inside its sequence) and returns EARN_ERR_INVALID_ARG, with a message naming the first offending
 * element, BEFORE any kernel is launched.  A call that passes behaves exactly as without validation.
 */
int earn_set_validation(int enabled);

/*
 * Launch-shape overrides for measurements (process-wide; the defaults are what was measured best, a value of 0
 * restores a default).  Returns EARN_OK, or EARN_ERR_INVALID_ARG for an unknown key.  Keys:
 *   "prefill_block_rows"    128 | 256: query rows per workgroup of the bf16 full-length prefill
 *   "decode_mfma_min_len"   shortest shared cache (rows) that always takes the matrix-core decode kernel (128)
 *   "decode_mfma_short_wgs" shorter caches take it when Hkv * batch is at most this (256)
 *   "decode_mfma_wgs"       workgroups the matrix-core decode kernel's key splits aim at (256)
 *   "decode_vec_wgs"        workgroups the vector decode kernel's key splits aim at (1024)
 *   "decode_vec_waves"      waves per workgroup of the vector decode kernel (1, 2 or 4)
 *   "compact_blocks"        16 KB blocks one compaction workgroup copies (1..4)
 *   "linear_tile"           1 | 2: output tile of the projection GEMMs, 256 x 128 (1) or 256 x 256 (2); default by size
 *   "linear_splits"         splits of the inner dimension when a workspace is given (default by size; 1 = none)
 */
int earn_set_tuning(const char* key, int32_t value);

/*
 * Causal prefill attention over a packed ragged batch (paper Section 2.2, Eq. 3; used for the "full computation"
 * layers 0..k-1 on all tokens and, with compacted inputs and explicit positions, for the "register-focused" layers
 * k..N-1 — Section 3.2, Inference).
 *
 * For each sequence s (tokens cu_seqlens[s] .. cu_seqlens[s+1]-1), query head a and its kv head c:
 *   q'_i = RoPE(q_i, p_i), k'_j = RoPE(k_j, p_j)   rotary embedding on half-split pairs (e, e + d/2),
 *                                                   theta_e = rope_base^(-2e/d), p = the token's ORIGINAL position
 *   out_i = sum_{j <= i} softmax_j(q'_i . k'_j * scale) v_j
 *
 *   q              [total_tokens, Hq, d]
 *   k, v           [total_tokens, Hkv, d]
 *   cu_seqlens     [batch+1] int32, cu_seqlens[0] = 0, non-decreasing, cu_seqlens[batch] = total_tokens
 *   positions      [total_tokens] int32 or NULL; NULL means p_i = i - cu_seqlens[s]. Compacted layers pass the
 *                  pos_out of earn_compact_registers so that suffix registers keep position h + L_s + j.
 *   max_seqlen     upper bound on any sequence length (grid sizing)
 *   out            [total_tokens, Hq, d]
 *   k_rot_out      [total_tokens, Hkv, d] or NULL: receives k' (this is what the layer's KV cache stores)
 *   lse_out        [total_tokens, Hq] fp32 or NULL: natural-log-sum-exp of each softmax row
 *   workspace      at least earn_prefill_workspace_bytes(...) bytes, 256-byte aligned; may be NULL when that is 0
 * With the rotation switched off (rope_base <= 0) and k_rot_out == NULL the keys are read in place: no rotation pass, no
 * workspace (the form used behind earn_qkv_rope_project, whose k_out already is the rotated cache).
 *
 * Errors: NULL required pointer, batch <= 0, total_tokens < 0, max_seqlen <= 0, Hq % Hkv != 0 -> INVALID_ARG;
 * head_dim not in {64,128} or unknown dtype -> UNSUPPORTED; workspace_bytes too small -> WORKSPACE_TOO_SMALL.
 * total_tokens == 0 is a no-op.
 */
int earn_prefill_attn(const earn_attn_desc* desc, const void* q, const void* k, const void* v,
                      const int32_t* cu_seqlens, const int32_t* positions, int32_t batch, int32_t total_tokens,
                      int32_t max_seqlen, void* out, void* k_rot_out, float* lse_out, void* workspace,
                      size_t workspace_bytes, void* stream);

/* Workspace earn_prefill_attn needs (bytes): the rotated keys when no k_rot_out is supplied, plus, for bf16, a
 * [total_tokens, d/2] table of (cos, sin) pairs that the query rotation reads. Scratch only: nothing in it outlives the
 * call. 0 on invalid desc. */
size_t earn_prefill_workspace_bytes(const earn_attn_desc* desc, int32_t batch, int32_t total_tokens,
                                    int32_t max_seqlen, int32_t have_k_rot_out);

/*
 * Register compaction at the input of layer k (paper Section 3.2, Inference item 2, prefilling bullet:
 * X = [X_prefix; X_prompt; X_suffix] -> X' = [X_prefix; X_suffix]).
 *
 * For every sequence keeps rows [0, h) and [n_s - t, n_s) in order; row m of the result (m in [0, batch*(h+t)))
 * comes from source row idx = cu_seqlens[s] + p with s = m / r, j = m % r, p = j < h ? j : n_s - t + (j - h).
 * The gather is a pure byte copy (bit-exact), applied to n_tensors tensors that share the packed row index
 * (the hidden state, or K/V of the layers that follow) in one launch.
 *
 *   src, dst       HOST arrays of n_tensors device pointers; src[i] is [total_tokens, row_bytes[i]] bytes,
 *                  dst[i] is [batch*(h+t), row_bytes[i]] bytes; 16-byte aligned; n_tensors may be 0 (indices only)
 *   row_bytes      HOST array, each a positive multiple of 16
 *   cu_seqlens     [batch+1] int32 (device)
 *   total_tokens   rows of every src[i] (>= cu_seqlens[batch]); source rows are held inside it
 *   idx_out        [batch*(h+t)] int32 or NULL: source row of every kept row
 *   pos_out        [batch*(h+t)] int32 or NULL: original position p of every kept row
 *   cu_out         [batch+1] int32 or NULL: cu_out[s] = s*(h+t)
 *
 * Precondition (device data): n_s >= h + t for every s.  n_s == h + t is the identity permutation.
 * Errors: batch <= 0, total_tokens < 0, h < 0, t < 0, h + t == 0, n_tensors < 0 or > EARN_MAX_COMPACT_TENSORS, NULL src/dst/row_bytes
 * with n_tensors > 0, a NULL or misaligned tensor pointer, row_bytes not a positive multiple of 16 -> INVALID_ARG.
 */
int earn_compact_registers(int32_t n_tensors, const void* const* src, void* const* dst, const int64_t* row_bytes,
                           const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t n_head_reg,
                           int32_t n_tail_reg, int32_t* idx_out, int32_t* pos_out, int32_t* cu_out, void* stream);

/*
 * Positions of decode step `step` (the reading of Section 3.2's decoding bullet that this library takes: a generated
 * token keeps the position it would have without compaction): for every stream u of sequence s = stream_to_seq[u]
 *   q_pos[u] = n_s + step     (n_s = cu_seqlens[s+1] - cu_seqlens[s], the FULL sequence length, registers included)
 *   gen_len[u] = step         (rows already in the stream's generated cache)
 * which are the q_pos / gen_len arguments of earn_decode_attn for that step.
 *   cu_seqlens [batch+1] device (of the full-length sequences, also for layers >= k); stream_to_seq [n_streams] device
 *   or NULL (identity, n_streams == batch); q_pos, gen_len [n_streams] device, either may be NULL.
 * Errors: NULL cu_seqlens, n_streams <= 0, batch <= 0, step < 0, NULL map with n_streams != batch -> INVALID_ARG.
 */
int earn_decode_step_positions(const int32_t* cu_seqlens, const int32_t* stream_to_seq, int32_t n_streams,
                               int32_t batch, int32_t step, int32_t* q_pos, int32_t* gen_len, void* stream);

/*
 * One decode step of attention (paper Section 2.2, Eq. 4: append K_t, V_t to the cache, then Q_t K_{1:t}^T;
 * Section 3.2, Inference, decoding bullet: layers >= k see [prefix; suffix; generated] only).
 *
 * There are n_streams decode streams (beams); stream u belongs to sequence s = stream_to_seq[u] and shares that
 * sequence's prefill cache rows shared_cu[s] .. shared_cu[s+1]-1 with the other beams of s.  For each stream:
 *   q' = RoPE(q_u, q_pos[u]);  k' = RoPE(k_new_u, q_pos[u]);
 *   gen_k[u, gen_len[u]] = k';  gen_v[u, gen_len[u]] = v_new_u            (cache append)
 *   out_u = softmax over { shared rows of s } ++ { gen rows 0 .. gen_len[u] } of (q' . key * scale), times values.
 * No mask: every key is in the past.  The same call serves layers < k (shared_* = the full-length cache of the
 * layer) and layers >= k (shared_* = the compacted register cache).
 *
 *   q                  [n_streams, Hq, d]
 *   k_new, v_new       [n_streams, Hkv, d], k_new NOT yet rotated
 *   q_pos              [n_streams] int32: original position of the new token (n_s + step)
 *   shared_k, shared_v [shared_total, Hkv, d]; shared_k already rotated (k_rot_out of the prefill)
 *   shared_cu          [batch+1] int32
 *   stream_to_seq      [n_streams] int32 or NULL (= identity, requires n_streams == batch); a sequence may hold any
 *                      number of streams, none included, but at most 1024 (device-side precondition, checked exactly in
 *                      the validation mode; streams of a sequence beyond its first 1024 get no output.  The host
 *                      rejects what it can tell from n_streams and batch alone: n_streams > 1024 batch -> UNSUPPORTED)
 *   gen_k, gen_v       [n_streams, gen_cap, Hkv, d]; slot gen_len[u] of stream u is written by this call
 *   gen_len            [n_streams] int32, 0 <= gen_len[u] < gen_cap
 *   max_shared_len     upper bound on shared_cu[s+1] - shared_cu[s]
 *   shared_total       rows of shared_k / shared_v (>= shared_cu[batch]); sequence bounds are held inside it
 *   out                [n_streams, Hq, d]
 *   workspace          at least earn_decode_workspace_bytes(...) bytes, 256-byte aligned
 *
 * Errors: as for earn_prefill_attn, plus gen_cap <= 0, n_streams <= 0, stream_to_seq == NULL with
 * n_streams != batch, max_shared_len < 0 -> INVALID_ARG; more than 8 query heads per kv head -> UNSUPPORTED.
 * Values in device memory (gen_len < gen_cap, monotone shared_cu, stream_to_seq in [0, batch)) are preconditions.
 */
int earn_decode_attn(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                     const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                     const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len, int32_t gen_cap,
                     int32_t n_streams, int32_t batch, int32_t max_shared_len, int32_t shared_total, void* out, void* workspace,
                     size_t workspace_bytes, void* stream);

/* Workspace earn_decode_attn needs (bytes) for split-key partial results. 0 on invalid desc. */
size_t earn_decode_workspace_bytes(const earn_attn_desc* desc, int32_t n_streams, int32_t batch,
                                   int32_t max_shared_len, int32_t gen_cap);

/*
 * Several INDEPENDENT layers in one launch (harness throughput mode; n_layers = 1 is the real-model use, in which layer
 * l+1 depends on layer l).  The register-focused layers k..N-1 of the paper's Section 3.2 work on a few dozen rows per
 * sequence, so a launch per layer is bound by launch latency, not by the arithmetic or the bytes of Eq. 3 / Eq. 4; with
 * synthetic per-layer inputs the layers do not depend on each other and one grid dimension can index the layer.
 * Layer l of a tensor starts `*_layer_stride` BYTES (a positive multiple of 16; of 4 for lse_out) after layer l-1; cu_seqlens, positions,
 * q_pos, gen_len and stream_to_seq are shared by all layers.  Every layer computes exactly what the single-layer call
 * computes (same kernels; only the number of key splits may differ, because the layers share the GPU).
 *
 * earn_prefill_attn_layers: k_rot_out is required; lse_out may be NULL; workspace as for earn_prefill_attn with
 * k_rot_out given (earn_prefill_workspace_bytes(desc, batch, total_tokens, max_seqlen, 1)), shared by the layers.
 * earn_decode_attn_layers: workspace of earn_decode_layers_workspace_bytes(...) bytes.
 * Errors: as the single-layer calls; n_layers outside [1, 65535] or a bad stride -> INVALID_ARG.
 */
int earn_prefill_attn_layers(const earn_attn_desc* desc, int32_t n_layers, const void* q, int64_t q_layer_stride,
                             const void* k, const void* v, int64_t kv_layer_stride, const int32_t* cu_seqlens,
                             const int32_t* positions, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                             void* out, int64_t out_layer_stride, void* k_rot_out, int64_t k_rot_layer_stride,
                             float* lse_out, int64_t lse_layer_stride, void* workspace, size_t workspace_bytes,
                             void* stream);
int earn_decode_attn_layers(const earn_attn_desc* desc, int32_t n_layers, const void* q, int64_t q_layer_stride,
                            const void* k_new, const void* v_new, int64_t kv_new_layer_stride, const int32_t* q_pos,
                            const void* shared_k, const void* shared_v, int64_t shared_layer_stride,
                            const int32_t* shared_cu, const int32_t* stream_to_seq, void* gen_k, void* gen_v,
                            int64_t gen_layer_stride, const int32_t* gen_len, int32_t gen_cap, int32_t n_streams,
                            int32_t batch, int32_t max_shared_len, int32_t shared_total, void* out, int64_t out_layer_stride, void* workspace,
                            size_t workspace_bytes, void* stream);
size_t earn_decode_layers_workspace_bytes(const earn_attn_desc* desc, int32_t n_layers, int32_t n_streams,
                                          int32_t batch, int32_t max_shared_len, int32_t gen_cap);

/*
 * earn_decode_attn for callers that cannot allocate or pass device scratch memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * earn_decode_attn, without the workspace: the split-key partial results go to a buffer that lives inside the library
 * (a file-scope device array of EARN_STATIC_SCRATCH_BYTES bytes, one copy per GPU, held until the process ends; its
 * device address is looked up once per GPU, on the first call made with that GPU current).  The call allocates
 * nothing and frees nothing (with earn_set_validation on, the debug checks do allocate host memory and wait for the
 * stream: keep validation off in such callers).
 *
 * Every call on a GPU uses that GPU's one buffer, which keeps the previous call's contents; nothing in it has to
 * start at zero (each partial result is written before it is read within a call).  Calls that overlap in time on one
 * GPU (different streams, or threads) RACE on the buffer: serialise them, or use earn_decode_attn with a workspace
 * per stream.
 *
 * Errors: as earn_decode_attn; a problem whose partial results need more than EARN_STATIC_SCRATCH_BYTES
 * (earn_decode_workspace_bytes tells) -> EARN_ERR_WORKSPACE_TOO_SMALL, nothing is launched.
 */
#define EARN_STATIC_SCRATCH_BYTES (8u << 20)
int earn_decode_attn_static(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                            const int32_t* q_pos, const void* shared_k, const void* shared_v,
                            const int32_t* shared_cu, const int32_t* stream_to_seq, void* gen_k, void* gen_v,
                            const int32_t* gen_len, int32_t gen_cap, int32_t n_streams, int32_t batch,
                            int32_t max_shared_len, int32_t shared_total, void* out, void* stream);

/*
 * Prefill attention of the LAST full-length layer (layer k-1) at the register rows only.
 *
 * Section 3.2 (inference): the input of layer k keeps only the register tokens, so of layer k-1's attention outputs
 * only the rows of the h prefix and t suffix registers are ever used; the layer's keys and values are still needed at
 * full length (they are the layer's cache, which decoding reads: Section 3.2, decoding; Section 3.3, N_KV's k L term).
 * This entry point computes exactly those rows of Eq. 3 — row m of sequence s is the causal attention of token
 * row_pos[s*r + m] over keys 0 .. row_pos[s*r + m] of the sequence — and rotates K into the cache, skipping the
 * other n_s - r query rows: an exact saving of about 1/k of the prefill attention work that the efficiency analysis
 * of Section 3.3 (Gamma_attn) does not count.
 *
 *   q_rows        device, [batch*r, Hq, d]: the query rows of the register tokens in compacted order, un-rotated
 *                 (what earn_compact_registers gathers from the layer's [total, Hq, d] queries)
 *   k, v          device, [total_tokens, Hkv, d], K un-rotated; rotary positions of K are the token indices in the
 *                 sequence (this entry point takes no explicit position list for K)
 *   cu_seqlens    device, [batch+1]
 *   row_pos       device, [batch*r]: token index inside its sequence (= rotary position) of every row, ascending per
 *                 sequence, each < the sequence's length (earn_compact_registers' pos_out); precondition, unchecked
 *   rows_per_seq  r = h + t, the same for every sequence, <= 1024
 *   out_rows      device, [batch*r, Hq, d]
 *   k_rot_out     device, [total_tokens, Hkv, d], required: the rotated keys = the layer's cache
 *   workspace     at least earn_prefill_register_rows_workspace_bytes(...) bytes, 256-byte aligned; may be NULL when 0
 * Both dtypes (fp32 needs no workspace).  Enqueues on `stream`, allocates nothing, does not synchronise.
 */
int earn_prefill_register_rows(const earn_attn_desc* desc, const void* q_rows, const void* k, const void* v,
                               const int32_t* cu_seqlens, const int32_t* row_pos, int32_t batch, int32_t total_tokens,
                               int32_t max_seqlen, int32_t rows_per_seq, void* out_rows, void* k_rot_out,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Workspace earn_prefill_register_rows needs (bytes) for split-key partial results. 0 on invalid arguments. */
size_t earn_prefill_register_rows_workspace_bytes(const earn_attn_desc* desc, int32_t batch, int32_t max_seqlen,
                                                  int32_t rows_per_seq);

/*
 * The dense projections of a decoder layer (paper Appendix A.2: per head, Q/K/V projections 3 x 2 L d_h d_a and the output
 * projection 2 L d_a d_h; feed-forward block, two projections, 4 L d_h d_f), bf16 with fp32 accumulation.
 *
 * earn_qkv_rope_project: [rows, d_model] x [(Hq + 2 Hkv) d, d_model]^T -> Q, K, V, with the rotary embedding applied to the
 * Q and K columns at each row's ORIGINAL position in the epilogue (same convention as earn_prefill_attn: half-split
 * pairs, theta_e = rope_base^(-2e/d); rope_base <= 0: no rotation).  k_out is what the layer's key cache stores, so the
 * attention entry points are then called with rope_base = 0 and, for the prefill, k_rot_out = NULL: they read q_out /
 * k_out as they are and run no rotation pass.  Rows of the register-focused layers (Section 3.2) are the gathered hidden
 * rows, with positions = pos_out of earn_compact_registers; decode rows are the new tokens with positions = q_pos.
 *   x          device, [rows, d_model] bf16           w_qkv   device, [(Hq + 2 Hkv) d, d_model] bf16, one row per output
 *                                                             (the layout checkpoints keep a linear layer's weight in):
 *                                                             the Q heads, then the K heads, then the V heads
 *   positions  device, [rows] int32 or NULL; NULL: row i of sequence s has position i - cu_seqlens[s] (cu_seqlens, batch
 *              required then)
 *   q_out      device, [rows, Hq, d];  k_out, v_out  device, [rows, Hkv, d]
 * earn_linear: out[rows, n] = act(x[rows, k] w[n, k]^T), activation 0 = none, 1 = SiLU (x / (1 + e^-x)); bf16; w holds
 * one row of k inputs per output.
 *   workspace  device, optional (NULL / 0: never needed for a correct result).  A product with few rows (register rows,
 *              decode rows) has too few output tiles to occupy the GPU; given earn_linear_workspace_bytes(rows, k, n)
 *              bytes (256-byte aligned; 0 when the product is large enough as it is) the inner dimension is split over
 *              more workgroups, fp32 partial sums pass through the workspace and a second kernel adds them and applies
 *              the epilogue.  Same results up to fp32 summation order.  For earn_qkv_rope_project, n = (Hq + 2 Hkv) d.
 * Errors: NULL pointer, non-positive size, positions and cu_seqlens both NULL with rotation on -> INVALID_ARG;
 * desc->dtype != EARN_BF16, an inner dimension that is not a multiple of 64, an output width that is not a multiple of
 * 8, 256 rows of the inner dimension reaching 2 GiB -> UNSUPPORTED.  Enqueue on `stream`, allocate nothing.
 */
int earn_qkv_rope_project(const earn_attn_desc* desc, const void* x, const void* w_qkv, int32_t rows, int32_t d_model,
                          const int32_t* cu_seqlens, const int32_t* positions, int32_t batch, void* q_out, void* k_out,
                          void* v_out, void* workspace, size_t workspace_bytes, void* stream);
int earn_linear(const void* x, const void* w, int32_t rows, int32_t k, int32_t n, int32_t activation, void* out,
                void* workspace, size_t workspace_bytes, void* stream);
size_t earn_linear_workspace_bytes(int32_t rows, int32_t k, int32_t n);

/*
 * Backward of the causal attention (paper Section 3.2, Training: the loss is differentiated through the same attention,
 * over all tokens in layers l <= k and over register + target tokens in layers l > k; Eq. 3).  Inputs are the forward's,
 * AS THE ATTENTION SAW THEM: q and k already rotated (q_out / k_out of earn_qkv_rope_project, or the k_rot_out of the
 * forward), out and lse_out of earn_prefill_attn, and d_out = dLoss/dOut.  Computes
 *   dq [total, Hq, d], dk, dv [total, Hkv, d]   (gradients with respect to the ROTATED q, k and to v; dk, dv summed over
 *                                               the query heads of each kv head; the rotation's own backward belongs
 *                                               to the projection's backward, which is not part of this library)
 * in the tensors' element type, fp32 arithmetic.  For the register-focused layers pass the compacted tensors and cu_out.
 * desc->rope_base must be <= 0 (nothing is rotated here); softmax_scale and q_to_kv as in the forward.
 *   workspace: at least earn_attn_backward_workspace_bytes(desc, total_tokens) bytes (one float per (token, query head))
 * Errors: NULL pointer, non-positive size -> INVALID_ARG; rope_base > 0 -> UNSUPPORTED; workspace -> WORKSPACE_TOO_SMALL.
 * A first form on the vector ALU (no matrix cores): correct at any length, meant for the short sequences of the
 * register-focused layers and for checking.
 */
int earn_attn_backward(const earn_attn_desc* desc, const void* q, const void* k, const void* v, const void* out,
                       const float* lse, const void* d_out, const int32_t* cu_seqlens, int32_t batch,
                       int32_t total_tokens, int32_t max_seqlen, void* dq, void* dk, void* dv, void* workspace,
                       size_t workspace_bytes, void* stream);
size_t earn_attn_backward_workspace_bytes(const earn_attn_desc* desc, int32_t total_tokens);

/*
 * Beam search around the decode step (paper Appendix, implementation details: inference decodes with beam search, beam
 * size 20).  The attention path has no logits; these calls take the per-beam token log-probabilities from the caller.
 *
 * earn_beam_topk: for every sequence b (beams live beams, streams b*beams .. b*beams + beams - 1) keeps the `beams` best of
 * the beams * vocab candidates  beam_scores[b*beams + w] + token_logprobs[b*beams + w][t]  (fp32 sum), best first, equal
 * scores in order of the candidate index w * vocab + t; NaN candidates never win.
 *   beam_scores    device, [batch*beams] fp32, or NULL (all zero)
 *   token_logprobs device, [batch*beams, vocab] fp32
 *   parent_out     device, [batch*beams] int32: STREAM index (b*beams + w) of each kept candidate's parent beam
 *   token_out      device, [batch*beams] int32;  score_out  device, [batch*beams] fp32
 *   (-1, -1, -inf for picks beyond the number of candidates)
 *   workspace      at least earn_beam_topk_workspace_bytes(batch, beams, vocab) bytes (0 when beams * vocab <= 8192)
 * Errors: NULL pointer, non-positive size -> INVALID_ARG; beams > 64 or beams * vocab beyond 3.3e6 -> UNSUPPORTED.
 *
 * earn_beam_reorder: the ancestor table after a beam step at decode step `step` (the step whose rows were just appended).
 * gen_src[u][g] names the physical stream whose cache slot g holds row g of stream u's generated history; the decode
 * entry point reads generated rows through it (earn_decode_attn_beams), so a beam step moves n_streams * step integers,
 * shared by all layers, instead of copying n_streams * step K/V rows in every layer.
 *   gen_src_out[u][g] = gen_src_in[parent[u]][g] for g < step (parent[u] itself when gen_src_in is NULL),
 *                       parent[u] for g == step, u for g > step.
 *   parent device [n_streams]; gen_src_in device [n_streams, gen_cap] or NULL (identity); gen_src_out device
 *   [n_streams, gen_cap], must not alias gen_src_in.
 * Errors: NULL parent / gen_src_out, aliasing, n_streams <= 0, gen_cap <= 0, step outside [0, gen_cap) -> INVALID_ARG.
 *
 * earn_decode_attn_beams: earn_decode_attn with the ancestor table: row g < gen_len[u] of stream u's generated cache is
 * read from slot (gen_src[u][g], g) of gen_k / gen_v; the new row is still appended at (u, gen_len[u]).
 * gen_src NULL = earn_decode_attn.
 */
int earn_beam_topk(const float* beam_scores, const float* token_logprobs, int32_t batch, int32_t beams, int32_t vocab,
                   int32_t* parent_out, int32_t* token_out, float* score_out, void* workspace, size_t workspace_bytes,
                   void* stream);
size_t earn_beam_topk_workspace_bytes(int32_t batch, int32_t beams, int32_t vocab);
int earn_beam_reorder(const int32_t* parent, const int32_t* gen_src_in, int32_t* gen_src_out, int32_t n_streams,
                      int32_t gen_cap, int32_t step, void* stream);
int earn_decode_attn_beams(const earn_attn_desc* desc, const void* q, const void* k_new, const void* v_new,
                           const int32_t* q_pos, const void* shared_k, const void* shared_v, const int32_t* shared_cu,
                           const int32_t* stream_to_seq, void* gen_k, void* gen_v, const int32_t* gen_len,
                           const int32_t* gen_src, int32_t gen_cap, int32_t n_streams, int32_t batch,
                           int32_t max_shared_len, int32_t shared_total, void* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Attention-score statistics of chosen query rows (paper Appendix, "Quantitative Measurements of Attention Score
 * Distributions"): for the causal softmax row p_1 .. p_n of a query row (Eq. 3; n = the row's token index + 1)
 *   stats[0] = Sparsity  = (1/n) * #{ j : p_j > epsilon }        (the paper sets epsilon = 0.05)
 *   stats[1] = Sink_head = sum_{j = 1}^{t_head} p_j              (t_head = 3)
 *   stats[2] = Sink_tail = sum_{j = n - tail_back}^{n} p_j       (tail_back = 3, i.e. T_t = n - 3: the last FOUR keys)
 * (rows shorter than a window sum what exists).  The rows are given as in earn_prefill_register_rows: r rows per
 * sequence, row m of sequence s being token row_pos[s*r + m] of the sequence, un-rotated queries; the keys are the
 * layer's cache (ROTATED keys, k_rot_out of the prefill).  The probabilities are recomputed in fp32.
 *
 *   q_rows     device, [batch*r, Hq, d], un-rotated      k_rot      device, [total_tokens, Hkv, d], rotated
 *   cu_seqlens device, [batch+1]                         row_pos    device, [batch*r], each inside its sequence
 *   stats_out  device, [batch*r, Hq, 3] fp32
 *   total_tokens  rows of k_rot (>= cu_seqlens[batch]); sequence bounds are held inside it
 * Errors: NULL pointer, batch <= 0, total_tokens < 0, rows_per_seq <= 0, epsilon < 0, t_head < 0, tail_back < 0 -> INVALID_ARG; desc as
 * for earn_prefill_attn.  Enqueues on `stream`, allocates nothing.
 */
int earn_attn_stats(const earn_attn_desc* desc, const void* q_rows, const void* k_rot, const int32_t* cu_seqlens,
                    const int32_t* row_pos, int32_t batch, int32_t total_tokens, int32_t rows_per_seq, float epsilon,
                    int32_t t_head, int32_t tail_back, float* stats_out, void* stream);

/*
 * KV-cache entries per attention head one sequence holds under EARN (paper Section 3.3, "KV Cache Size":
 * N_KV = n_h (k L + (N-k) r), here per head and with L = the length the first k layers see, plus `gen`
 * generated tokens kept by every layer).  Used for allocation and as an invariant.
 */
int64_t earn_cache_entries(int32_t n_layers, int32_t split_k, int64_t seq_len, int32_t n_registers, int64_t gen);

#ifdef __cplusplus
}
#endif
#endif /* EARN_H */
