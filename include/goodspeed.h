/*
 * goodspeed.h - C ABI of the verification-server hot path of GoodSpeed
 * (adaptive speculative decoding with N draft servers and one verifier).
 *
 * One round, verifier side (paper: Algorithm 1, verification-server steps;
 * Figure 1 steps 3-5):
 *   gs_verify_batch   target-decoder forward over the ragged speculative blocks
 *                     of all servers, then rejection-verification
 *   gs_accept_reject  rejection-verification alone, on given target logits
 *   gs_schedule_gamma estimator updates and the per-round scheduling problem
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers ordinary host
 *     memory.  Every buffer is owned by the caller; the library allocates no
 *     device memory and keeps no pointer after a call returns, except that a
 *     gs_ctx keeps the weight pointers given to gs_create.
 *   - GPU entry points only enqueue work on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); outputs are valid once the caller has
 *     synchronised that stream.  Two calls that share a workspace must be
 *     ordered on one stream.
 *   - Every entry point returns a gs_status; nothing throws or aborts.  All
 *     argument checks happen on the host before the first launch, so a failed
 *     call has launched nothing.  gs_last_error() gives the message of the last
 *     failure on the calling thread.
 *   - Server i drafts gamma[i] tokens (the paper's S_i(t)).  Its block has
 *     T_i = gamma[i] + 1 target rows: the pending token (the correction/bonus
 *     token of the previous round, not yet in the KV cache) followed by the
 *     drafts.  Row j (0-based) of a block yields p_{j+1}, so the block yields
 *     p_1 .. p_{gamma+1} as the rejection rule needs (paper Section II-A-2).
 *     Rows of all servers are concatenated in server order: R = sum T_i target
 *     rows, G = sum gamma[i] draft rows.  cu_rows[i] = first target row of
 *     server i, cu_rows[N] = R; the first draft row of server i is cu_rows[i] - i.
 */
#ifndef GOODSPEED_H
#define GOODSPEED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GS_OK = 0,
  GS_EINVAL = -1,       /* null pointer, negative size, inconsistent descriptor */
  GS_ESHAPE = -2,       /* model shape the kernels do not support              */
  GS_ECAPACITY = -3,    /* workspace or KV pages too small                     */
  GS_EDEVICE = -4,      /* a HIP call failed                                   */
  GS_EUNSUPPORTED = -5
} gs_status;

enum { GS_F32 = 0, GS_BF16 = 1, GS_W4 = 2 /* bf16 activations, KV and embedding; 4-bit projection weights */ };

/* Message of the last error on this thread (static storage, never NULL). */
const char* gs_last_error(void);

/* ------------------------------------------------------------------------- */
/* Rejection-verification (paper Section II-A-2; statistic: the sum inside the  */
/* acceptance-rate update of Section III-C).                                    */
/* ------------------------------------------------------------------------- */

/* The output arrays are written by the kernels with plain stores: any memory the device can address
 * will do, device memory or pinned host memory mapped into the device address space (then the results
 * are on the host once the stream has been synchronised, without a copy). */
typedef struct {
  int* accepted_len;   /* dev [N]  m_i in [0, gamma_i]: drafts kept before the first rejection      */
  int* next_token;     /* dev [N]  s'_i: drawn from normalised max(0, p_{m+1} - q_{m+1}) if          */
                       /*          m_i < gamma_i, else from p_{gamma+1}                              */
  float* accept_stat;  /* dev [N]  (1/gamma_i) sum over ALL gamma_i positions of min(1, p/q);        */
                       /*          0 when gamma_i = 0                                                */
  float* ratio;        /* dev [G]  p_j(s_j)/q_j(s_j) per draft row (+inf when q = 0); may be NULL    */
} gs_accept_out;

/* Bytes of device workspace gs_accept_reject needs for these sizes. */
size_t gs_accept_workspace_bytes(int n_servers, int n_rows, int vocab);

/*
 * Accept/reject + resample for N servers.
 *   gamma_host    host [N]      draft lengths, each >= 0
 *   cu_rows       dev  [N+1]    prefix offsets of T_i = gamma_i + 1 (must match gamma_host)
 *   target_logits dev  [R, V]   fp32 row-major; p = softmax(row)
 *   q_probs       dev  [G, V]   fp32 draft probabilities
 *   draft_tokens  dev  [G]      token ids in [0, V)
 *   u_accept      dev  [G]      uniforms in [0,1): token j accepted iff u <= p/q
 *   u_resample    dev  [N]      uniforms in [0,1) for the inverse-CDF draw of s'
 * The draw returns the smallest token whose running sum of weights exceeds
 * u * (total weight), tokens in index order; a zero-weight token is never
 * returned.  If max(0, p - q) has no mass the draw falls back to p.
 * Token ids are device data, so they cannot be checked before the launch: a server with a draft token id
 * outside [0, V) gets accepted_len = -1 (the id is never used as an index; its next_token is drawn as for m = 0).
 * Errors: GS_EINVAL (null pointers, N <= 0, vocab <= 0, gamma < 0, more than 2^22 rows),
 * GS_ECAPACITY (workspace too small), GS_EDEVICE.
 */
gs_status gs_accept_reject(int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                           const float* target_logits, const float* q_probs,
                           const int* draft_tokens, const float* u_accept, const float* u_resample,
                           const gs_accept_out* out, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * The same rule on bfloat16 inputs (half the bytes of the bandwidth-bound pass): target_logits dev [R, V] and
 * q_probs dev [G, V] hold bfloat16 bit patterns; everything else as gs_accept_reject, arithmetic in fp32.
 * The inputs are taken as the exact numbers they encode: p = softmax of the bfloat16 logits, q the bfloat16
 * values (which need not sum to one), so decisions and tokens are again defined exactly by the paper's rule
 * (Section II-A-2) and held to the same parity bar.  What rounding q to bfloat16 costs the method is on the
 * caller's side of the boundary: a draft token sampled from the unrounded q is accepted with probability
 * min(1, p/q~) instead of min(1, p/q), so the law of the emitted token is no longer exactly p: it differs
 * from p by less than 2^-8 in total variation (q~/q lies within 1 +- 2^-9).
 */
gs_status gs_accept_reject_bf16(int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                                const void* target_logits, const void* q_probs, const int* draft_tokens,
                                const float* u_accept, const float* u_resample, const gs_accept_out* out,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * gs_accept_reject for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * gs_accept_reject without the workspace; the kernels' scratch (chunk statistics, per-server decisions,
 * tile sums) lives in a device array of GS_ACCEPT_STATIC_SCRATCH_BYTES that is part of the library image
 * (every GPU the library runs on holds its own copy until the process ends).  The call allocates nothing
 * and frees nothing.  Its first call on a device looks up the array's address on that device
 * (hipGetSymbolAddress); make that call outside a graph capture.  All calls on one GPU share the array, which
 * keeps the last call's contents (every word a call reads it has written itself first): calls that overlap
 * in time on one GPU, on any streams, race.
 * Errors: as gs_accept_reject; GS_ECAPACITY when gs_accept_workspace_bytes(n_servers, rows, vocab) exceeds
 * GS_ACCEPT_STATIC_SCRATCH_BYTES (nothing is launched).
 */
#define GS_ACCEPT_STATIC_SCRATCH_BYTES (4u << 20)
gs_status gs_accept_reject_static(int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                                  const float* target_logits, const float* q_probs,
                                  const int* draft_tokens, const float* u_accept, const float* u_resample,
                                  const gs_accept_out* out, void* hip_stream);

/* ------------------------------------------------------------------------- */
/* Estimators and GoodSpeed-sched (paper Section III-C: the alpha-hat and X      */
/* smoothing equations and the scheduling problem; Algorithm 1 orders the       */
/* updates before the solve).  Pure host code.                                  */
/* ------------------------------------------------------------------------- */

/*
 *   accepted_len host [N]  m_i of the round just verified
 *   accept_stat  host [N]  mean min(1, p/q) of that round (ignored where gamma_prev = 0)
 *   gamma_prev   host [N]  draft lengths of that round
 *   alpha_hat    host [N]  in/out: (1-eta) alpha_hat + eta * accept_stat
 *   x_smooth     host [N]  in/out: (1-beta) X + beta * (m_i + 1)
 *   gamma_next   host [N]  out: maximiser of sum_i (1/X_i) (1 - a_i^(S_i+1))/(1 - a_i)
 *                          subject to sum S_i <= capacity, gamma_min <= S_i <= gamma_max
 * alpha_hat is clamped to [1e-6, 1-1e-6] inside the solve only.  gamma_max < 0
 * means unbounded.  The gain of a server's next slot is formed as (1/X) * pow(a, S + 1) in double; equal
 * gains go to the lowest server index.
 * Errors: GS_EINVAL (null, n <= 0, eta/beta outside [0,1], X <= 0 after update,
 * capacity < n * gamma_min, gamma_min < 0).
 */
gs_status gs_schedule_gamma(int n, const int* accepted_len, const float* accept_stat,
                            const int* gamma_prev, double* alpha_hat, double* x_smooth,
                            double eta, double beta, int capacity, int gamma_min, int gamma_max,
                            int* gamma_next);

/*
 * The two baseline allocation policies the paper compares GoodSpeed with (Section IV-A, Baselines).  Host code.
 *   gs_allocate_fixed   Fixed-S: capacity / n drafts for every server, the remainder to the lowest indices
 *   gs_allocate_random  Random-S: each of the `capacity` draft slots goes to server floor(u * n), u = uniforms[k]
 *                       (host [capacity], each in [0, 1))
 * gamma_next host [n], out.  Errors: GS_EINVAL.
 */
gs_status gs_allocate_fixed(int n, int capacity, int* gamma_next);
gs_status gs_allocate_random(int n, int capacity, const float* uniforms, int* gamma_next);

/* ------------------------------------------------------------------------- */
/* Batched verification step: decoder forward + rejection-verification          */
/* (paper Section II-A-1 for p = softmax(W h); Section II-A-2 for verification;  */
/* Figure 1 steps 3 and 4).  The decoder is a Llama-style stack: pre-norm        */
/* RMSNorm, rotary embedding (pairs (i, i + hd/2), inverse frequency             */
/* theta^(-2i/hd)), grouped-query causal attention, SwiGLU, no biases.           */
/* ------------------------------------------------------------------------- */

typedef struct {
  int n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_theta, rms_eps;
  int dtype;            /* GS_F32 or GS_BF16: storage type of weights, KV pages and GEMM operands;  */
                        /* GS_W4: as GS_BF16, but the projection matrices are 4-bit (see below)   */
} gs_model_desc;

/*
 * Projection matrices are logically [out_features, in_features] in the model dtype and must be
 * given in the layout gs_pack_weight produces (one-time repack at load):
 *   GS_F32 : row-major, unchanged
 *   GS_BF16: tile-packed [in/64][out/16][2][64][8]: for a tile of 16 output rows and a step of 64
 *            inputs, lane l = 16 g + c (c = row in tile, g = 0..3) owns inputs 16 g .. 16 g + 15 of
 *            row c, the first 8 in half 0 and the last 8 in half 1; so the 2 KB one wavefront needs
 *            per step are contiguous, and the blocks of all tiles at one step form one band.
 * The embedding table is gathered by row and stays row-major.
 */
gs_status gs_pack_weight(const void* w_rowmajor /* dev */, void* w_packed /* dev, same size, not in place */,
                         int n_out, int k_in, int dtype, void* hip_stream);

/*
 * 4-bit projection weights for GS_W4 models (weight-only quantisation in groups of 128 inputs, the format
 * family of the AWQ checkpoints of the paper's 70B verifier, Section IV-A):
 *   W[n][k] = (code[n][k] - zero[n][k/128]) * scale[n][k/128],  codes and zeros in 0..15, scales bf16;
 * every dequantised weight is rounded to bf16 (nearest even) before it enters the product.
 * gs_pack_weight_w4 turns the three arrays into the layout the projection kernel streams
 * (gs_w4_packed_bytes bytes: the codes tile-packed like the bf16 weights, then one word of scale and zero
 * per column and group).  k_in must be a multiple of 128, n_out of 64.
 *   codes   dev uint8 [n_out][k_in]      one code per byte
 *   scales  dev bf16  [n_out][k_in/128]
 *   zeros   dev uint8 [n_out][k_in/128]
 * Errors: GS_EINVAL, GS_ESHAPE, GS_EDEVICE.
 */
size_t gs_w4_packed_bytes(int n_out, int k_in);
gs_status gs_pack_weight_w4(const uint8_t* codes, const void* scales, const uint8_t* zeros, void* w_packed,
                            int n_out, int k_in, void* hip_stream);

typedef struct {
  const void* embed;          /* dev [V, d] row-major                                    */
  const void* lm_head;        /* dev [V, d] packed                                       */
  const float* final_norm;    /* dev [d] fp32                                            */
  const void* const* wqkv;    /* host [n_layers] of dev packed [(H + 2 H_kv) hd, d]: Q, K, V heads */
  const void* const* wo;      /* host [n_layers] of dev packed [d, H hd]                 */
  const void* const* wgu;     /* host [n_layers] of dev packed [2 F, d]: gate rows, up rows */
  const void* const* wd;      /* host [n_layers] of dev packed [d, F]                    */
  const float* const* norm1;  /* host [n_layers] of dev [d] fp32 (attention pre-norm)    */
  const float* const* norm2;  /* host [n_layers] of dev [d] fp32 (FFN pre-norm)          */
} gs_weights;

/* Paged KV cache in the model dtype.  K pages are key-major, V pages channel-major
 * (so that the slots of one channel are contiguous, which is what the second attention
 * product reads):
 *   k_pages [n_layers][n_pages][H_kv][page_size][hd]   K stored rotated
 *   v_pages [n_layers][n_pages][H_kv][hd][page_size]
 * page_size must be a multiple of 16 for GS_BF16 models. */
typedef struct {
  void* k_pages;
  void* v_pages;
  int page_size;
  int n_pages;
} gs_kv_cache;

typedef struct {
  int n_servers;
  const int* gamma_host;     /* host [N]                                                       */
  const int* ctx_len_host;   /* host [N]  tokens already cached per server                     */
  const int* cu_rows;        /* dev  [N+1] (matches gamma_host)                                */
  const int* ctx_len;        /* dev  [N]   (matches ctx_len_host)                              */
  const int* tokens;         /* dev  [R]   pending token then drafts, per server               */
  const int* block_table;    /* dev  [N, max_blocks] physical page of each logical block       */
  int max_blocks;
  const float* q_probs;      /* dev  [G, V]                                                    */
  const float* u_accept;     /* dev  [G]                                                       */
  const float* u_resample;   /* dev  [N]                                                       */
} gs_batch;

/* A gs_ctx holds the model description, the weight pointers and small host-side planning tables.
 * Calls on one context must not overlap in time (use one context per calling thread). */
typedef struct gs_ctx gs_ctx;

/* Validates the shape and copies the descriptor and the per-layer pointer tables.
 * Supported: head_dim in {64, 128}; n_heads a multiple of n_kv_heads with group <= 8;
 * d_model, d_ffn and every projection width multiples of 64.  Errors: GS_EINVAL, GS_ESHAPE. */
gs_status gs_create(const gs_model_desc* desc, const gs_weights* weights, gs_ctx** out);
gs_status gs_destroy(gs_ctx* ctx);

/* Device workspace gs_verify_batch needs for batches of at most max_rows target rows,
 * max_servers servers and max_ctx tokens of context (cached + block) per server. */
size_t gs_workspace_bytes(const gs_ctx* ctx, int max_rows, int max_servers, int max_ctx);

/*
 * One verification step.  Runs the decoder over all R rows at positions
 * ctx_len[i] + j, WRITES the block's K/V rows into the cache pages at those
 * positions (the caller advances ctx_len by m_i + 1 afterwards; rows beyond
 * that are dead and overwritten next round), then runs gs_accept_reject on the
 * resulting logits.
 *   logits_out  dev [R, V] fp32, or NULL to keep the logits in the workspace only
 * For bf16 models whose LM-head projection runs as one launch, that projection also leaves every row's softmax
 * statistics (max, sum exp) per column block, so the accept stage does not read the logits again for them.
 *   out->*      as for gs_accept_reject; if batch->q_probs is NULL the step stops
 *               after the logits (prefill use) and `out` may be NULL.
 * Errors: GS_EINVAL, GS_ECAPACITY (workspace; a block table too short for
 * ctx_len + T_i tokens), GS_EDEVICE.
 */
gs_status gs_verify_batch(gs_ctx* ctx, const gs_kv_cache* kv, const gs_batch* batch,
                          const gs_accept_out* out, float* logits_out,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Debug aid.  gs_verify_batch trusts the device-resident parts of a batch (it cannot read them without
 * waiting for the GPU): cu_rows and ctx_len must equal their host copies, token ids must lie in [0, vocab) and
 * the block-table entries that cover ctx_len + T_i tokens must name pages of the cache.  gs_check_batch
 * verifies exactly that with one small kernel, SYNCHRONISES the stream, and returns GS_EINVAL with a
 * message naming the first violation (GS_OK if there is none).  Call it while bringing up a caller, not in
 * the serving loop.  workspace: dev, at least 4 * (2 N + 4) bytes.  Without the check, an out-of-range
 * token id is clamped into the vocabulary by the embedding gather and reported as accepted_len = -1 by the
 * accept stage when it is a draft token; a wrong page id or row offset is read as given.
 */
gs_status gs_check_batch(const gs_ctx* ctx, const gs_kv_cache* kv, const gs_batch* batch, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/* Host-only aid (no GPU call): the launch plan of the ragged attention (Section II-A-1's target forward over
 * N contexts of different length) that gs_verify_batch would use for a batch of this geometry.  n_kv_heads,
 * group = query heads per KV head; gamma_host, ctx_len_host: host, [n_servers].  Out: steps_per_split = the
 * longest run of 32-key steps one workgroup takes (a server with s steps is cut into ceil(s / steps_per_split)
 * splits of equal length up to one step); n_workgroups = (server, split, KV head) items of the launch;
 * busiest_cu_steps = the most steps any of the 256 compute units is dealt.  GS_EINVAL on negative entries. */
gs_status gs_plan_attention(int n_kv_heads, int group, int n_servers, const int* gamma_host,
                            const int* ctx_len_host, int* steps_per_split, long* n_workgroups,
                            long* busiest_cu_steps);

/* Test aid: with a non-NULL `trace` (dev, fp32 [(n_layers + 1)][R][d_model], caller-owned),
 * every later gs_verify_batch on this ctx also copies the residual stream entering each decoder
 * layer, and the final one that feeds the last norm, into it.  NULL switches it off. */
gs_status gs_trace_residual(gs_ctx* ctx, float* trace);

/* ------------------------------------------------------------------------- */
/* Measurement aid (not part of the method): when enabled, gs_verify_batch      */
/* brackets every stage with a pair of HIP events recorded on the caller's      */
/* stream.  gs_profile_read waits for the recorded events, returns per stage    */
/* the summed milliseconds and the number of bracketed launches since the last  */
/* read (arrays of GS_N_STAGES, host), and clears the record.                   */
/* ------------------------------------------------------------------------- */
/* Plain streaming read of `bytes` bytes at src (dev, 16-byte aligned): 16-byte non-temporal loads, four per lane
 * in flight, nothing else.  Timing it gives the practical ceiling of a read stream on the machine at hand,
 * against which bench.py states what the bandwidth-bound kernels reach.  sink: dev, at least 64 KiB (16384
 * words, practically never written). */
gs_status gs_probe_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream);

enum { GS_STAGE_GEMM = 0, GS_STAGE_ATTENTION = 1, GS_STAGE_GLUE = 2, GS_STAGE_ACCEPT = 3, GS_N_STAGES = 4 };
gs_status gs_profile_enable(gs_ctx* ctx, int on);
gs_status gs_profile_read(gs_ctx* ctx, double* stage_ms, long* stage_launches);

#ifdef __cplusplus
}
#endif
#endif /* GOODSPEED_H */
