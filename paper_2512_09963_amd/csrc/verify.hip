// gs_verify_batch: the decoder forward over the ragged speculative blocks followed by
// rejection-verification, enqueued on one stream without host synchronisation.
// Per layer: add+RMSNorm -> QKV projection -> rotary + KV append -> attention -> O projection
//            -> add+RMSNorm -> gate/up projection -> SwiGLU -> down projection.
// The residual stream and the logits are fp32; tensors fed to a projection and the KV
// pages are in the model's storage type.
#include <new>
#include <vector>
#include "common.h"

namespace gs {

int gemm_splits(int dtype, int M, int N, int K);
gs_status launch_pack_weight(const void* src, void* dst, int N, int K, hipStream_t stream);
size_t w4_packed_bytes(int N, int K);
gs_status launch_pack_weight_w4(const void* q, const void* scales, const void* zeros, void* packed, int N, int K,
                                hipStream_t stream);
gs_status launch_gemm(int dtype, const void* X, const void* W, float* P, int M, int N, int K, hipStream_t stream);
bool gate_up_fused(int dtype, int M, int F, int K);
gs_status launch_gemm_gate_up(const void* X, const void* W, void* act, int M, int F, int K, hipStream_t stream);
gs_status launch_embed(int dtype, const void* embed, const int* tokens, float* x, int n_rows, int d, int vocab,
                       hipStream_t);
gs_status launch_add_rmsnorm(int dtype, float* x, const float* partial, int n_splits, int n_rows, const float* w,
                             float eps, void* h, int d, hipStream_t stream);
gs_status launch_row_meta(const int* cu_rows, const int* ctx_len, int n_servers, int n_rows, const int* block_table,
                          int max_blocks, int page_size, int hd, float rope_theta, void* row_slot, void* rope,
                          hipStream_t stream);
gs_status launch_rope_append(int dtype, const float* qkv, int n_splits, int n_rows, const void* row_slot,
                             const void* rope, int page_size, int n_heads, int n_kv, int hd, void* q_out,
                             void* k_pages, void* v_pages, hipStream_t stream);
gs_status launch_swiglu(int dtype, const float* gu, int n_splits, int n_rows, int F, void* act, hipStream_t stream);
void attention_plan(int n_kv, int group, int max_block_tokens, int n_servers, const int* gamma_host,
                    const int* ctx_len_host, int* steps_per_split, int* max_splits);
long attention_busiest_cu(int n_kv, int n_servers, const int* gamma_host, const int* ctx_len_host, long t,
                          long* items_out);
size_t attention_workspace_floats(int n_rows, int n_heads, int hd, int max_splits);
gs_status launch_attention(int dtype, const void* q, const void* k_pages, const void* v_pages,
                           const int* block_table, int max_blocks, const int* cu_rows, const int* ctx_len,
                           int n_servers, int n_rows, int page_size, int n_heads, int n_kv, int hd,
                           int max_block_tokens, int steps_per_split, int max_splits, const void* row_info,
                           const int* work, int n_work, float* scratch, void* attn_out, hipStream_t stream);
size_t attention_work_ints(int capacity);
gs_status launch_attention_work(const int* cu_rows, const int* ctx_len, int n_servers, const int* block_table,
                                int max_blocks, int page_size, int steps_per_split, int capacity, int* work,
                                hipStream_t stream);
gs_status launch_accept(int n_servers, int n_rows, const int* cu_rows, int vocab, int elem, const void* target_logits,
                        const void* q_probs, const int* draft_tokens, const float* u_accept,
                        const float* u_resample, const gs_accept_out* out, void* workspace, hipStream_t stream,
                        const void* row_stats, int n_stat_blocks);
int gemm_stat_blocks(int dtype, int M, int N, int K);
gs_status launch_gemm_stats(const void* X, const void* W, float* Y, void* stats, int M, int N, int K,
                            hipStream_t stream);
size_t accept_workspace_bytes(int n_servers, int n_rows, int vocab);

}  // namespace gs

struct gs_ctx {
  gs_model_desc desc;
  const void* embed;
  const void* lm_head;
  const float* final_norm;
  std::vector<const void*> wqkv, wo, wgu, wd;
  std::vector<const float*> norm1, norm2;
  size_t elem;   // bytes per stored element
  float* residual_trace = nullptr;   // optional: copies of the residual stream, see gs_trace_residual
  // optional per-stage timing with HIP events on the caller's stream
  bool profile = false;
  std::vector<hipEvent_t> ev_start, ev_stop;
  std::vector<int> ev_stage;
  size_t ev_used = 0;
  // workspace planning: prefix maxima of the split-K partial sizes over the row count (filled on demand;
  // a context is used by one thread at a time)
  mutable std::vector<size_t> partial_prefix_max;
};

namespace {

struct Plan {
  float* x;
  void* h;
  float* partial;
  void* q;
  void* attn;
  void* act;
  float* attn_scratch;
  float* logits;
  int* draft_tokens;
  void* row_slot;   // [R] (page, slot of the row's own K/V, keys of its server, server)
  void* rope;       // [R][hd/2] (cos, sin)
  int* attn_work;   // the step's (server, split) work list of the attention kernel
  int attn_work_capacity;
  void* accept_ws;
  void* lm_stats;   // [R][column blocks] (max, sum exp) pairs from the LM-head projection's epilogue
  size_t bytes;
};

// Largest split-K partial buffer any projection needs for up to max_rows rows.  The split counts are not
// monotone in the row count, so the maximum runs over every row count; the prefix maxima are kept in the
// context (one entry per row count seen so far), which makes the per-call cost a table lookup.
size_t max_partial_floats(const gs_ctx* ctx, int max_rows) {
  const gs_model_desc& m = ctx->desc;
  const int qkv = (m.n_heads + 2 * m.n_kv_heads) * m.head_dim;
  const int hq = m.n_heads * m.head_dim;
  std::vector<size_t>& best = ctx->partial_prefix_max;
  if (best.empty()) best.push_back(0);
  for (int M = (int)best.size(); M <= max_rows; ++M) {
    size_t a = (size_t)gs::gemm_splits(m.dtype, M, qkv, m.d_model) * M * qkv;
    size_t b = (size_t)gs::gemm_splits(m.dtype, M, m.d_model, hq) * M * m.d_model;
    size_t c = (size_t)gs::gemm_splits(m.dtype, M, 2 * m.d_ffn, m.d_model) * M * 2 * m.d_ffn;
    size_t d = (size_t)gs::gemm_splits(m.dtype, M, m.d_model, m.d_ffn) * M * m.d_model;
    const int sv = gs::gemm_splits(m.dtype, M, m.vocab, m.d_model);
    size_t e = sv > 1 ? (size_t)sv * M * m.vocab : 0;   // LM head partials only when it is split
    best.push_back(std::max(std::max(best.back(), a), std::max(std::max(b, e), std::max(c, d))));
  }
  return best[max_rows];
}

Plan make_plan(const gs_ctx* ctx, int max_rows, int max_servers, int max_ctx, void* ws) {
  const gs_model_desc& m = ctx->desc;
  const size_t R = max_rows;
  const int hq = m.n_heads * m.head_dim;
  gs::Carver c(ws);
  Plan p;
  p.x = c.take<float>(R * m.d_model);
  p.h = c.take<char>(R * m.d_model * ctx->elem);
  p.partial = c.take<float>(max_partial_floats(ctx, max_rows));
  p.q = c.take<char>(R * hq * ctx->elem);
  p.attn = c.take<char>(R * hq * ctx->elem);
  p.act = c.take<char>(R * m.d_ffn * ctx->elem);
  // the planner never uses more than 32 splits per server and never fewer than 6 steps per split
  const int max_steps = (max_ctx + 31) / 32;
  const int max_splits = std::max(1, std::min(32, (max_steps + 5) / 6)) | 1;   // odd, like the planner's
  p.attn_scratch = c.take<float>(gs::attention_workspace_floats(max_rows, m.n_heads, m.head_dim, max_splits));
  p.attn_work_capacity = max_servers * max_splits;
  p.attn_work = c.take<int>(gs::attention_work_ints(p.attn_work_capacity));
  p.logits = c.take<float>(R * m.vocab);
  p.draft_tokens = c.take<int>(R);
  p.row_slot = c.take<int>(4 * R);
  p.rope = c.take<float>(R * m.head_dim);
  size_t acc = 0;
  for (int n = 1; n <= max_servers; ++n) acc = std::max(acc, gs::accept_workspace_bytes(n, max_rows, m.vocab));
  p.accept_ws = c.take<char>(acc);
  p.lm_stats = c.take<float>(2 * R * (size_t)(m.vocab / 64 + 1));     // at least 64 columns per block
  p.bytes = c.used();
  return p;
}

// y[i] = sum_s partial[s][i]
__global__ void sum_partials_kernel(const float* __restrict__ partial, int n_splits, size_t n, float* __restrict__ y) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
  for (int s = 0; s < n_splits; ++s) acc += partial[(size_t)s * n + i];
  y[i] = acc;
}

// draft_tokens[cu_rows[i] - i + j] = tokens[cu_rows[i] + 1 + j]: the drafts without the pending tokens
__global__ void gather_draft_tokens_kernel(const int* __restrict__ tokens, const int* __restrict__ cu_rows,
                                           int n_servers, int* __restrict__ draft_tokens) {
  const int srv = blockIdx.x;
  const int r0 = cu_rows[srv], gamma = cu_rows[srv + 1] - r0 - 1;
  for (int j = threadIdx.x; j < gamma; j += blockDim.x) draft_tokens[r0 - srv + j] = tokens[r0 + 1 + j];
}

// Measurement aid (gs_probe_stream_read): the plainest possible streaming read, 16-byte non-temporal loads,
// four per lane in flight, each workgroup folding its 16 KB pieces into one word.  What this kernel reaches is
// the practical ceiling of a read stream on the machine at hand.
typedef unsigned int probe_uint4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const probe_uint4* __restrict__ src, size_t n16,
                                                          unsigned* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 1024;
  unsigned acc = 0;
  for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
    probe_uint4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const size_t j = i + (size_t)k * 256;
      v[k] = j < n16 ? __builtin_nontemporal_load(src + j) : probe_uint4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  if (acc == 0x9e3779b9u) sink[blockIdx.x] = acc;      // (keeps the loads alive; practically never stores)
}

// Debug check of the device-resident descriptor (gs_check_batch).  One workgroup per server; the first
// inconsistency found is recorded as (kind, server, index, value) with a compare-and-swap on err[0].
enum { kBadCuRows = 1, kBadCtxLen = 2, kBadToken = 3, kBadPage = 4 };
__global__ __launch_bounds__(256) void check_batch_kernel(const int* __restrict__ cu_rows,
                                                          const int* __restrict__ ctx_len,
                                                          const int* __restrict__ tokens,
                                                          const int* __restrict__ block_table, int max_blocks,
                                                          const int* __restrict__ gamma_ref,     // device copies of the
                                                          const int* __restrict__ ctx_ref,       // host arrays
                                                          int vocab, int n_pages, int page_size, int* __restrict__ err) {
  const int srv = blockIdx.x;
  int row0 = 0;
  for (int i = 0; i < srv; ++i) row0 += gamma_ref[i] + 1;
  const int T = gamma_ref[srv] + 1;
  auto report = [&](int kind, int index, int value) {
    if (atomicCAS(&err[0], 0, kind) == 0) {
      err[1] = srv;
      err[2] = index;
      err[3] = value;
    }
  };
  if (threadIdx.x == 0) {
    if (cu_rows[srv] != row0) report(kBadCuRows, srv, cu_rows[srv]);
    else if (cu_rows[srv + 1] != row0 + T) report(kBadCuRows, srv + 1, cu_rows[srv + 1]);
    if (ctx_len[srv] != ctx_ref[srv]) report(kBadCtxLen, srv, ctx_len[srv]);
  }
  for (int j = threadIdx.x; j < T; j += blockDim.x) {
    const int t = tokens[row0 + j];
    if (t < 0 || t >= vocab) report(kBadToken, row0 + j, t);
  }
  const int n_blocks = (ctx_ref[srv] + T + page_size - 1) / page_size;     // <= max_blocks (checked on the host)
  for (int blk = threadIdx.x; blk < n_blocks; blk += blockDim.x) {
    const int pg = block_table[(size_t)srv * max_blocks + blk];
    if (pg < 0 || pg >= n_pages) report(kBadPage, blk, pg);
  }
}

}  // namespace

extern "C" gs_status gs_pack_weight(const void* w_rowmajor, void* w_packed, int n_out, int k_in, int dtype,
                                    void* hip_stream) {
  if (!w_rowmajor || !w_packed) return gs::fail(GS_EINVAL, "null argument");
  if (w_rowmajor == w_packed) return gs::fail(GS_EINVAL, "gs_pack_weight does not work in place");
  if (n_out <= 0 || k_in <= 0) return gs::fail(GS_EINVAL, "matrix dimensions must be positive");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (dtype == GS_F32) {
    GS_HIP_CHECK(hipMemcpyAsync(w_packed, w_rowmajor, sizeof(float) * (size_t)n_out * k_in, hipMemcpyDeviceToDevice,
                                stream));
    return GS_OK;
  }
  if (dtype != GS_BF16) return gs::fail(GS_EINVAL, "dtype must be GS_F32 or GS_BF16");
  if (n_out % 64 || k_in % 64) return gs::fail(GS_ESHAPE, "bf16 matrices need both dimensions to be multiples of 64");
  return gs::launch_pack_weight(w_rowmajor, w_packed, n_out, k_in, stream);
}

extern "C" size_t gs_w4_packed_bytes(int n_out, int k_in) {
  if (n_out <= 0 || k_in <= 0 || n_out % 64 || k_in % 128) return 0;
  return gs::w4_packed_bytes(n_out, k_in);
}

extern "C" gs_status gs_pack_weight_w4(const uint8_t* codes, const void* scales, const uint8_t* zeros, void* w_packed,
                                       int n_out, int k_in, void* hip_stream) {
  if (!codes || !scales || !zeros || !w_packed) return gs::fail(GS_EINVAL, "null argument");
  if (n_out <= 0 || k_in <= 0) return gs::fail(GS_EINVAL, "matrix dimensions must be positive");
  if (n_out % 64 || k_in % 128)
    return gs::fail(GS_ESHAPE, "4-bit matrices need n_out to be a multiple of 64 and k_in of 128");
  return gs::launch_pack_weight_w4(codes, scales, zeros, w_packed, n_out, k_in, static_cast<hipStream_t>(hip_stream));
}

extern "C" gs_status gs_create(const gs_model_desc* desc, const gs_weights* w, gs_ctx** out) {
  if (!desc || !w || !out) return gs::fail(GS_EINVAL, "null argument");
  const gs_model_desc& m = *desc;
  if (m.n_layers <= 0 || m.d_model <= 0 || m.n_heads <= 0 || m.n_kv_heads <= 0 || m.head_dim <= 0 || m.d_ffn <= 0 ||
      m.vocab <= 0)
    return gs::fail(GS_EINVAL, "model dimensions must be positive");
  if (m.d_model % 4) return gs::fail(GS_ESHAPE, "d_model must be a multiple of 4");
  if (m.dtype != GS_F32 && m.dtype != GS_BF16 && m.dtype != GS_W4)
    return gs::fail(GS_EINVAL, "dtype must be GS_F32, GS_BF16 or GS_W4");
  if (m.head_dim != 64 && m.head_dim != 128) return gs::fail(GS_ESHAPE, "head_dim must be 64 or 128");
  if (m.n_heads % m.n_kv_heads != 0) return gs::fail(GS_ESHAPE, "n_heads must be a multiple of n_kv_heads");
  const int group = m.n_heads / m.n_kv_heads;
  if (group != 1 && group != 2 && group != 4 && group != 8) return gs::fail(GS_ESHAPE, "GQA group must be 1, 2, 4 or 8");
  if (m.dtype == GS_BF16 || m.dtype == GS_W4) {
    const int qkv = (m.n_heads + 2 * m.n_kv_heads) * m.head_dim;
    if (m.d_model % 64 || m.d_ffn % 64 || qkv % 64 || m.vocab % 64)
      return gs::fail(GS_ESHAPE, "bf16 models need d_model, d_ffn, projection widths and vocab to be multiples of 64");
    if (m.dtype == GS_W4 && (m.d_model % 128 || m.d_ffn % 128 || (m.n_heads * m.head_dim) % 128))
      return gs::fail(GS_ESHAPE, "4-bit models need d_model, d_ffn and n_heads * head_dim to be multiples of 128");
  }
  if (!(m.rope_theta > 1.f) || !(m.rms_eps >= 0.f)) return gs::fail(GS_EINVAL, "rope_theta must exceed 1, rms_eps >= 0");
  if (!w->embed || !w->lm_head || !w->final_norm || !w->wqkv || !w->wo || !w->wgu || !w->wd || !w->norm1 || !w->norm2)
    return gs::fail(GS_EINVAL, "null weight table");
  for (int l = 0; l < m.n_layers; ++l)
    if (!w->wqkv[l] || !w->wo[l] || !w->wgu[l] || !w->wd[l] || !w->norm1[l] || !w->norm2[l])
      return gs::fail(GS_EINVAL, "null weight pointer in layer %d", l);
  gs_ctx* c = new (std::nothrow) gs_ctx;
  if (!c) return gs::fail(GS_EINVAL, "out of host memory");
  c->desc = m;
  c->embed = w->embed;
  c->lm_head = w->lm_head;
  c->final_norm = w->final_norm;
  c->wqkv.assign(w->wqkv, w->wqkv + m.n_layers);
  c->wo.assign(w->wo, w->wo + m.n_layers);
  c->wgu.assign(w->wgu, w->wgu + m.n_layers);
  c->wd.assign(w->wd, w->wd + m.n_layers);
  c->norm1.assign(w->norm1, w->norm1 + m.n_layers);
  c->norm2.assign(w->norm2, w->norm2 + m.n_layers);
  c->elem = m.dtype == GS_F32 ? 4 : 2;
  *out = c;
  return GS_OK;
}

extern "C" gs_status gs_destroy(gs_ctx* ctx) {
  if (ctx) {
    for (hipEvent_t e : ctx->ev_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_stop) (void)hipEventDestroy(e);
  }
  delete ctx;
  return GS_OK;
}

extern "C" gs_status gs_trace_residual(gs_ctx* ctx, float* trace) {
  if (!ctx) return gs::fail(GS_EINVAL, "null ctx");
  ctx->residual_trace = trace;
  return GS_OK;
}

extern "C" gs_status gs_profile_enable(gs_ctx* ctx, int on) {
  if (!ctx) return gs::fail(GS_EINVAL, "null ctx");
  ctx->profile = on != 0;
  ctx->ev_used = 0;
  return GS_OK;
}

extern "C" gs_status gs_profile_read(gs_ctx* ctx, double* stage_ms, long* stage_launches) {
  if (!ctx || !stage_ms || !stage_launches) return gs::fail(GS_EINVAL, "null argument");
  for (int s = 0; s < GS_N_STAGES; ++s) {
    stage_ms[s] = 0.0;
    stage_launches[s] = 0;
  }
  for (size_t i = 0; i < ctx->ev_used; ++i) {
    GS_HIP_CHECK(hipEventSynchronize(ctx->ev_stop[i]));
    float ms = 0.f;
    GS_HIP_CHECK(hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i]));
    stage_ms[ctx->ev_stage[i]] += ms;
    stage_launches[ctx->ev_stage[i]] += 1;
  }
  ctx->ev_used = 0;
  return GS_OK;
}

namespace {

// Brackets the launches of one stage with a pair of events when profiling is on.
struct StageTimer {
  gs_ctx* ctx;
  hipStream_t stream;
  bool active = false;
  StageTimer(gs_ctx* c, hipStream_t s) : ctx(c), stream(s) {}
  gs_status begin(int stage) {
    if (!ctx->profile) return GS_OK;
    if (ctx->ev_used == ctx->ev_start.size()) {
      hipEvent_t a, b;
      GS_HIP_CHECK(hipEventCreate(&a));
      GS_HIP_CHECK(hipEventCreate(&b));
      ctx->ev_start.push_back(a);
      ctx->ev_stop.push_back(b);
      ctx->ev_stage.push_back(0);
    }
    ctx->ev_stage[ctx->ev_used] = stage;
    GS_HIP_CHECK(hipEventRecord(ctx->ev_start[ctx->ev_used], stream));
    active = true;
    return GS_OK;
  }
  gs_status end() {
    if (!active) return GS_OK;
    GS_HIP_CHECK(hipEventRecord(ctx->ev_stop[ctx->ev_used], stream));
    ctx->ev_used += 1;
    active = false;
    return GS_OK;
  }
};

}  // namespace

extern "C" size_t gs_workspace_bytes(const gs_ctx* ctx, int max_rows, int max_servers, int max_ctx) {
  if (!ctx || max_rows <= 0 || max_servers <= 0 || max_ctx <= 0) return 0;
  return make_plan(ctx, max_rows, max_servers, max_ctx, nullptr).bytes;
}

extern "C" gs_status gs_verify_batch(gs_ctx* ctx, const gs_kv_cache* kv, const gs_batch* b, const gs_accept_out* out,
                                     float* logits_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!ctx || !kv || !b || !workspace) return gs::fail(GS_EINVAL, "null argument");
  const gs_model_desc& m = ctx->desc;
  const int n = b->n_servers;
  if (n <= 0) return gs::fail(GS_EINVAL, "n_servers must be positive");
  if (!b->gamma_host || !b->ctx_len_host || !b->cu_rows || !b->ctx_len || !b->tokens || !b->block_table)
    return gs::fail(GS_EINVAL, "null batch field");
  if (!kv->k_pages || !kv->v_pages || kv->page_size <= 0 || kv->n_pages <= 0 || b->max_blocks <= 0)
    return gs::fail(GS_EINVAL, "invalid KV cache descriptor");
  const int act = m.dtype == GS_W4 ? GS_BF16 : m.dtype;     // storage type of activations, KV pages, embedding
  if (act == GS_BF16 && kv->page_size % 16 != 0)
    return gs::fail(GS_ESHAPE, "bf16 attention needs a page size that is a multiple of 16");
  long R = 0, G = 0;
  int max_t = 0, max_ctx = 0;
  for (int i = 0; i < n; ++i) {
    const int g = b->gamma_host[i], L = b->ctx_len_host[i];
    if (g < 0 || L < 0) return gs::fail(GS_EINVAL, "server %d: gamma = %d, ctx_len = %d", i, g, L);
    const long need = ((long)L + g + 1 + kv->page_size - 1) / kv->page_size;
    if (need > b->max_blocks)
      return gs::fail(GS_ECAPACITY, "server %d needs %ld KV blocks for %d + %d tokens, block table has %d", i, need, L,
                      g + 1, b->max_blocks);
    R += g + 1;
    G += g;
    max_t = std::max(max_t, g + 1);
    max_ctx = std::max(max_ctx, L + g + 1);
  }
  if (R > (1 << 20)) return gs::fail(GS_EINVAL, "too many rows");
  const bool do_accept = b->q_probs != nullptr;
  if (do_accept) {
    if (!out || !out->accepted_len || !out->next_token || !out->accept_stat)
      return gs::fail(GS_EINVAL, "accept outputs are required when q_probs is given");
    if (!b->u_resample || (G > 0 && !b->u_accept)) return gs::fail(GS_EINVAL, "uniforms are required");
  }
  const Plan p = make_plan(ctx, (int)R, n, max_ctx, workspace);      // carves addresses only
  if (workspace_bytes < p.bytes)
    return gs::fail(GS_ECAPACITY, "workspace of %zu bytes, this batch needs %zu", workspace_bytes, p.bytes);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int rows = (int)R, d = m.d_model, hq = m.n_heads * m.head_dim, qkv = (m.n_heads + 2 * m.n_kv_heads) * m.head_dim;
  const int F = m.d_ffn;
  const size_t layer_stride = (size_t)kv->n_pages * m.n_kv_heads * kv->page_size * m.head_dim * ctx->elem;
  int attn_sps = 1, attn_splits = 1;
  gs::attention_plan(m.n_kv_heads, m.n_heads / m.n_kv_heads, max_t, n, b->gamma_host, b->ctx_len_host, &attn_sps,
                     &attn_splits);
  gs_status st;
#define GS_TRY(call)          \
  do {                        \
    st = (call);              \
    if (st != GS_OK) return st; \
  } while (0)

  int attn_items = 0;      // (server, split) pairs with keys: the length of the attention work list
  for (int i = 0; i < n; ++i)
    attn_items += ((b->ctx_len_host[i] + b->gamma_host[i] + 1 + 31) / 32 + attn_sps - 1) / attn_sps;
  if (attn_items > p.attn_work_capacity) return gs::fail(GS_ECAPACITY, "attention work list overflow");

  StageTimer timer(ctx, stream);
#define GS_STAGE(stage, call)   \
  do {                          \
    GS_TRY(timer.begin(stage)); \
    GS_TRY(call);               \
    GS_TRY(timer.end());        \
  } while (0)
  GS_STAGE(GS_STAGE_GLUE, gs::launch_embed(act, ctx->embed, b->tokens, p.x, rows, d, m.vocab, stream));
  GS_STAGE(GS_STAGE_GLUE, gs::launch_row_meta(b->cu_rows, b->ctx_len, n, rows, b->block_table, b->max_blocks, kv->page_size,
                                              m.head_dim, m.rope_theta, p.row_slot, p.rope, stream));
  if (act == GS_BF16)
    GS_STAGE(GS_STAGE_GLUE, gs::launch_attention_work(b->cu_rows, b->ctx_len, n, b->block_table, b->max_blocks,
                                                      kv->page_size, attn_sps, p.attn_work_capacity, p.attn_work, stream));
  const float* pending = nullptr;   // split-K partials of the projection whose result is still to be added to x
  int pending_splits = 0;
  for (int l = 0; l < m.n_layers; ++l) {
    GS_STAGE(GS_STAGE_GLUE, gs::launch_add_rmsnorm(act, p.x, pending, pending_splits, rows, ctx->norm1[l], m.rms_eps, p.h, d, stream));
    if (ctx->residual_trace)   // residual stream entering layer l (complete once the pending partials are added)
      GS_HIP_CHECK(hipMemcpyAsync(ctx->residual_trace + (size_t)l * rows * d, p.x, sizeof(float) * rows * d,
                                  hipMemcpyDeviceToDevice, stream));
    GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm(m.dtype, p.h, ctx->wqkv[l], p.partial, rows, qkv, d, stream));
    char* kl = static_cast<char*>(kv->k_pages) + layer_stride * l;
    char* vl = static_cast<char*>(kv->v_pages) + layer_stride * l;
    GS_STAGE(GS_STAGE_GLUE, gs::launch_rope_append(act, p.partial, gs::gemm_splits(m.dtype, rows, qkv, d), rows, p.row_slot,
                                  p.rope, kv->page_size, m.n_heads, m.n_kv_heads, m.head_dim, p.q, kl, vl, stream));
    GS_STAGE(GS_STAGE_ATTENTION, gs::launch_attention(act, p.q, kl, vl, b->block_table, b->max_blocks, b->cu_rows, b->ctx_len, n, rows,
                                kv->page_size, m.n_heads, m.n_kv_heads, m.head_dim, max_t, attn_sps, attn_splits,
                                p.row_slot, p.attn_work, attn_items, p.attn_scratch, p.attn, stream));
    GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm(m.dtype, p.attn, ctx->wo[l], p.partial, rows, d, hq, stream));
    GS_STAGE(GS_STAGE_GLUE, gs::launch_add_rmsnorm(act, p.x, p.partial, gs::gemm_splits(m.dtype, rows, d, hq), rows,
                                                   ctx->norm2[l], m.rms_eps, p.h, d, stream));
    if (gs::gate_up_fused(m.dtype, rows, F, d)) {
      GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm_gate_up(p.h, ctx->wgu[l], p.act, rows, F, d, stream));
    } else {
      GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm(m.dtype, p.h, ctx->wgu[l], p.partial, rows, 2 * F, d, stream));
      GS_STAGE(GS_STAGE_GLUE, gs::launch_swiglu(act, p.partial, gs::gemm_splits(m.dtype, rows, 2 * F, d), rows, F, p.act, stream));
    }
    GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm(m.dtype, p.act, ctx->wd[l], p.partial, rows, d, F, stream));
    pending = p.partial;
    pending_splits = gs::gemm_splits(m.dtype, rows, d, F);
  }
  GS_STAGE(GS_STAGE_GLUE, gs::launch_add_rmsnorm(act, p.x, pending, pending_splits, rows, ctx->final_norm, m.rms_eps, p.h, d, stream));
  if (ctx->residual_trace)
    GS_HIP_CHECK(hipMemcpyAsync(ctx->residual_trace + (size_t)m.n_layers * rows * d, p.x, sizeof(float) * rows * d,
                                hipMemcpyDeviceToDevice, stream));
  float* logits = logits_out ? logits_out : p.logits;
  const int lm_splits = gs::gemm_splits(m.dtype, rows, m.vocab, d);
  // Where the LM-head projection runs as one bf16 launch, its epilogue also leaves the softmax statistics of
  // every row per column block, and the accept stage does not read the logits again for them.
  const int stat_blocks = do_accept ? gs::gemm_stat_blocks(m.dtype, rows, m.vocab, d) : 0;
  if (stat_blocks > 0) {
    GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm_stats(p.h, ctx->lm_head, logits, p.lm_stats, rows, m.vocab, d, stream));
  } else if (lm_splits == 1) {
    GS_STAGE(GS_STAGE_GEMM, gs::launch_gemm(m.dtype, p.h, ctx->lm_head, logits, rows, m.vocab, d, stream));
  } else {   // small vocabularies only: the partials fit the projection scratch
    GS_TRY(gs::launch_gemm(m.dtype, p.h, ctx->lm_head, p.partial, rows, m.vocab, d, stream));
    const size_t n_out = (size_t)rows * m.vocab;
    sum_partials_kernel<<<(unsigned)((n_out + 255) / 256), 256, 0, stream>>>(p.partial, lm_splits, n_out, logits);
    GS_LAUNCH_CHECK("sum_partials");
  }
  if (do_accept) {
    if (G > 0) {
      gather_draft_tokens_kernel<<<n, 64, 0, stream>>>(b->tokens, b->cu_rows, n, p.draft_tokens);
      GS_LAUNCH_CHECK("gather_draft_tokens");
    }
    GS_STAGE(GS_STAGE_ACCEPT, gs::launch_accept(n, rows, b->cu_rows, m.vocab, GS_F32, logits, b->q_probs, p.draft_tokens,
                                                b->u_accept, b->u_resample, out, p.accept_ws, stream,
                                                stat_blocks > 0 ? p.lm_stats : nullptr, stat_blocks));
  }
#undef GS_STAGE
#undef GS_TRY
  return GS_OK;
}

extern "C" gs_status gs_check_batch(const gs_ctx* ctx, const gs_kv_cache* kv, const gs_batch* b, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  if (!ctx || !kv || !b || !workspace) return gs::fail(GS_EINVAL, "null argument");
  const int n = b->n_servers;
  if (n <= 0) return gs::fail(GS_EINVAL, "n_servers must be positive");
  if (!b->gamma_host || !b->ctx_len_host || !b->cu_rows || !b->ctx_len || !b->tokens || !b->block_table)
    return gs::fail(GS_EINVAL, "null batch field");
  if (kv->page_size <= 0 || kv->n_pages <= 0 || b->max_blocks <= 0) return gs::fail(GS_EINVAL, "invalid KV cache descriptor");
  for (int i = 0; i < n; ++i) {
    const int g = b->gamma_host[i], L = b->ctx_len_host[i];
    if (g < 0 || L < 0) return gs::fail(GS_EINVAL, "server %d: gamma = %d, ctx_len = %d", i, g, L);
    if (((long)L + g + 1 + kv->page_size - 1) / kv->page_size > b->max_blocks)
      return gs::fail(GS_ECAPACITY, "server %d needs more KV blocks than the block table has", i);
  }
  const size_t need = sizeof(int) * (2 * (size_t)n + 4);
  if (workspace_bytes < need) return gs::fail(GS_ECAPACITY, "workspace of %zu bytes, the check needs %zu", workspace_bytes, need);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int* dev = static_cast<int*>(workspace);          // [4] error record, [n] gamma, [n] ctx_len
  const int zero[4] = {0, 0, 0, 0};
  GS_HIP_CHECK(hipMemcpyAsync(dev, zero, sizeof(zero), hipMemcpyHostToDevice, stream));
  GS_HIP_CHECK(hipMemcpyAsync(dev + 4, b->gamma_host, sizeof(int) * n, hipMemcpyHostToDevice, stream));
  GS_HIP_CHECK(hipMemcpyAsync(dev + 4 + n, b->ctx_len_host, sizeof(int) * n, hipMemcpyHostToDevice, stream));
  check_batch_kernel<<<n, 256, 0, stream>>>(b->cu_rows, b->ctx_len, b->tokens, b->block_table, b->max_blocks, dev + 4,
                                            dev + 4 + n, ctx->desc.vocab, kv->n_pages, kv->page_size, dev);
  GS_LAUNCH_CHECK("check_batch");
  int err[4] = {0, 0, 0, 0};
  GS_HIP_CHECK(hipMemcpyAsync(err, dev, sizeof(err), hipMemcpyDeviceToHost, stream));
  GS_HIP_CHECK(hipStreamSynchronize(stream));
  switch (err[0]) {
    case 0: return GS_OK;
    case kBadCuRows: return gs::fail(GS_EINVAL, "device cu_rows[%d] = %d does not match gamma_host", err[2], err[3]);
    case kBadCtxLen: return gs::fail(GS_EINVAL, "device ctx_len[%d] = %d does not match ctx_len_host", err[2], err[3]);
    case kBadToken: return gs::fail(GS_EINVAL, "tokens[%d] = %d of server %d is outside the vocabulary", err[2], err[3], err[1]);
    default: return gs::fail(GS_EINVAL, "block_table[%d][%d] = %d is not a page of the cache", err[1], err[2], err[3]);
  }
}

extern "C" gs_status gs_plan_attention(int n_kv_heads, int group, int n_servers, const int* gamma_host,
                                       const int* ctx_len_host, int* steps_per_split, long* n_workgroups,
                                       long* busiest_cu_steps) {
  if (n_kv_heads <= 0 || group <= 0 || n_servers <= 0 || !gamma_host || !ctx_len_host || !steps_per_split)
    return gs::fail(GS_EINVAL, "gs_plan_attention: bad argument");
  int max_t = 0;
  for (int i = 0; i < n_servers; ++i) {
    if (gamma_host[i] < 0 || ctx_len_host[i] < 0)
      return gs::fail(GS_EINVAL, "server %d: gamma = %d, ctx_len = %d", i, gamma_host[i], ctx_len_host[i]);
    max_t = std::max(max_t, gamma_host[i] + 1);
  }
  int sps = 1, splits = 1;
  gs::attention_plan(n_kv_heads, group, max_t, n_servers, gamma_host, ctx_len_host, &sps, &splits);
  long items = 0;
  const long busiest = gs::attention_busiest_cu(n_kv_heads, n_servers, gamma_host, ctx_len_host, sps, &items);
  *steps_per_split = sps;
  if (n_workgroups) *n_workgroups = items;
  if (busiest_cu_steps) *busiest_cu_steps = busiest;
  return GS_OK;
}

extern "C" gs_status gs_probe_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || bytes < 16) return gs::fail(GS_EINVAL, "null argument or fewer than 16 bytes");
  if (reinterpret_cast<uintptr_t>(src) % 16) return gs::fail(GS_EINVAL, "source must be 16-byte aligned");
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n16 + 1023) / 1024, 16384);
  stream_read_kernel<<<grid, 256, 0, static_cast<hipStream_t>(hip_stream)>>>(
      static_cast<const probe_uint4*>(src), n16, static_cast<unsigned*>(sink));
  GS_LAUNCH_CHECK("stream_read");
  return GS_OK;
}
