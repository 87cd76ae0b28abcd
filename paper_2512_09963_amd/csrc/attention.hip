// Ragged, paged-KV, grouped-query causal attention for the speculative blocks.
//
// Row j of server i (position L_i + j) attends to keys 0 .. L_i + j of that server; the
// cache holds L_i keys and the block's own T_i keys were appended just before.  Page layouts:
//   K pages [page][H_kv][slot][hd]   (key-major: a key's head vector is contiguous)
//   V pages [page][H_kv][hd][slot]   (transposed: the slots of one channel are contiguous)
//
// bf16 path (MFMA, no LDS staging of K/V): one workgroup per (server, KV head, KV split), one
// wave per 16 of the T_i * G query rows that share the KV head (token-major, head-minor), so
// each K/V byte leaves HBM once per workgroup and the other waves hit it in cache.
//   S^T = K Q^T : A operand = 16 keys x 32 channels read straight from the K page (16 bytes
//                 per lane), B operand = Q rows (kept in registers for the whole kernel).
//   The result layout puts a query row in lane%16 and 4 consecutive keys in each lane, which
//   is already the A-operand layout of the second product, so P never leaves registers:
//   O = P V     : B operand = V^T read straight from the transposed V page (8 bytes = 4
//                 keys of one channel per lane).
// The online-softmax state (running max, running sum) lives per query row in lane%16.
// Partial results of the splits are merged by combine_kernel.
//
// fp32 path: one wave per (row, head), lanes over keys, online softmax per lane.
#include "common.h"
#include "device_types.h"
#include <cmath>

namespace gs {
namespace {

constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ int server_of_row(const int* __restrict__ cu_rows, int n_servers, int r) {
  int lo = 0, hi = n_servers;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu_rows[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------------------------------
// fp32 / generic path.  grid (R, H), block 64.  Writes attn_out [R][H*hd] in storage type T.
// ------------------------------------------------------------------------------------------
template <typename T, int HD>
__global__ __launch_bounds__(64) void attn_rowwise_kernel(const T* __restrict__ q, const T* __restrict__ k_pages,
                                                          const T* __restrict__ v_pages,
                                                          const int* __restrict__ block_table, int max_blocks,
                                                          const int* __restrict__ cu_rows,
                                                          const int* __restrict__ ctx_len, int n_servers,
                                                          int page_size, int n_heads, int n_kv,
                                                          T* __restrict__ attn_out) {
  const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int srv = server_of_row(cu_rows, n_servers, r);
  const int n_keys = ctx_len[srv] + (r - cu_rows[srv]) + 1;
  const int kh = h / (n_heads / n_kv);
  __shared__ float qs[HD];
  __shared__ float red_m[64], red_l[64];
  __shared__ float red_o[64][HD + 1];
  for (int d = lane; d < HD; d += 64) qs[d] = Storage<T>::load(q + ((size_t)r * n_heads + h) * HD + d);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)HD);
  float m = kNegBig, l = 0.f;
  float o[HD];
#pragma unroll
  for (int d = 0; d < HD; ++d) o[d] = 0.f;
  for (int key = lane; key < n_keys; key += 64) {
    const int page = block_table[(size_t)srv * max_blocks + key / page_size];
    const int slot = key % page_size;
    const T* kp = k_pages + (((size_t)page * n_kv + kh) * page_size + slot) * HD;
    float s = 0.f;
#pragma unroll
    for (int d = 0; d < HD; ++d) s = fmaf(qs[d], Storage<T>::load(kp + d), s);
    s *= scale;
    const float m_new = fmaxf(m, s);
    const float corr = expf(m - m_new), p = expf(s - m_new);
    l = l * corr + p;
    const T* vp = v_pages + ((size_t)page * n_kv + kh) * HD * page_size + slot;
#pragma unroll
    for (int d = 0; d < HD; ++d) o[d] = o[d] * corr + p * Storage<T>::load(vp + (size_t)d * page_size);
    m = m_new;
  }
  red_m[lane] = m;
  red_l[lane] = l;
#pragma unroll
  for (int d = 0; d < HD; ++d) red_o[lane][d] = o[d];
  __syncthreads();
  float M = kNegBig;
  for (int t = 0; t < 64; ++t) M = fmaxf(M, red_m[t]);
  float L = 0.f;
  for (int t = 0; t < 64; ++t) L += red_l[t] * expf(red_m[t] - M);
  for (int d = lane; d < HD; d += 64) {
    float acc = 0.f;
    for (int t = 0; t < 64; ++t) acc += red_o[t][d] * expf(red_m[t] - M);
    Storage<T>::store(attn_out + ((size_t)r * n_heads + h) * HD + d, acc / L);
  }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA path.  grid (n_splits, H_kv, N); one wave per 16-row query tile (blockDim = 64 *
// tiles); the waves of a workgroup read the same K/V (served by L1/L2 after the first) and
// never synchronise.  partial_o [R][H][n_splits][HD] fp32, partial_ml [R][H][n_splits][2].
// ------------------------------------------------------------------------------------------
template <int HD, int G>
__global__ __launch_bounds__(512) void attn_mfma_kernel(const bf16_t* __restrict__ q,
                                                         const bf16_t* __restrict__ k_pages,
                                                         const bf16_t* __restrict__ v_pages,
                                                         const int* __restrict__ block_table, int max_blocks,
                                                         const int* __restrict__ cu_rows,
                                                         const int* __restrict__ ctx_len, int page_size, int n_heads,
                                                         int n_kv, int n_splits, int q_row_offset,
                                                         float* __restrict__ partial_o,
                                                         float* __restrict__ partial_ml) {
  constexpr int KS = HD / 32;   // k steps of the first product
  constexpr int DT = HD / 16;   // channel tiles of the second product
  const int split = blockIdx.x, kh = blockIdx.y, srv = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, c = lane & 15;
  const int row0 = cu_rows[srv];
  const int T = cu_rows[srv + 1] - row0;
  const int L = ctx_len[srv];
  const int n_keys = L + T;
  const int tile_row0 = q_row_offset + wave * 16;   // first query row (token-major, head-minor) of this wave
  const int rows = T * G - tile_row0;                // valid rows in this tile (may exceed 16)
  if (rows <= 0) return;
  const int* bt = block_table + (size_t)srv * max_blocks;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);   // scores in log2 units

  // Q fragment (B operand of the first product): query row = c, channels ks*32 + g*8 ..
  const int my_lr = tile_row0 + c;
  const bool my_ok = c < rows;
  const int my_j = my_ok ? my_lr / G : 0, my_hg = my_ok ? my_lr - my_j * G : 0;
  const int limit = my_ok ? L + my_j : -1;           // last key this lane's query row may see
  bf16x8_t qf[KS];
  {
    const bf16_t* src = q + ((size_t)(row0 + my_j) * n_heads + kh * G + my_hg) * HD + g * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (my_ok) v = *reinterpret_cast<const uint4*>(src + ks * 32);
      qf[ks] = *reinterpret_cast<const bf16x8_t*>(&v);
    }
  }
  float m_run = kNegBig, l_run = 0.f;
  floatx4_t oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) oacc[dt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  const int n_steps = (n_keys + 31) >> 5;
  const int per_split = (n_steps + n_splits - 1) / n_splits;
  const int step_begin = split * per_split;
  // a tile whose rows all belong to block tokens < j_max sees no key beyond L + j_max
  const int j_max = min(T - 1, (tile_row0 + 15) / G);
  const int step_end = min(min(n_steps, step_begin + per_split), ((L + j_max) >> 5) + 1);
  const int last_tile_key = ((n_keys - 1) >> 4) << 4;   // first key of the last 16-key tile that exists

  auto tile_base = [&](int step, int t, int& page, int& slot0) {
    const int key0 = min(step * 32 + t * 16, last_tile_key);   // a tile past the end re-reads the last one (masked)
    page = bt[key0 / page_size];
    slot0 = key0 % page_size;
  };
  auto load_k = [&](int page, int slot0, uint4 (&kraw)[KS]) {
    const bf16_t* kp = k_pages + (((size_t)page * n_kv + kh) * page_size + slot0 + c) * HD + g * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kraw[ks] = *reinterpret_cast<const uint4*>(kp + ks * 32);
  };
  int page_cur[2] = {0, 0}, slot_cur[2] = {0, 0};
  uint4 k_cur[2][KS];
  if (step_begin < step_end) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      tile_base(step_begin, t, page_cur[t], slot_cur[t]);
      load_k(page_cur[t], slot_cur[t], k_cur[t]);
    }
  }

  for (int step = step_begin; step < step_end; ++step) {
    uint2 vraw[2][DT];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const bf16_t* vp = v_pages + (((size_t)page_cur[t] * n_kv + kh) * HD + c) * page_size + slot_cur[t] + g * 4;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) vraw[t][dt] = *reinterpret_cast<const uint2*>(vp + (size_t)dt * 16 * page_size);
    }
    // first product S^T = K Q^T for the two 16-key tiles, then fetch the next step's K
    floatx4_t sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx4_t acc = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(&k_cur[t][ks]), qf[ks], acc, 0,
                                                      0, 0);
      sacc[t] = acc;
    }
    if (step + 1 < step_end) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        tile_base(step + 1, t, page_cur[t], slot_cur[t]);
        load_k(page_cur[t], slot_cur[t], k_cur[t]);
      }
    }
    // keys past the end of the sequence inside the last page hold stale data: zero their V
    if (step * 32 + 32 > n_keys) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int kbase = step * 32 + t * 16 + g * 4;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uint2 v = vraw[t][dt];
          if (kbase + 0 >= n_keys) v.x &= 0xffff0000u;
          if (kbase + 1 >= n_keys) v.x &= 0x0000ffffu;
          if (kbase + 2 >= n_keys) v.y &= 0xffff0000u;
          if (kbase + 3 >= n_keys) v.y &= 0x0000ffffu;
          vraw[t][dt] = v;
        }
      }
    }
    // mask and online softmax: the query row is lane%16, its 32 keys are spread over the 4 lane groups
    float sv[8];
    float mx = kNegBig;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = step * 32 + t * 16 + g * 4 + i;
        const float v = (key <= limit) ? sacc[t][i] * scale_log2 : kNegBig;
        sv[t * 4 + i] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float corr = exp2f(m_run - m_new);
    float sum = 0.f;
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = (sv[e] > kNegBig) ? exp2f(sv[e] - m_new) : 0.f;
      sum += p[e];
    }
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    l_run = l_run * corr + sum;
    m_run = m_new;
    // P enters the second product as a sum of two bf16 terms (value and rounding remainder), so
    // the product sees 16 mantissa bits of P instead of 8
    float plo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) plo[e] = p[e] - bf16_to_float(float_to_bf16(p[e]));
    uint4 packed, packed_lo;
    packed.x = pack_bf16x2(p[0], p[1]);
    packed.y = pack_bf16x2(p[2], p[3]);
    packed.z = pack_bf16x2(p[4], p[5]);
    packed.w = pack_bf16x2(p[6], p[7]);
    packed_lo.x = pack_bf16x2(plo[0], plo[1]);
    packed_lo.y = pack_bf16x2(plo[2], plo[3]);
    packed_lo.z = pack_bf16x2(plo[4], plo[5]);
    packed_lo.w = pack_bf16x2(plo[6], plo[7]);
    const bf16x8_t pf = *reinterpret_cast<const bf16x8_t*>(&packed);
    const bf16x8_t pf_lo = *reinterpret_cast<const bf16x8_t*>(&packed_lo);
    // the output accumulators hold query rows g*4 + i; their rescale factor sits in lane g*4 + i
    float f[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = __shfl(corr, g * 4 + i);
    // second product O += P V
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int i = 0; i < 4; ++i) oacc[dt][i] *= f[i];
      uint4 vv = make_uint4(vraw[0][dt].x, vraw[0][dt].y, vraw[1][dt].x, vraw[1][dt].y);
      const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(&vv);
      oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf, vf, oacc[dt], 0, 0, 0);
      oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_lo, vf, oacc[dt], 0, 0, 0);
    }
  }

  // this split's partial result for the tile's rows
  if (g == 0 && my_ok) {
    const size_t idx = ((size_t)(row0 + my_j) * n_heads + kh * G + my_hg) * n_splits + split;
    partial_ml[idx * 2 + 0] = m_run;
    partial_ml[idx * 2 + 1] = l_run;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int lrow = g * 4 + i;
    if (lrow < rows) {
      const int lr = tile_row0 + lrow;
      const int j = lr / G, hg = lr - j * G;
      float* dst = partial_o + (((size_t)(row0 + j) * n_heads + kh * G + hg) * n_splits + split) * HD;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) dst[dt * 16 + c] = oacc[dt][i];
    }
  }
}

// attn_out[r][h*HD + d] = sum_s o_s * 2^(m_s - M) / sum_s l_s * 2^(m_s - M).  grid (R*H), block HD.
template <int HD>
__global__ void attn_combine_kernel(const float* __restrict__ partial_o, const float* __restrict__ partial_ml,
                                    int n_splits, bf16_t* __restrict__ attn_out) {
  const size_t rh = blockIdx.x;
  const int d = threadIdx.x;
  float M = kNegBig;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, partial_ml[(rh * n_splits + s) * 2]);
  float L = 0.f, acc = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float f = exp2f(partial_ml[(rh * n_splits + s) * 2] - M);
    L += partial_ml[(rh * n_splits + s) * 2 + 1] * f;
    acc += partial_o[(rh * n_splits + s) * HD + d] * f;
  }
  attn_out[rh * HD + d] = float_to_bf16(acc / L);
}

}  // namespace

// Splits of the KV range per (server, KV head) so that the grid fills the chip.
int attention_splits(int n_servers, int n_kv, int max_ctx) {
  const int pairs = n_servers * n_kv;
  int want = ceil_div(512, pairs > 0 ? pairs : 1);
  int max_s = ceil_div(max_ctx, 256);      // at least 256 keys (8 steps, 2 per wave) per split
  int s = want < max_s ? want : max_s;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  return s;
}

size_t attention_workspace_floats(int n_rows, int n_heads, int hd, int n_splits) {
  return (size_t)n_rows * n_heads * n_splits * (hd + 2);
}

template <int HD, int G>
static gs_status launch_mfma_g(const bf16_t* q, const bf16_t* k_pages, const bf16_t* v_pages, const int* block_table,
                               int max_blocks, const int* cu_rows, const int* ctx_len, int n_servers, int page_size,
                               int n_heads, int n_kv, int max_block_tokens, int n_splits, float* po, float* pml,
                               hipStream_t stream) {
  const int tiles = ceil_div(max_block_tokens * G, 16);
  dim3 grid(n_splits, n_kv, n_servers);
  for (int t0 = 0; t0 < tiles; t0 += 8) {      // at most 8 query tiles (waves) per workgroup
    const int waves = tiles - t0 < 8 ? tiles - t0 : 8;
    attn_mfma_kernel<HD, G><<<grid, 64 * waves, 0, stream>>>(q, k_pages, v_pages, block_table, max_blocks, cu_rows,
                                                             ctx_len, page_size, n_heads, n_kv, n_splits, t0 * 16, po,
                                                             pml);
    GS_LAUNCH_CHECK("attn_mfma");
  }
  return GS_OK;
}

// attn_out [R][H*hd] (storage type).  scratch: attention_workspace_floats floats (bf16 path only).
gs_status launch_attention(int dtype, const void* q, const void* k_pages, const void* v_pages,
                           const int* block_table, int max_blocks, const int* cu_rows, const int* ctx_len,
                           int n_servers, int n_rows, int page_size, int n_heads, int n_kv, int hd,
                           int max_block_tokens, int n_splits, float* scratch, void* attn_out, hipStream_t stream) {
  if (dtype == GS_F32) {
    dim3 grid(n_rows, n_heads);
    const float* qf = static_cast<const float*>(q);
    const float* kf = static_cast<const float*>(k_pages);
    const float* vf = static_cast<const float*>(v_pages);
    float* of = static_cast<float*>(attn_out);
    if (hd == 64)
      attn_rowwise_kernel<float, 64><<<grid, 64, 0, stream>>>(qf, kf, vf, block_table, max_blocks, cu_rows, ctx_len,
                                                             n_servers, page_size, n_heads, n_kv, of);
    else
      attn_rowwise_kernel<float, 128><<<grid, 64, 0, stream>>>(qf, kf, vf, block_table, max_blocks, cu_rows, ctx_len,
                                                              n_servers, page_size, n_heads, n_kv, of);
    GS_LAUNCH_CHECK("attn_rowwise");
    return GS_OK;
  }
  const bf16_t* qb = static_cast<const bf16_t*>(q);
  const bf16_t* kb = static_cast<const bf16_t*>(k_pages);
  const bf16_t* vb = static_cast<const bf16_t*>(v_pages);
  float* po = scratch;
  float* pml = scratch + (size_t)n_rows * n_heads * n_splits * hd;
  const int G = n_heads / n_kv;
  gs_status st = GS_OK;
#define GS_ATTN_CASE(HD_, G_)                                                                                     \
  if (hd == HD_ && G == G_)                                                                                       \
    st = launch_mfma_g<HD_, G_>(qb, kb, vb, block_table, max_blocks, cu_rows, ctx_len, n_servers, page_size,     \
                                n_heads, n_kv, max_block_tokens, n_splits, po, pml, stream);
  GS_ATTN_CASE(128, 1) GS_ATTN_CASE(128, 2) GS_ATTN_CASE(128, 4) GS_ATTN_CASE(128, 8)
  GS_ATTN_CASE(64, 1) GS_ATTN_CASE(64, 2) GS_ATTN_CASE(64, 4) GS_ATTN_CASE(64, 8)
#undef GS_ATTN_CASE
  if (st != GS_OK) return st;
  if (hd == 128)
    attn_combine_kernel<128><<<n_rows * n_heads, 128, 0, stream>>>(po, pml, n_splits, static_cast<bf16_t*>(attn_out));
  else
    attn_combine_kernel<64><<<n_rows * n_heads, 64, 0, stream>>>(po, pml, n_splits, static_cast<bf16_t*>(attn_out));
  GS_LAUNCH_CHECK("attn_combine");
  return GS_OK;
}

}  // namespace gs
