// Ragged, paged-KV, grouped-query causal attention for the speculative blocks.
//
// Row j of server i (position L_i + j) attends to keys 0 .. L_i + j of that server; the
// cache holds L_i keys and the block's own T_i keys were appended just before.  Page layouts:
//   K pages [page][H_kv][slot][hd]   (key-major: a key's head vector is contiguous)
//   V pages [page][H_kv][hd][slot]   (transposed: the slots of one channel are contiguous)
//
// bf16 path (MFMA): one workgroup per (server, KV head, KV split), one wave per 16 of the
// T_i * G query rows that share the KV head (token-major, head-minor), so each K/V byte leaves
// HBM once per workgroup; K/V stream through a two-stage LDS buffer filled by direct global->LDS loads.
//   S^T = K Q^T : A operand = 16 keys x 32 channels, B operand = Q rows (kept in registers).
//   The result layout puts a query row in lane%16 and 4 consecutive keys in each lane, which
//   is already the A-operand layout of the second product, so P never leaves registers:
//   O = P V     : B operand = V^T, 4 keys of one channel per lane, read from the verbatim copy
//                 of the transposed V page.
// The online-softmax state (running max, running sum) lives per query row in lane%16.  The
// number of KV splits of a server follows its own context length (a fixed number of 32-key steps
// per workgroup), so ragged batches stay balanced.  Partial results of the splits are merged by
// attn_combine_kernel.
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
// bf16 MFMA path.  grid (max_splits, H_kv, N), NW waves per workgroup.
//
// A workgroup owns steps [split * steps_per_split, ...) of one (server, KV head); a step is 32
// keys = two 16-key tiles = 16 KB of K and V at hd 128.  K/V go from global memory straight into
// a two-stage LDS buffer with direct global->LDS loads (no register staging).  A stage has four
// parts, K and V of either tile; part p is loaded by wave p % NW (waves 0..3 when NW > 4), whose
// HD/32 load instructions of 1 KB each share one scalar base address.  One barrier per step both
// publishes the stage that has landed and frees the stage that is refilled next.  K is placed in
// LDS in MFMA-fragment order (lane l of fragment (tile, ks) finds its 16 bytes at fragment * 1 KB
// + l * 16); V pages are copied verbatim ([channel][16 slots] per tile), which the second product
// reads as 8-byte pieces without bank conflicts.
// Wave w computes query tile w (16 of the T_i * G rows that share the KV head, token-major,
// head-minor): S^T = K Q^T, online softmax per query row (lane%16), O += P V with P as a two-term
// bf16 sum.  partial_o [R][H][max_splits][HD] fp32, partial_ml [R][H][max_splits][2]; splits
// beyond a server's own count are never written and never read.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void wait_all_vector_loads() {
  // s_waitcnt vmcnt(0) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8;
  // the other two fields at their maximum mean "do not wait")
  __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));
}

// Reductions over the four 16-lane rows of a wave (lanes c, c+16, c+32, c+48), result in every lane.
// The two swap instructions exchange rows between a register pair; fed the same value twice they
// return (rows 0,0,2,2 | rows 1,1,3,3) and then (low half twice | high half twice).
__device__ __forceinline__ float rows_max(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <int HD, int G, int NW>
__global__ __launch_bounds__(64 * NW) void attn_ring_kernel(const bf16_t* __restrict__ q,
                                                            const bf16_t* __restrict__ k_pages,
                                                            const bf16_t* __restrict__ v_pages,
                                                            const int* __restrict__ block_table, int max_blocks,
                                                            const int* __restrict__ cu_rows,
                                                            const int* __restrict__ ctx_len, int page_size,
                                                            int n_heads, int n_kv, int steps_per_split,
                                                            int max_splits, int q_row_offset,
                                                            float* __restrict__ partial_o,
                                                            float* __restrict__ partial_ml) {
  constexpr int KS = HD / 32;            // k steps of the first product = 1 KB loads per part
  constexpr int DT = HD / 16;            // channel tiles of the second product
  constexpr int PART = HD * 32;          // bytes of K (or V) of one 16-key tile
  constexpr int STAGE = 4 * PART;        // K tile 0, K tile 1, V tile 0, V tile 1
  __shared__ __attribute__((aligned(16))) unsigned char ring[2 * STAGE];

  const int split = blockIdx.x, kh = blockIdx.y, srv = blockIdx.z;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // provably uniform: scalar page lookups
  const int g = lane >> 4, c = lane & 15;
  const int row0 = cu_rows[srv];
  const int T = cu_rows[srv + 1] - row0;
  const int L = ctx_len[srv];
  const int n_keys = L + T;
  const int n_steps_all = (n_keys + 31) >> 5;
  const int step_begin = split * steps_per_split;
  if (step_begin >= n_steps_all) return;                                // this server has fewer splits
  const int n = min(steps_per_split, n_steps_all - step_begin);        // steps of this workgroup
  const int* bt = block_table + (size_t)srv * max_blocks;
  const bool page_pow2 = (page_size & (page_size - 1)) == 0;
  const int page_shift = 31 - __builtin_clz(page_size);
  const int last_tile_key = ((n_keys - 1) >> 4) << 4;                   // first key of the last existing tile

  // ---- this wave's query tile
  const int tile_row0 = q_row_offset + wave * 16;
  const int rows = T * G - tile_row0;                                   // valid rows of the tile (<= 0: none)
  const bool has_rows = rows > 0;
  const int my_lr = tile_row0 + c;
  const bool my_ok = c < rows;
  const int my_j = my_ok ? my_lr / G : 0, my_hg = my_ok ? my_lr - my_j * G : 0;
  const int limit = my_ok ? L + my_j : -1;                              // last key this lane's row may see
  const int j_max = min(T - 1, (tile_row0 + 15) / G);
  const int my_step_end = has_rows ? ((L + j_max) >> 5) + 1 : 0;       // causal: no key beyond L + j_max
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
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

  // ---- page-table lookup of the two 16-key tiles of a step (scalar loads; done one iteration before
  // the stage is issued, so that no load instruction waits for it)
  auto lookup = [&](int step, int (&page)[2], int (&slot0)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key0 = min(step * 32 + t * 16, last_tile_key);   // a tile past the end re-reads the last one
      // (page sizes are powers of two in practice: shifts instead of a scalar division sequence)
      const int blk = page_pow2 ? key0 >> page_shift : key0 / page_size;
      page[t] = bt[blk];
      slot0[t] = key0 - blk * page_size;
    }
  };
  // ---- stage loader.  Part p (0, 1: K of tile 0, 1; 2, 3: V of tile 0, 1) belongs to one wave; its
  // address is a wave-uniform base (scalar registers) plus a per-lane byte offset that never changes:
  //   K: lane (c, g) of fragment ks holds key slot0 + c, channels ks*32 + g*8 ..
  //   V: 16-byte piece ch*64 + lane of the [HD][16 slots] tile is channel ch*32 + lane/2, half lane%2
  const unsigned k_lane_off = (unsigned)(c * HD + g * 8) * 2u;
  const unsigned v_lane_off = (unsigned)((lane >> 1) * page_size + (lane & 1) * 8) * 2u;
  const char* k_bytes = reinterpret_cast<const char*>(k_pages);
  const char* v_bytes = reinterpret_cast<const char*>(v_pages);
  auto issue = [&](int slot, const int (&page)[2], const int (&slot0)[2]) {
    unsigned char* stage = ring + slot * STAGE;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if (wave != (NW > 4 ? p : p % NW)) continue;           // uniform branch
      const int t = p & 1;
      const size_t head = (size_t)page[t] * n_kv + kh;
      if (p < 2) {
        const char* src = k_bytes + (head * page_size + slot0[t]) * (HD * 2) + k_lane_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          __builtin_amdgcn_global_load_lds(src + ks * 64,
                                           (__attribute__((address_space(3))) void*)(stage + p * PART + ks * 1024),
                                           16, 0, 0);
      } else {
        const char* src = v_bytes + (head * HD * page_size + slot0[t]) * 2 + v_lane_off;
        const size_t stride = (size_t)64 * page_size;        // 32 channels
#pragma unroll
        for (int ch = 0; ch < KS; ++ch)
          __builtin_amdgcn_global_load_lds(src + ch * stride,
                                           (__attribute__((address_space(3))) void*)(stage + p * PART + ch * 1024),
                                           16, 0, 0);
      }
    }
  };

  int pg_next[2], sl_next[2];
  lookup(step_begin, pg_next, sl_next);
  issue(0, pg_next, sl_next);
  if (1 < n) lookup(step_begin + 1, pg_next, sl_next);

  for (int s = 0; s < n; ++s) {
    const int step = step_begin + s;
    wait_all_vector_loads();     // this wave's parts of stage s have landed
    __syncthreads();             // stage s complete for all waves; the other stage is free
    if (s + 1 < n) {
      issue((s + 1) & 1, pg_next, sl_next);
      if (s + 2 < n) lookup(step + 2, pg_next, sl_next);     // for the next iteration's issue
    }
    if (step >= my_step_end) continue;

    const unsigned char* base = ring + (s & 1) * STAGE;
    // first product S^T = K Q^T for the two 16-key tiles
    bf16x8_t kf[2 * KS];
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i) kf[i] = *reinterpret_cast<const bf16x8_t*>(base + i * 1024 + lane * 16);
    floatx4_t sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      floatx4_t acc = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t * KS + ks], qf[ks], acc, 0, 0, 0);
      sacc[t] = acc;
    }
    // online softmax: the query row is lane%16, its 32 keys are spread over the 4 lane groups
    float p[8];
    float corr;
    if (step * 32 + 31 <= L) {
      // every key of the step is visible to every valid row: no masks
      float mx = fmaxf(fmaxf(fmaxf(sacc[0][0], sacc[0][1]), fmaxf(sacc[0][2], sacc[0][3])),
                       fmaxf(fmaxf(sacc[1][0], sacc[1][1]), fmaxf(sacc[1][2], sacc[1][3])));
      mx = rows_max(mx);
      const float m_new = fmaxf(m_run, mx * scale_log2);
      corr = __builtin_amdgcn_exp2f(m_run - m_new);
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(fmaf(sacc[e >> 2][e & 3], scale_log2, -m_new));
        sum += p[e];
      }
      l_run = l_run * corr + rows_sum(sum);
      m_run = m_new;
    } else {
      float sv[8];
      float mx = kNegBig;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = step * 32 + (e >> 2) * 16 + g * 4 + (e & 3);
        sv[e] = key <= limit ? sacc[e >> 2][e & 3] * scale_log2 : kNegBig;
        mx = fmaxf(mx, sv[e]);
      }
      mx = rows_max(mx);
      const float m_new = fmaxf(m_run, mx);
      corr = __builtin_amdgcn_exp2f(m_run - m_new);
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = (sv[e] > kNegBig) ? __builtin_amdgcn_exp2f(sv[e] - m_new) : 0.f;
        sum += p[e];
      }
      l_run = l_run * corr + rows_sum(sum);
      m_run = m_new;
    }
    // P enters the second product as a sum of two bf16 terms (value and rounding remainder), so
    // the product sees 16 mantissa bits of P instead of 8
    uint4 packed, packed_lo;
    packed.x = pack_bf16x2(p[0], p[1]);
    packed.y = pack_bf16x2(p[2], p[3]);
    packed.z = pack_bf16x2(p[4], p[5]);
    packed.w = pack_bf16x2(p[6], p[7]);
    packed_lo.x = pack_bf16x2(p[0] - __uint_as_float(packed.x << 16), p[1] - __uint_as_float(packed.x & 0xffff0000u));
    packed_lo.y = pack_bf16x2(p[2] - __uint_as_float(packed.y << 16), p[3] - __uint_as_float(packed.y & 0xffff0000u));
    packed_lo.z = pack_bf16x2(p[4] - __uint_as_float(packed.z << 16), p[5] - __uint_as_float(packed.z & 0xffff0000u));
    packed_lo.w = pack_bf16x2(p[6] - __uint_as_float(packed.w << 16), p[7] - __uint_as_float(packed.w & 0xffff0000u));
    const bf16x8_t pf = *reinterpret_cast<const bf16x8_t*>(&packed);
    const bf16x8_t pf_lo = *reinterpret_cast<const bf16x8_t*>(&packed_lo);
    // the output accumulators hold query rows g*4 + i; their rescale factor sits in lane g*4 + i.
    // Once the running maxima have settled every factor is exactly 1 and the rescale is skipped.
    if (__any(corr != 1.0f)) {
      float f[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) f[i] = __shfl(corr, g * 4 + i);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) oacc[dt][i] *= f[i];
    }
    // second product O += P V
    const unsigned char* vb = base + 2 * PART + (c * 16 + g * 4) * 2;
    uint2 v0[DT], v1[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      v0[dt] = *reinterpret_cast<const uint2*>(vb + dt * 512);
      v1[dt] = *reinterpret_cast<const uint2*>(vb + PART + dt * 512);
    }
    if (step * 32 + 32 > n_keys) {
      // keys past the end of the sequence inside the last page hold stale data, so their V is
      // zeroed (P is 0 there, but 0 * NaN would not be)
      const int kb0 = step * 32 + g * 4, kb1 = kb0 + 16;
      uint2 keep0, keep1;
      keep0.x = (kb0 + 0 < n_keys ? 0x0000ffffu : 0u) | (kb0 + 1 < n_keys ? 0xffff0000u : 0u);
      keep0.y = (kb0 + 2 < n_keys ? 0x0000ffffu : 0u) | (kb0 + 3 < n_keys ? 0xffff0000u : 0u);
      keep1.x = (kb1 + 0 < n_keys ? 0x0000ffffu : 0u) | (kb1 + 1 < n_keys ? 0xffff0000u : 0u);
      keep1.y = (kb1 + 2 < n_keys ? 0x0000ffffu : 0u) | (kb1 + 3 < n_keys ? 0xffff0000u : 0u);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        v0[dt].x &= keep0.x; v0[dt].y &= keep0.y;
        v1[dt].x &= keep1.x; v1[dt].y &= keep1.y;
      }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const uint4 vv = make_uint4(v0[dt].x, v0[dt].y, v1[dt].x, v1[dt].y);
      const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(&vv);
      oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf, vf, oacc[dt], 0, 0, 0);
      oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_lo, vf, oacc[dt], 0, 0, 0);
    }
  }

  // ---- this split's partial result for the tile's rows
  if (!has_rows) return;
  if (g == 0 && my_ok) {
    const size_t idx = ((size_t)(row0 + my_j) * n_heads + kh * G + my_hg) * max_splits + split;
    partial_ml[idx * 2 + 0] = m_run;
    partial_ml[idx * 2 + 1] = l_run;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int lrow = g * 4 + i;
    if (lrow < rows) {
      const int lr = tile_row0 + lrow;
      const int j = lr / G, hg = lr - j * G;
      float* dst = partial_o + (((size_t)(row0 + j) * n_heads + kh * G + hg) * max_splits + split) * HD;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) dst[dt * 16 + c] = oacc[dt][i];
    }
  }
}

// attn_out[r][h*HD + d] = sum_s o_s * 2^(m_s - M) / sum_s l_s * 2^(m_s - M) over the row's server's own
// splits.  grid (R*H), block HD.
template <int HD>
__global__ void attn_combine_kernel(const float* __restrict__ partial_o, const float* __restrict__ partial_ml,
                                    int max_splits, int steps_per_split, const int* __restrict__ cu_rows,
                                    const int* __restrict__ ctx_len, int n_servers, int n_heads,
                                    bf16_t* __restrict__ attn_out) {
  const size_t rh = blockIdx.x;
  const int d = threadIdx.x;
  const int r = (int)(rh / n_heads);
  const int srv = server_of_row(cu_rows, n_servers, r);
  const int n_keys = ctx_len[srv] + (cu_rows[srv + 1] - cu_rows[srv]);
  const int n_splits = (((n_keys + 31) >> 5) + steps_per_split - 1) / steps_per_split;
  float M = kNegBig;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, partial_ml[(rh * max_splits + s) * 2]);
  float Lsum = 0.f, acc = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float f = exp2f(partial_ml[(rh * max_splits + s) * 2] - M);
    Lsum += partial_ml[(rh * max_splits + s) * 2 + 1] * f;
    acc += partial_o[(rh * max_splits + s) * HD + d] * f;
  }
  attn_out[rh * HD + d] = float_to_bf16(acc / Lsum);
}

}  // namespace

// KV steps (32 keys) per workgroup, and the resulting largest split count, for a batch with
// total_steps steps summed over servers, max_steps on its longest server and query tiles of at most
// max_block_tokens rows per server.  Workgroups take equally many steps, so a launch runs in rounds of
// as many workgroups as fit the chip at once; enough rounds (4) keep the last, partly filled one cheap,
// while a floor on the steps per workgroup bounds what the partial results cost.
void attention_plan(int n_kv, int group, int max_block_tokens, long total_steps, int max_steps, int* steps_per_split,
                    int* max_splits) {
  const int tiles = ceil_div(max_block_tokens * group, 16);
  const int waves = tiles < 8 ? (tiles > 0 ? tiles : 1) : 8;
  const int wgs_per_cu = 16 / waves < 5 ? 16 / waves : 5;      // 16 waves by registers, 5 workgroups by LDS
  const long slots = 256L * wgs_per_cu;
  long sps = (total_steps * n_kv + 4 * slots - 1) / (4 * slots);
  if (sps < 6) sps = 6;
  const long lo = (max_steps + 31) / 32;                        // at most 32 splits per server
  if (sps < lo) sps = lo;
  if (sps > max_steps) sps = max_steps > 0 ? max_steps : 1;
  *steps_per_split = (int)sps;
  *max_splits = (int)((max_steps + sps - 1) / sps);
}

size_t attention_workspace_floats(int n_rows, int n_heads, int hd, int max_splits) {
  return (size_t)n_rows * n_heads * max_splits * (hd + 2);
}

template <int HD, int G>
static gs_status launch_mfma_g(const bf16_t* q, const bf16_t* k_pages, const bf16_t* v_pages, const int* block_table,
                               int max_blocks, const int* cu_rows, const int* ctx_len, int n_servers, int page_size,
                               int n_heads, int n_kv, int max_block_tokens, int steps_per_split, int max_splits,
                               float* po, float* pml, hipStream_t stream) {
  const int tiles = ceil_div(max_block_tokens * G, 16);
  dim3 grid(max_splits, n_kv, n_servers);
  for (int t0 = 0; t0 < tiles; t0 += 8) {      // at most 8 query tiles (waves) per workgroup
    const int waves = tiles - t0 < 8 ? tiles - t0 : 8;
#define GS_RING(NW_)                                                                                              \
  attn_ring_kernel<HD, G, NW_><<<grid, 64 * NW_, 0, stream>>>(q, k_pages, v_pages, block_table, max_blocks,    \
                                                                 cu_rows, ctx_len, page_size, n_heads, n_kv,      \
                                                                 steps_per_split, max_splits, t0 * 16, po, pml)
    switch (waves) {
      case 1: GS_RING(1); break;
      case 2: GS_RING(2); break;
      case 3: GS_RING(3); break;
      case 4: GS_RING(4); break;
      case 5: GS_RING(5); break;
      case 6: GS_RING(6); break;
      case 7: GS_RING(7); break;
      default: GS_RING(8); break;
    }
#undef GS_RING
    GS_LAUNCH_CHECK("attn_ring");
  }
  return GS_OK;
}

// attn_out [R][H*hd] (storage type).  scratch: attention_workspace_floats floats (bf16 path only).
gs_status launch_attention(int dtype, const void* q, const void* k_pages, const void* v_pages,
                           const int* block_table, int max_blocks, const int* cu_rows, const int* ctx_len,
                           int n_servers, int n_rows, int page_size, int n_heads, int n_kv, int hd,
                           int max_block_tokens, int steps_per_split, int max_splits, float* scratch, void* attn_out,
                           hipStream_t stream) {
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
  float* pml = scratch + (size_t)n_rows * n_heads * max_splits * hd;
  const int G = n_heads / n_kv;
  gs_status st = GS_OK;
#define GS_ATTN_CASE(HD_, G_)                                                                                     \
  if (hd == HD_ && G == G_)                                                                                       \
    st = launch_mfma_g<HD_, G_>(qb, kb, vb, block_table, max_blocks, cu_rows, ctx_len, n_servers, page_size,     \
                                n_heads, n_kv, max_block_tokens, steps_per_split, max_splits, po, pml, stream);
  GS_ATTN_CASE(128, 1) GS_ATTN_CASE(128, 2) GS_ATTN_CASE(128, 4) GS_ATTN_CASE(128, 8)
  GS_ATTN_CASE(64, 1) GS_ATTN_CASE(64, 2) GS_ATTN_CASE(64, 4) GS_ATTN_CASE(64, 8)
#undef GS_ATTN_CASE
  if (st != GS_OK) return st;
  if (hd == 128)
    attn_combine_kernel<128><<<n_rows * n_heads, 128, 0, stream>>>(po, pml, max_splits, steps_per_split, cu_rows,
                                                                   ctx_len, n_servers, n_heads,
                                                                   static_cast<bf16_t*>(attn_out));
  else
    attn_combine_kernel<64><<<n_rows * n_heads, 64, 0, stream>>>(po, pml, max_splits, steps_per_split, cu_rows,
                                                                 ctx_len, n_servers, n_heads,
                                                                 static_cast<bf16_t*>(attn_out));
  GS_LAUNCH_CHECK("attn_combine");
  return GS_OK;
}

}  // namespace gs
