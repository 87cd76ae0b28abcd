// Ragged, paged-KV, grouped-query causal attention for the speculative blocks.
//
// Row j of server i (position L_i + j) attends to keys 0 .. L_i + j of that server; the
// cache holds L_i keys and the block's own T_i keys were appended just before.  Page layouts:
//   K pages [page][H_kv][slot][hd]   (key-major: a key's head vector is contiguous)
//   V pages [page][H_kv][hd][slot]   (transposed: the slots of one channel are contiguous)
//
// bf16 path (MFMA): one workgroup per (server, KV head, KV split), one wave per 32 of the
// T_i * G query rows that share the KV head (token-major, head-minor), so each K/V byte leaves
// HBM once per workgroup; K/V stream through a two-stage LDS buffer filled by direct global->LDS
// loads.  The first product is computed transposed (S^T = K Q^T), which leaves a query's scores in
// the registers of two lanes, in exactly the order the second product (O^T += V^T P) wants its P
// operand, so P never leaves registers and neither product needs an LDS transpose.  The number of
// KV splits of a server follows its own context length (a fixed number of 32-key steps per
// workgroup), so ragged batches stay balanced.  Partial results of the splits are merged by
// attn_combine_kernel.
//
// fp32 path: one wave per (row, head), lanes over keys, online softmax per lane.
#include "common.h"
#include "device_types.h"
#include <algorithm>
#include <cmath>
#include <limits>

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
// bf16 MFMA path.  1-D grid over the (work list entry, KV head) items (item_of_workgroup), NW waves per workgroup.
//
// A workgroup owns one split of one (server, KV head): a server's steps are dealt evenly to its
// ceil(steps / steps_per_split) splits; a step is 32
// keys = two 16-key tiles = 16 KB of K and V at hd 128.  K/V go from global memory straight into
// a two-stage LDS buffer with direct global->LDS loads (no register staging).  A stage has four
// parts, K and V of either tile; part p is loaded by wave p % NW (waves 0..3 when NW > 4), whose
// HD/32 load instructions of 1 KB each share one scalar base address.  One barrier per step both
// publishes the stage that has landed and frees the stage that is refilled next.  (Deeper buffers
// were measured, with and without the arithmetic: no gain.)  K is placed in LDS so that lane (g, c) of fragment (tile, ks) holds
// key c, channels 32 ks + 8 g .. at fragment * 1 KB + lane * 16; V pages are copied verbatim
// ([channel][16 slots] per tile).
// Wave w computes query rows 32 w .. 32 w + 31 of the T_i * G rows that share the KV head (token-major,
// head-minor); both products use the 32x32x16 MFMA (twice the issue rate of the 16x16x32 one on this
// chip):
//   S^T (32 keys x 32 queries) = K Q^T : A = K, lane l holds key l%32 (tile l%32/16 of the step),
//       channels 16 kk + 8 (l/32) .. of k step kk; B = Q^T, lane l holds query row l%32, same channels.
//       Result register v of lane l is key 8 (v/4) + 4 (l/32) + v%4 of query l%32.
//   O^T (hd x 32 queries) += V^T P : B = P straight from the result registers of the first product:
//       k slot i of k step kk' (16 keys) is register 8 kk' + i, i.e. key 16 kk' + 8 (i/4) + 4 (l/32) + i%4;
//       A = V^T in the same key order: channel 32 dt + l%32, two 8-byte runs of the transposed page.
// A query row lives in lanes l and l + 32: one lane swap finishes its max and its sum, and the
// accumulator rescale is a per-lane multiply.  P enters the second product as a two-term bf16 sum.
// partial_o [R][H][max_splits][HD] fp32, partial_ml [R][H][max_splits][2]; splits beyond a server's own
// count are never written and never read.
// ------------------------------------------------------------------------------------------
// Work list of a step: one entry per (server, split) that has keys, so that the grid holds no workgroup
// that starts only to find its split empty (ragged contexts), and an entry carries all a workgroup needs
// before its first load, the pages of its first step included: start-up costs one dependent read instead
// of three.  list = int header[8] (header[0] = number of entries), then the entries.
struct AttnWork {
  int srv, split, row0, n_tokens, ctx, page0, page1, pad;
};
static_assert(sizeof(AttnWork) == 32, "entries are read as one 32-byte load");

// One workgroup.  The entries are written in the order of decreasing split length (counting sort over the
// lengths, which the splits of a server take only two of), because the hardware deals the workgroups of a
// launch to the compute units round robin by their linear index and a compute unit's finishing time follows
// the sum of the steps it was dealt: attn_kernel walks the sorted list in a serpentine (item_of_workgroup),
// so every compute unit gets one long, one medium, ... split instead of whatever the server order brings.
// Splits longer than kSortBins - 1 steps are not sorted (server order).  Entries beyond the capacity are
// dropped (cannot happen when the host's copy of the batch geometry matches the device's).
constexpr int kSortBins = 1024;

__global__ __launch_bounds__(256) void attn_work_kernel(const int* __restrict__ cu_rows,
                                                        const int* __restrict__ ctx_len, int n_servers,
                                                        const int* __restrict__ block_table, int max_blocks,
                                                        int page_size, int steps_per_split, int capacity,
                                                        int* __restrict__ list) {
  __shared__ int bin[kSortBins];      // entries per split length, then the first position of a length
  __shared__ int scan[256];
  __shared__ int total_sh;
  const int tid = threadIdx.x;
  const bool sorted = steps_per_split < kSortBins;
  for (int b = tid; b < kSortBins; b += 256) bin[b] = 0;
  if (tid == 0) total_sh = 0;
  __syncthreads();
  // a server's splits: count of them, `rem` of base + 1 steps followed by count - rem of base steps
  auto shape = [&](int srv, int& row0, int& T, int& L, int& count, int& base, int& rem) {
    row0 = cu_rows[srv];
    T = cu_rows[srv + 1] - row0;
    L = ctx_len[srv];
    const int steps = (L + T + 31) >> 5;
    count = (steps + steps_per_split - 1) / steps_per_split;
    base = count > 0 ? steps / count : 0;
    rem = steps - base * count;
  };
  if (sorted) {
    for (int srv = tid; srv < n_servers; srv += 256) {
      int row0, T, L, count, base, rem;
      shape(srv, row0, T, L, count, base, rem);
      if (rem > 0) atomicAdd(&bin[base + 1], rem);
      if (count - rem > 0) atomicAdd(&bin[base], count - rem);
    }
    __syncthreads();
    // first position of each length, longest first: lane t owns bins kSortBins - 1 - 4 t down to ... - 3
    int mine[4], sum = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      mine[k] = bin[kSortBins - 1 - (4 * tid + k)];
      sum += mine[k];
    }
    scan[tid] = sum;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
      const int v = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += v;
      __syncthreads();
    }
    int at = scan[tid] - sum;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      bin[kSortBins - 1 - (4 * tid + k)] = at;
      at += mine[k];
    }
    if (tid == 255) total_sh = scan[255];
    __syncthreads();
  }
  AttnWork* entries = reinterpret_cast<AttnWork*>(list + 8);
  for (int c0 = 0; c0 < n_servers; c0 += 256) {
    const int srv = c0 + tid;
    int row0 = 0, T = 0, L = 0, count = 0, base = 0, rem = 0;
    if (srv < n_servers) shape(srv, row0, T, L, count, base, rem);
    int first_long = 0, first_short = 0;      // positions of the server's base + 1 and base step splits
    if (sorted) {
      if (rem > 0) first_long = atomicAdd(&bin[base + 1], rem);
      if (count - rem > 0) first_short = atomicAdd(&bin[base], count - rem);
    } else {
      scan[tid] = count;
      __syncthreads();
      for (int off = 1; off < 256; off <<= 1) {
        const int v = tid >= off ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
      }
      first_long = total_sh + scan[tid] - count;
      first_short = first_long + rem;
      __syncthreads();
      if (tid == 255) total_sh += scan[255];
      __syncthreads();
    }
    const int last_tile_key = ((L + T - 1) >> 4) << 4;
    for (int sp = 0; sp < count; ++sp) {
      const int pos = sp < rem ? first_long + sp : first_short + (sp - rem);
      if (pos >= capacity) continue;
      AttnWork w;
      w.srv = srv; w.split = sp; w.row0 = row0; w.n_tokens = T; w.ctx = L; w.pad = 0;
      // (the server's steps are dealt evenly to its splits, as in attn_kernel)
      const int key0 = min((sp * base + min(sp, rem)) * 32, last_tile_key), key1 = min(key0 + 16, last_tile_key);
      w.page0 = block_table[(size_t)srv * max_blocks + key0 / page_size];
      w.page1 = block_table[(size_t)srv * max_blocks + key1 / page_size];
      entries[pos] = w;
    }
  }
  __syncthreads();
  if (tid == 0) list[0] = min(total_sh, capacity);
}

// Which (work list entry, KV head) a workgroup of the 1-D attention grid takes: the items, entry-major (the KV
// heads of an entry are neighbours, so they go to the 8 XCDs), in rounds of one item per compute unit, the
// rounds alternately forwards and backwards, counted from the last one, which is taken forwards (it may be
// partial, and the grid has no workgroup beyond the items: padding workgroups in the middle of a launch that
// fills every slot kept the last workgroups of one XCD waiting for a slot).  The list being sorted by
// length, the sums of the items that meet on a compute unit are nearly equal, and the compute units that get
// one item more get the shortest ones on top of the smaller sums.
constexpr int kComputeUnits = 256;
__device__ __forceinline__ void item_of_workgroup(int wg, int n_items, int n_kv, int& entry, int& kh) {
  const int rounds = (n_items + kComputeUnits - 1) / kComputeUnits;
  const int round = wg / kComputeUnits, c = wg - round * kComputeUnits;
  const bool backwards = ((rounds - 1 - round) & 1) != 0;      // (a backward round is never the partial one)
  const int item = round * kComputeUnits + (backwards ? kComputeUnits - 1 - c : c);
  entry = item / n_kv;
  kh = item - entry * n_kv;
}

// cache policy of the K/V loads (the builtin's last argument; bit 1 = non-temporal): a step reads its keys and
// values once, so they should not displace the partial results and the block tables in L2 (measured: config 4
// 3.4 instead of 3.6 ms of attention per step, config 3 unchanged)
constexpr int kKvLoadPolicy = 2;

__device__ __forceinline__ void wait_all_vector_loads() {
  // s_waitcnt vmcnt(0) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8;
  // the other two fields at their maximum mean "do not wait")
  __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));
}

typedef unsigned int uintx2_t __attribute__((ext_vector_type(2)));

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;

__device__ __forceinline__ float halves_max(float x) {
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// (164 vector registers: three waves per SIMD, i.e. up to four 3-wave workgroups per CU, which hides a
// workgroup's start-up and barrier stalls behind the others' loads)
template <int HD, int G, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW == 1 ? 2 : 3))) void attn_kernel(const bf16_t* __restrict__ q,
                                                         const bf16_t* __restrict__ k_pages,
                                                         const bf16_t* __restrict__ v_pages,
                                                         const int* __restrict__ block_table, int max_blocks,
                                                         const int* __restrict__ work, int n_work, int page_size,
                                                         int n_heads, int n_kv, int steps_per_split,
                                                         int max_splits, int q_row_offset,
                                                         float* __restrict__ partial_o,
                                                         float* __restrict__ partial_ml) {
  constexpr int KS = HD / 32;            // 1 KB loads per part
  constexpr int KK = HD / 16;            // k steps of the first product
  constexpr int DT = HD / 32;            // 32-channel tiles of the second product
  constexpr int PART = HD * 32;          // bytes of K (or V) of one 16-key tile
  constexpr int STAGE = 4 * PART;        // K tile 0, K tile 1, V tile 0, V tile 1
  __shared__ __attribute__((aligned(16))) unsigned char ring[2 * STAGE];

  int entry, kh;
  item_of_workgroup(blockIdx.x, n_work * n_kv, n_kv, entry, kh);
  // (n_work never exceeds the list's capacity, so the entry may be read before the device's count is known)
  const AttnWork wk = *reinterpret_cast<const AttnWork*>(work + 8 + 8 * entry);
  if (entry >= work[0]) return;
  const int srv = wk.srv, split = wk.split, row0 = wk.row0, T = wk.n_tokens, L = wk.ctx;
  const int first_pages[2] = {wk.page0, wk.page1};
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = lane >> 5, c32 = lane & 31;
  const int g = lane >> 4, c = lane & 15;            // loader roles
  const int n_keys = L + T;
  const int n_steps_all = (n_keys + 31) >> 5;
  // the server's steps are dealt evenly to its ceil(steps / steps_per_split) splits (sizes differ by at most
  // one): a short remainder split would leave its slot idle while the full-length ones decide the duration
  const int n_splits = (n_steps_all + steps_per_split - 1) / steps_per_split;
  if (split >= n_splits) return;
  const int base_steps = n_steps_all / n_splits, extra = n_steps_all - base_steps * n_splits;
  const int step_begin = split * base_steps + min(split, extra);
  const int n = base_steps + (split < extra ? 1 : 0);
  const int* bt = block_table + (size_t)srv * max_blocks;
  const bool page_pow2 = (page_size & (page_size - 1)) == 0;
  const int page_shift = 31 - __builtin_clz(page_size);
  const int last_tile_key = ((n_keys - 1) >> 4) << 4;

  // ---- this wave's 32 query rows
  const int tile_row0 = q_row_offset + wave * 32;
  const int rows = T * G - tile_row0;
  const bool has_rows = rows > 0;
  const int my_lr = tile_row0 + c32;
  const bool my_ok = c32 < rows;
  const int my_j = my_ok ? my_lr / G : 0, my_hg = my_ok ? my_lr - my_j * G : 0;
  const int limit = my_ok ? L + my_j : -1;
  const int j_max = min(T - 1, (tile_row0 + 31) / G);
  const int my_step_end = has_rows ? ((L + j_max) >> 5) + 1 : 0;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  bf16x8_t qf[KK];
  {
    const bf16_t* src = q + ((size_t)(row0 + my_j) * n_heads + kh * G + my_hg) * HD + h * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (my_ok) v = *reinterpret_cast<const uint4*>(src + kk * 16);
      qf[kk] = *reinterpret_cast<const bf16x8_t*>(&v);
    }
  }
  float m_run = kNegBig, l_run = 0.f;
  floatx16_t oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;

  // block-table entry and first slot of the two 16-key tiles of a step (a tile past the end re-reads the last one)
  auto locate = [&](int step, int (&blk)[2], int (&slot0)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key0 = min(step * 32 + t * 16, last_tile_key);
      blk[t] = page_pow2 ? key0 >> page_shift : key0 / page_size;
      slot0[t] = key0 - blk[t] * page_size;
    }
  };
  auto lookup = [&](int step, int (&page)[2], int (&slot0)[2]) {
    int blk[2];
    locate(step, blk, slot0);
    page[0] = bt[blk[0]];
    page[1] = bt[blk[1]];
  };
  const unsigned k_lane_off = (unsigned)(c * HD + g * 8) * 2u;
  const unsigned v_lane_off = (unsigned)((lane >> 1) * page_size + (lane & 1) * 8) * 2u;
  const char* k_bytes = reinterpret_cast<const char*>(k_pages);
  const char* v_bytes = reinterpret_cast<const char*>(v_pages);
  auto issue = [&](int slot, const int (&page)[2], const int (&slot0)[2]) {
    unsigned char* stage = ring + slot * STAGE;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if (wave != (NW > 4 ? p : p % NW)) continue;
      const int t = p & 1;
      const size_t head = (size_t)page[t] * n_kv + kh;
      if (p < 2) {
        const char* src = k_bytes + (head * page_size + slot0[t]) * (HD * 2) + k_lane_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          __builtin_amdgcn_global_load_lds(src + ks * 64,
                                           (__attribute__((address_space(3))) void*)(stage + p * PART + ks * 1024),
                                           16, 0, kKvLoadPolicy);
      } else {
        const char* src = v_bytes + (head * HD * page_size + slot0[t]) * 2 + v_lane_off;
        const size_t stride = (size_t)64 * page_size;
#pragma unroll
        for (int ch = 0; ch < KS; ++ch)
          __builtin_amdgcn_global_load_lds(src + ch * stride,
                                           (__attribute__((address_space(3))) void*)(stage + p * PART + ch * 1024),
                                           16, 0, kKvLoadPolicy);
      }
    }
  };

  int pg_next[2], sl_next[2];
  {
    int blk[2];
    locate(step_begin, blk, sl_next);
    issue(0, first_pages, sl_next);
  }
  if (1 < n) lookup(step_begin + 1, pg_next, sl_next);

  // K fragment of k step kk for this lane: tile c32/16, fragment kk/2, lane group 2 (kk%2) + h, key c32%16
  const int k_lane = ((c32 >> 4) * KS * 64 + h * 16 + (c32 & 15)) * 16;
  // V: channel c32 of a 32-channel tile is 32 bytes per 16-key tile; this lane's runs start at slot 4h and 8 + 4h
  const int v_lane = 2 * PART + c32 * 32 + h * 8;

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
    bf16x8_t kf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      kf[kk] = *reinterpret_cast<const bf16x8_t*>(base + k_lane + (kk >> 1) * 1024 + (kk & 1) * 512);
    floatx16_t sacc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sacc, 0, 0, 0);

    float p[16];
    float corr;
    if (step * 32 + 31 <= L) {
      float mx = sacc[0];
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[e]);
      mx = halves_max(mx);
      const float m_new = fmaxf(m_run, mx * scale_log2);
      corr = __builtin_amdgcn_exp2f(m_run - m_new);
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        p[e] = __builtin_amdgcn_exp2f(fmaf(sacc[e], scale_log2, -m_new));
        sum += p[e];
      }
      l_run = l_run * corr + halves_sum(sum);
      m_run = m_new;
    } else {
      float sv[16];
      float mx = kNegBig;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = step * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
        sv[e] = key <= limit ? sacc[e] * scale_log2 : kNegBig;
        mx = fmaxf(mx, sv[e]);
      }
      mx = halves_max(mx);
      const float m_new = fmaxf(m_run, mx);
      corr = __builtin_amdgcn_exp2f(m_run - m_new);
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        p[e] = (sv[e] > kNegBig) ? __builtin_amdgcn_exp2f(sv[e] - m_new) : 0.f;
        sum += p[e];
      }
      l_run = l_run * corr + halves_sum(sum);
      m_run = m_new;
    }
    // P as a two-term bf16 sum (value and rounding remainder); k step kk' takes registers 8 kk' .. 8 kk' + 7
    bf16x8_t pf[2], pf_lo[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      uint4 hi, lo;
      const float* pp = p + 8 * kk;
      hi.x = pack_bf16x2(pp[0], pp[1]);
      hi.y = pack_bf16x2(pp[2], pp[3]);
      hi.z = pack_bf16x2(pp[4], pp[5]);
      hi.w = pack_bf16x2(pp[6], pp[7]);
      lo.x = pack_bf16x2(pp[0] - __uint_as_float(hi.x << 16), pp[1] - __uint_as_float(hi.x & 0xffff0000u));
      lo.y = pack_bf16x2(pp[2] - __uint_as_float(hi.y << 16), pp[3] - __uint_as_float(hi.y & 0xffff0000u));
      lo.z = pack_bf16x2(pp[4] - __uint_as_float(hi.z << 16), pp[5] - __uint_as_float(hi.z & 0xffff0000u));
      lo.w = pack_bf16x2(pp[6] - __uint_as_float(hi.w << 16), pp[7] - __uint_as_float(hi.w & 0xffff0000u));
      pf[kk] = *reinterpret_cast<const bf16x8_t*>(&hi);
      pf_lo[kk] = *reinterpret_cast<const bf16x8_t*>(&lo);
    }
    // the rescale factor of a query row sits in the lanes that hold the row: a per-lane multiply,
    // skipped once the running maxima have settled
    if (__any(corr != 1.0f)) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[dt][e] *= corr;
    }
    // second product, two channel tiles at a time (16 fragment registers live instead of 32)
    const bool tail = step * 32 + 32 > n_keys;
    uint4 keep[2];
    if (tail) {
      // keys past the end of the sequence inside the last page hold stale data: zero their V
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const int kb0 = step * 32 + 16 * kk + 4 * h, kb1 = kb0 + 8;
        keep[kk].x = (kb0 + 0 < n_keys ? 0x0000ffffu : 0u) | (kb0 + 1 < n_keys ? 0xffff0000u : 0u);
        keep[kk].y = (kb0 + 2 < n_keys ? 0x0000ffffu : 0u) | (kb0 + 3 < n_keys ? 0xffff0000u : 0u);
        keep[kk].z = (kb1 + 0 < n_keys ? 0x0000ffffu : 0u) | (kb1 + 1 < n_keys ? 0xffff0000u : 0u);
        keep[kk].w = (kb1 + 2 < n_keys ? 0x0000ffffu : 0u) | (kb1 + 3 < n_keys ? 0xffff0000u : 0u);
      }
    }
#pragma unroll
    for (int d0 = 0; d0 < DT; d0 += 2) {
      uint4 vv[2][2];
#pragma unroll
      for (int dd = 0; dd < 2; ++dd)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const unsigned char* vp = base + v_lane + kk * PART + (d0 + dd) * 1024;
          // (native vector type: an LDS read without type metadata makes the compiler wait for every
          // outstanding global->LDS load first, which would drain the prefetched stage in mid-step)
          const uintx2_t a = *reinterpret_cast<const uintx2_t*>(vp);
          const uintx2_t b = *reinterpret_cast<const uintx2_t*>(vp + 16);
          vv[dd][kk] = make_uint4(a.x, a.y, b.x, b.y);
        }
      if (tail) {
#pragma unroll
        for (int dd = 0; dd < 2; ++dd)
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            vv[dd][kk].x &= keep[kk].x; vv[dd][kk].y &= keep[kk].y; vv[dd][kk].z &= keep[kk].z; vv[dd][kk].w &= keep[kk].w;
          }
      }
#pragma unroll
      for (int dd = 0; dd < 2; ++dd)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(&vv[dd][kk]);
          oacc[d0 + dd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kk], oacc[d0 + dd], 0, 0, 0);
          oacc[d0 + dd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf_lo[kk], oacc[d0 + dd], 0, 0, 0);
        }
    }
  }

  // ---- this split's partial result: lane l holds query row l%32, channels 32 dt + 8 b + 4 h + (0..3)
  if (!my_ok) return;
  const size_t out_idx = ((size_t)(row0 + my_j) * n_heads + kh * G + my_hg) * max_splits + split;
  if (h == 0) {
    partial_ml[out_idx * 2 + 0] = m_run;
    partial_ml[out_idx * 2 + 1] = l_run;
  }
  float* dst = partial_o + out_idx * HD + 4 * h;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int b = 0; b < 4; ++b)
      *reinterpret_cast<float4*>(dst + dt * 32 + b * 8) =
          make_float4(oacc[dt][4 * b], oacc[dt][4 * b + 1], oacc[dt][4 * b + 2], oacc[dt][4 * b + 3]);
}

// attn_out[r][h*HD + d] = sum_s o_s * 2^(m_s - M) / sum_s l_s * 2^(m_s - M) over the row's server's own
// splits.  grid (R*H), block HD.
template <int HD>
__global__ void attn_combine_kernel(const float* __restrict__ partial_o, const float* __restrict__ partial_ml,
                                    int max_splits, int steps_per_split, const int4* __restrict__ row_info,
                                    int n_heads, bf16_t* __restrict__ attn_out) {
  const size_t rh = blockIdx.x;
  const int d = threadIdx.x;
  const int n_keys = row_info[rh / n_heads].z;      // keys of the row's server (per-row table of the step)
  const int n_splits = (((n_keys + 31) >> 5) + steps_per_split - 1) / steps_per_split;
  // one pass with a running maximum, so that no load waits for the maximum over all splits
  const float2* ml = reinterpret_cast<const float2*>(partial_ml) + rh * max_splits;
  const float* po = partial_o + rh * max_splits * HD + d;
  float M = kNegBig, Lsum = 0.f, acc = 0.f;
#pragma unroll 4
  for (int s = 0; s < n_splits; ++s) {
    const float2 st = ml[s];
    const float o = po[(size_t)s * HD];
    const float Mn = fmaxf(M, st.x);
    const float c = exp2f(M - Mn), f = exp2f(st.x - Mn);
    Lsum = Lsum * c + st.y * f;
    acc = acc * c + o * f;
    M = Mn;
  }
  attn_out[rh * HD + d] = float_to_bf16(acc / Lsum);
}

}  // namespace

// The most 32-key steps any compute unit is dealt when every server's steps are cut into splits of at most t
// steps: item_of_workgroup's serpentine over the (server, split, KV head) items in the order of decreasing
// length, which is the order of the work list.  items: their number.  Splits of 2047 steps and more are not
// modelled (the histogram lives on the stack): the largest long.
long attention_busiest_cu(int n_kv, int n_servers, const int* gamma_host, const int* ctx_len_host, long t,
                          long* items_out) {
  constexpr long kCus = kComputeUnits, kMaxLen = 2048;
  long n_of_len[kMaxLen] = {0};
  long items = 0;
  for (int i = 0; i < n_servers; ++i) {
    const long st = ((long)ctx_len_host[i] + gamma_host[i] + 1 + 31) / 32, n = (st + t - 1) / t;
    const long base = st / n, rem = st - base * n;
    items += n * n_kv;
    if (t + 2 > kMaxLen) continue;
    n_of_len[base + 1] += rem * n_kv;
    n_of_len[base] += (n - rem) * n_kv;
  }
  if (items_out) *items_out = items;
  if (t + 2 > kMaxLen) return std::numeric_limits<long>::max();
  const long rounds = (items + kCus - 1) / kCus;
  long load[kCus] = {0};
  long pos = 0;
  for (long len = t + 1; len >= 1; --len)
    for (long k = 0; k < n_of_len[len]; ++k, ++pos) {
      const long round = pos / kCus, c = pos - round * kCus;
      load[((rounds - 1 - round) & 1) ? kCus - 1 - c : c] += len;
    }
  return *std::max_element(load, load + kCus);
}

// KV steps (32 keys) per split, and the resulting largest split count, for a batch of n_servers servers with
// the given draft lengths and contexts and query tiles of at most max_block_tokens rows.  A server's steps
// are cut into ceil(steps / steps_per_split) splits of equal length up to one step.  All workgroups of the
// launch should be resident at once (they share the memory bandwidth; a second round starts with the chip
// half empty: measured on the 70B shape, 5.9 instead of 6.7 ms per step), which also keeps the partial
// results few; a floor on the steps per split bounds what the partial results cost on small batches.
void attention_plan(int n_kv, int group, int max_block_tokens, int n_servers, const int* gamma_host,
                    const int* ctx_len_host, int* steps_per_split, int* max_splits) {
  const int tiles = ceil_div(max_block_tokens * group, 32);
  const int waves = tiles < 8 ? (tiles > 0 ? tiles : 1) : 8;
  constexpr int kWavesPerCu = 12;    // by registers (three waves per SIMD)
  const int wgs_per_cu = kWavesPerCu / waves < 5 ? (kWavesPerCu / waves > 0 ? kWavesPerCu / waves : 1) : 5;   // 5 workgroups by LDS
  const long slots = (long)kComputeUnits * wgs_per_cu;
  auto steps_of = [&](int i) { return ((long)ctx_len_host[i] + gamma_host[i] + 1 + 31) / 32; };
  long total_steps = 0, max_steps = 1;
  for (int i = 0; i < n_servers; ++i) {
    total_steps += steps_of(i);
    if (steps_of(i) > max_steps) max_steps = steps_of(i);
  }
  // workgroups of a launch with splits of at most t steps
  auto workgroups = [&](long t) {
    long c = 0;
    for (int i = 0; i < n_servers; ++i) c += (steps_of(i) + t - 1) / t;
    return c * n_kv;
  };
  long lo = (max_steps + 31) / 32;                        // at most 32 splits per server
  if (lo < 6) lo = 6;                                     // at least 6 steps per split (partial-result traffic)
  if (lo > max_steps) lo = max_steps;
  const long fit = slots - slots / 16;                    // all resident at once, with some slack for placement
  long sps;
  if (workgroups(max_steps) <= fit) {
    // the shortest splits whose workgroups are all resident at once ...
    long a = lo, b = max_steps;
    while (a < b) {
      const long mid = (a + b) / 2;
      if (workgroups(mid) <= fit) b = mid; else a = mid + 1;
    }
    sps = a;
    // ... unless splits up to half longer load the busiest compute unit clearly less (a compute unit's
    // finishing time follows the steps it is dealt): 3 x 22 instead of 4 x 19 steps at the 70B shape with 16
    // servers (5.3 against 5.6 ms of attention per step).  Small differences do not pay for the workgroups that
    // are then missing per compute unit (8 servers at 2048 tokens: 2 x 9 steps on 512 workgroups took 17.1 us
    // per layer, 3 x 6 on 704 take 15.1), hence the margin of 8 %.
    long best = attention_busiest_cu(n_kv, n_servers, gamma_host, ctx_len_host, sps, nullptr);
    for (long t = sps + 1; t <= sps + sps / 2 && t <= max_steps; ++t) {
      const long l = attention_busiest_cu(n_kv, n_servers, gamma_host, ctx_len_host, t, nullptr);
      if (l * 100 < best * 92) {
        best = l;
        sps = t;
      }
    }
  } else {
    // more (server, KV head) pairs than slots: several rounds of workgroups anyway
    sps = (total_steps * n_kv + slots / 2 - 1) / (slots / 2);
    if (sps < lo) sps = lo;
    if (sps > max_steps) sps = max_steps;
  }
  *steps_per_split = (int)sps;
  // the split count is also the stride (in 512-byte partial rows) between the partial results of
  // neighbouring (row, head) pairs: kept odd, because a power-of-two stride sends all partial stores of a
  // workgroup to the same few memory channels (measured: 110 instead of 81 us per layer at a stride of 32)
  *max_splits = (int)((max_steps + sps - 1) / sps) | 1;
}

size_t attention_workspace_floats(int n_rows, int n_heads, int hd, int max_splits) {
  return (size_t)n_rows * n_heads * max_splits * (hd + 2);
}

template <int HD, int G>
static gs_status launch_mfma_g(const bf16_t* q, const bf16_t* k_pages, const bf16_t* v_pages, const int* block_table,
                               int max_blocks, const int* work, int n_work, int page_size,
                               int n_heads, int n_kv, int max_block_tokens, int steps_per_split, int max_splits,
                               float* po, float* pml, hipStream_t stream) {
  const int tiles = ceil_div(max_block_tokens * G, 32);
  dim3 grid((unsigned)n_work * (unsigned)n_kv);      // one workgroup per (entry, KV head) item, see item_of_workgroup
  for (int t0 = 0; t0 < tiles; t0 += 8) {      // at most 8 query tiles (waves) per workgroup
    const int waves = tiles - t0 < 8 ? tiles - t0 : 8;
#define GS_RING(NW_)                                                                                              \
  attn_kernel<HD, G, NW_><<<grid, 64 * NW_, 0, stream>>>(q, k_pages, v_pages, block_table, max_blocks, work,      \
                                                         n_work, page_size, n_heads, n_kv, steps_per_split, max_splits,   \
                                                         t0 * 32, po, pml)
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
    GS_LAUNCH_CHECK("attn");
  }
  return GS_OK;
}

// Number of ints of a work list with room for `capacity` entries.
size_t attention_work_ints(int capacity) { return 8 + 8 * (size_t)capacity; }

// Builds the step's work list (bf16 path): once per step, the block tables being the same for every layer.
gs_status launch_attention_work(const int* cu_rows, const int* ctx_len, int n_servers, const int* block_table,
                                int max_blocks, int page_size, int steps_per_split, int capacity, int* work,
                                hipStream_t stream) {
  attn_work_kernel<<<1, 256, 0, stream>>>(cu_rows, ctx_len, n_servers, block_table, max_blocks, page_size,
                                          steps_per_split, capacity, work);
  GS_LAUNCH_CHECK("attn_work");
  return GS_OK;
}

// attn_out [R][H*hd] (storage type).  scratch: attention_workspace_floats floats; work, n_work: the step's work
// list and its length as the host computes it from its copy of the batch geometry (bf16 path only).
gs_status launch_attention(int dtype, const void* q, const void* k_pages, const void* v_pages,
                           const int* block_table, int max_blocks, const int* cu_rows, const int* ctx_len,
                           int n_servers, int n_rows, int page_size, int n_heads, int n_kv, int hd,
                           int max_block_tokens, int steps_per_split, int max_splits, const void* row_info,
                           const int* work, int n_work, float* scratch, void* attn_out, hipStream_t stream) {
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
    st = launch_mfma_g<HD_, G_>(qb, kb, vb, block_table, max_blocks, work, n_work, page_size, n_heads, n_kv,     \
                                max_block_tokens, steps_per_split, max_splits, po, pml, stream);
  GS_ATTN_CASE(128, 1) GS_ATTN_CASE(128, 2) GS_ATTN_CASE(128, 4) GS_ATTN_CASE(128, 8)
  GS_ATTN_CASE(64, 1) GS_ATTN_CASE(64, 2) GS_ATTN_CASE(64, 4) GS_ATTN_CASE(64, 8)
#undef GS_ATTN_CASE
  if (st != GS_OK) return st;
  if (hd == 128)
    attn_combine_kernel<128><<<n_rows * n_heads, 128, 0, stream>>>(po, pml, max_splits, steps_per_split,
                                                                   static_cast<const int4*>(row_info), n_heads,
                                                                   static_cast<bf16_t*>(attn_out));
  else
    attn_combine_kernel<64><<<n_rows * n_heads, 64, 0, stream>>>(po, pml, max_splits, steps_per_split,
                                                                 static_cast<const int4*>(row_info), n_heads,
                                                                 static_cast<bf16_t*>(attn_out));
  GS_LAUNCH_CHECK("attn_combine");
  return GS_OK;
}

}  // namespace gs
