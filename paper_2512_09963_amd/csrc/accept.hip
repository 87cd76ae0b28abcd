// Rejection-verification on the GPU: vocabulary softmax statistics, the accept
// test, and the residual / bonus draw (paper Section II-A-2; the per-server
// statistic is the sum inside the acceptance-rate update of Section III-C).
//
// Three launches on one stream, no host synchronisation:
//   row_stats   every target row is read once, with non-temporal 16-byte loads, four per lane
//               in flight; each workgroup reduces one chunk of one row to an online-softmax
//               pair (max, sum exp(l - max))
//   draw_tiles  grid (tile groups, servers).  Every workgroup first repeats its server's
//               decision (merge the chunk pairs of its rows, gather p_j(s_j) and q_j(s_j),
//               accept tests, m, statistic: a few hundred bytes out of L2), then sums
//               max(0, p - q) (or p for the bonus draw) over its 2048-token tiles of the one
//               row the extra token is drawn from
//   pick_token  one workgroup per server: scans the tile sums, then the one tile, for the
//               token whose running sum first exceeds u * total
// Bandwidth-bound: row_stats streams 4*V bytes per target row; the draw touches O(N*V) bytes.
#include "common.h"
#include "device_types.h"
#include <cmath>
#include <mutex>

namespace gs {
namespace {

constexpr int kStatsThreads = 256;
constexpr int kTileThreads = 256;
constexpr int kTileElems = 2048;              // 256 lanes x 8 tokens
constexpr int kMaxChunks = 64;
}  // namespace
// Rows and servers are laid out along gridDim.x (chunks or tile groups fastest), which HIP bounds by
// 2^31 - 1 workgroups: 2^22 rows of at most 64 chunks stay below it.
constexpr long kMaxAcceptRows = 1L << 22;
namespace {

struct Decision {    // per server, written by decide, read by the draw kernels
  int row;           // target row the extra token is drawn from (first row + m)
  int q_row;         // draft row whose q is subtracted, or -1 for the bonus draw from p
  float row_max;     // softmax statistics of that row
  float inv_z;
};

__device__ __forceinline__ void merge_pair(float& m, float& s, float m2, float s2) {
  float M = fmaxf(m, m2);
  float a = (m == -INFINITY) ? 0.f : s * __expf(m - M);
  float b = (m2 == -INFINITY) ? 0.f : s2 * __expf(m2 - M);
  m = M;
  s = a + b;
}

__device__ __forceinline__ float max4(const float4& v) { return fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)); }

// Sixteen bytes of a row: 4 floats or 8 bfloat16, widened to float.  STREAM: the load does not displace
// cache lines (the logits are read once by the statistics pass).
typedef float __attribute__((ext_vector_type(4))) float4_vec;
typedef unsigned int __attribute__((ext_vector_type(4))) uint4_vec;
template <typename T> struct Pack;
template <> struct Pack<float> {
  static constexpr int W = 4;
  template <bool STREAM>
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4_vec x = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const float4_vec*>(p))
                                : *reinterpret_cast<const float4_vec*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
};
template <> struct Pack<bf16_t> {
  static constexpr int W = 8;
  template <bool STREAM>
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4_vec x = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const uint4_vec*>(p))
                               : *reinterpret_cast<const uint4_vec*>(p);
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xffff0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xffff0000u);
  }
};
template <int W>
__device__ __forceinline__ float max_of(const float (&v)[W]) {
  float m = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
  if constexpr (W == 8) m = fmaxf(m, fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
  return m;
}
template <int W>
__device__ __forceinline__ float sum_exp_of(const float (&v)[W], float mm) {
  float a = __expf(v[0] - mm) + __expf(v[1] - mm) + __expf(v[2] - mm) + __expf(v[3] - mm);
  if constexpr (W == 8) a += __expf(v[4] - mm) + __expf(v[5] - mm) + __expf(v[6] - mm) + __expf(v[7] - mm);
  return a;
}

// ---------------------------------------------------------------------------------------
// row_stats: grid chunks * rows (chunk fastest).  VEC: rows are 16-byte aligned and V % 4 == 0.
// ---------------------------------------------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(kStatsThreads) void row_stats_kernel(const T* __restrict__ logits, int vocab,
                                                                   int chunk_len, int n_chunks,
                                                                   float2* __restrict__ partial) {
  constexpr int W = Pack<T>::W;
  const int row = blockIdx.x / n_chunks, chunk = blockIdx.x - row * n_chunks;
  const int begin = chunk * chunk_len;
  const int end = min(vocab, begin + chunk_len);
  const T* base = logits + (size_t)row * vocab;
  float m = -INFINITY, s = 0.f;

  if (VEC) {
    const T* p = base + begin;
    const int n_pk = (end - begin) / W;
    for (int i = threadIdx.x; i < n_pk; i += 4 * kStatsThreads) {
      float v0[W], v1[W], v2[W], v3[W];
#pragma unroll
      for (int k = 0; k < W; ++k) v1[k] = v2[k] = v3[k] = -INFINITY;
      Pack<T>::template load<true>(p + (size_t)i * W, v0);
      if (i + kStatsThreads < n_pk) Pack<T>::template load<true>(p + (size_t)(i + kStatsThreads) * W, v1);
      if (i + 2 * kStatsThreads < n_pk) Pack<T>::template load<true>(p + (size_t)(i + 2 * kStatsThreads) * W, v2);
      if (i + 3 * kStatsThreads < n_pk) Pack<T>::template load<true>(p + (size_t)(i + 3 * kStatsThreads) * W, v3);
      const float bm = fmaxf(fmaxf(max_of<W>(v0), max_of<W>(v1)), fmaxf(max_of<W>(v2), max_of<W>(v3)));
      if (bm > m) {
        s *= __expf(m - bm);     // m = -inf gives exp(-inf) = 0 and s is 0 anyway
        m = bm;
      }
      const float mm = (m == -INFINITY) ? 0.f : m;   // a lane that has seen only -inf adds exp(-inf) = 0
      const float a0 = sum_exp_of<W>(v0, mm), a1 = sum_exp_of<W>(v1, mm);
      const float a2 = sum_exp_of<W>(v2, mm), a3 = sum_exp_of<W>(v3, mm);
      s += (a0 + a1) + (a2 + a3);
    }
  } else {
    for (int i = begin + threadIdx.x; i < end; i += kStatsThreads) {
      const float v = Storage<T>::load(base + i);
      if (v > m) {
        s *= __expf(m - v);
        m = v;
      }
      s += __expf(v - ((m == -INFINITY) ? 0.f : m));
    }
  }

  // wavefront then workgroup merge (fixed order: deterministic)
  for (int off = 32; off > 0; off >>= 1) {
    float m2 = __shfl_down(m, off);
    float s2 = __shfl_down(s, off);
    merge_pair(m, s, m2, s2);
  }
  __shared__ float sm[kStatsThreads / 64], ss[kStatsThreads / 64];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    sm[wave] = m;
    ss[wave] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kStatsThreads / 64; ++w) merge_pair(m, s, sm[w], ss[w]);
    partial[(size_t)row * n_chunks + chunk] = make_float2(m, s);
  }
}

// merge_stats: the statistics of a row from the per-column-block pairs that the LM-head projection left
// (stats [rows][n_blocks]).  grid rows, 256 lanes: every lane issues its (up to four at a time) loads back to
// back, then a fixed-order merge over the lanes of a wave and over the waves.
__global__ __launch_bounds__(256) void merge_stats_kernel(const float2* __restrict__ stats, int n_blocks,
                                                          float2* __restrict__ row_stat) {
  const int row = blockIdx.x, tid = threadIdx.x;
  const float2* p = stats + (size_t)row * n_blocks;
  float m = -INFINITY, s = 0.f;
  for (int b0 = tid; b0 < n_blocks; b0 += 4 * 256) {
    float2 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = (b0 + k * 256 < n_blocks) ? p[b0 + k * 256] : make_float2(-INFINITY, 0.f);
#pragma unroll
    for (int k = 0; k < 4; ++k) merge_pair(m, s, v[k].x, v[k].y);
  }
  for (int off = 32; off > 0; off >>= 1) {
    const float m2 = __shfl_down(m, off), s2 = __shfl_down(s, off);
    merge_pair(m, s, m2, s2);
  }
  __shared__ float sm[4], ss[4];
  if ((tid & 63) == 0) {
    sm[tid >> 6] = m;
    ss[tid >> 6] = s;
  }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w) merge_pair(m, s, sm[w], ss[w]);
    row_stat[row] = make_float2(m, s);
  }
}

// Weight of token t in the draw: max(0, p - q) or p.
__device__ __forceinline__ float draw_weight(float logit, float q, float row_max, float inv_z, bool residual) {
  float p = expf(logit - row_max) * inv_z;
  return residual ? fmaxf(0.f, p - q) : p;
}

// Loads this lane's 8 consecutive weights of a tile; tokens >= vocab weigh 0.
template <typename T, bool VEC>
__device__ __forceinline__ void load_weights8(const T* __restrict__ lrow, const T* __restrict__ qrow, int t0,
                                              int vocab, float row_max, float inv_z, bool residual, float w[8]) {
  if (VEC && t0 + 8 <= vocab) {
    constexpr int W = Pack<T>::W;
    float l[8], q[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) q[k] = 0.f;
#pragma unroll
    for (int h = 0; h < 8 / W; ++h) {
      float part[W];
      Pack<T>::template load<false>(lrow + t0 + h * W, part);
#pragma unroll
      for (int k = 0; k < W; ++k) l[h * W + k] = part[k];
    }
    if (residual) {
#pragma unroll
      for (int h = 0; h < 8 / W; ++h) {
        float part[W];
        Pack<T>::template load<false>(qrow + t0 + h * W, part);
#pragma unroll
        for (int k = 0; k < W; ++k) q[h * W + k] = part[k];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = draw_weight(l[k], q[k], row_max, inv_z, residual);
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int t = t0 + k;
      w[k] = (t < vocab) ? draw_weight(Storage<T>::load(lrow + t), residual ? Storage<T>::load(qrow + t) : 0.f, row_max,
                                       inv_z, residual)
                         : 0.f;
    }
  }
}

__device__ __forceinline__ float sum8(const float w[8]) {
  return ((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]));
}

// Workgroup-wide scan of one double per lane (256 lanes).  Returns the inclusive sum and sets
// excl to the inclusive sum of the previous lane (0 for lane 0), bit-identical to what that
// lane returns, so "first lane whose inclusive sum crosses a threshold" is unique.
__device__ __forceinline__ double block_scan(double v, double* wave_tot /*[4] shared*/, double& excl) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int off = 1; off < 64; off <<= 1) {
    double o = __shfl_up(v, off);
    if (lane >= off) v += o;
  }
  double prev = __shfl_up(v, 1);
  if (lane == 63) wave_tot[wave] = v;
  __syncthreads();
  double add = 0.0, add_prev = 0.0;
  for (int wv = 0; wv < wave; ++wv) {
    add_prev = add;
    add += wave_tot[wv];
  }
  // previous lane of lane 0 is lane 63 of the wave before: its value is wave_tot[wave-1] + add_prev
  excl = (lane == 0) ? (wave == 0 ? 0.0 : wave_tot[wave - 1] + add_prev) : prev + add;
  __syncthreads();
  return v + add;
}

// Softmax statistics of one row from its chunk pairs.
__device__ __forceinline__ void row_max_sum(const float2* __restrict__ partial, int row, int n_chunks, float& m,
                                            float& s) {
  m = -INFINITY;
  s = 0.f;
  const float2* p = partial + (size_t)row * n_chunks;
#pragma unroll 8
  for (int c = 0; c < n_chunks; ++c) {
    const float2 ps = p[c];
    merge_pair(m, s, ps.x, ps.y);
  }
}

// The accept decisions of one server, computed by one wavefront (lanes over draft positions).
// Returns the decision in every lane; lane 0 of a workgroup with write_out set stores the outputs.
template <typename T>
__device__ __forceinline__ Decision decide_server(int srv, const int* __restrict__ cu_rows, int vocab, int n_chunks,
                                                  const float2* __restrict__ partial,
                                                  const T* __restrict__ logits, const T* __restrict__ q_probs,
                                                  const int* __restrict__ draft_tokens,
                                                  const float* __restrict__ u_accept, bool write_out,
                                                  int* __restrict__ accepted_len, float* __restrict__ accept_stat,
                                                  float* __restrict__ ratio_out) {
  const int lane = threadIdx.x & 63;
  const int row0 = cu_rows[srv];
  const int gamma = cu_rows[srv + 1] - row0 - 1;
  const int d0 = row0 - srv;
  int first_reject = gamma;    // smallest rejected draft index seen by this lane
  float stat = 0.f;
  bool bad_id = false;         // a draft token id outside the vocabulary: never used as an index
  for (int j = lane; j < gamma; j += 64) {
    const int row = row0 + j;
    int tok = draft_tokens[d0 + j];
    if (tok < 0 || tok >= vocab) {
      bad_id = true;
      tok = 0;
    }
    const float u = u_accept[d0 + j];
    const float lg = Storage<T>::load(logits + (size_t)row * vocab + tok);
    const float q = Storage<T>::load(q_probs + (size_t)(d0 + j) * vocab + tok);
    float m, s;
    row_max_sum(partial, row, n_chunks, m, s);
    const float p = expf(lg - m) / s;
    const float ratio = (q == 0.f) ? INFINITY : p / q;
    if (write_out && ratio_out) ratio_out[d0 + j] = ratio;
    stat += fminf(1.f, ratio);
    if (u > ratio) first_reject = min(first_reject, j);
  }
  for (int off = 32; off > 0; off >>= 1) {
    first_reject = min(first_reject, __shfl_xor(first_reject, off));
    stat += __shfl_xor(stat, off);
  }
  const bool any_bad = __any(bad_id);      // (all 64 lanes of the wave are here)
  const int m_acc = any_bad ? 0 : first_reject;
  if (write_out && lane == 0) {
    accepted_len[srv] = any_bad ? -1 : m_acc;
    accept_stat[srv] = gamma > 0 ? stat / (float)gamma : 0.f;
  }
  Decision d;
  d.row = row0 + m_acc;
  d.q_row = (m_acc < gamma) ? d0 + m_acc : -1;
  float m, s;
  row_max_sum(partial, d.row, n_chunks, m, s);
  d.row_max = m;
  d.inv_z = 1.f / s;
  return d;
}

// ---------------------------------------------------------------------------------------
// draw_tiles: grid tile groups * servers (group fastest), 256 lanes.  A workgroup owns kTilesPerGroup
// consecutive 2048-token tiles; group 0 also stores the server's outputs and its decision.
// ---------------------------------------------------------------------------------------
constexpr int kTilesPerGroup = 4;

template <typename T, bool VEC>
__global__ __launch_bounds__(kTileThreads) void draw_tiles_kernel(const int* __restrict__ cu_rows, int vocab,
                                                                  int n_chunks, int n_tiles, int n_groups,
                                                                  const float2* __restrict__ partial,
                                                                  const T* __restrict__ logits,
                                                                  const T* __restrict__ q_probs,
                                                                  const int* __restrict__ draft_tokens,
                                                                  const float* __restrict__ u_accept,
                                                                  int* __restrict__ accepted_len,
                                                                  float* __restrict__ accept_stat,
                                                                  float* __restrict__ ratio_out,
                                                                  Decision* __restrict__ decision,
                                                                  double* __restrict__ tile_sums) {
  const int srv = blockIdx.x / n_groups, group = blockIdx.x - srv * n_groups;
  __shared__ Decision sh_d;
  __shared__ double part[kTileThreads / 64];
  if (threadIdx.x < 64) {
    const Decision dd = decide_server<T>(srv, cu_rows, vocab, n_chunks, partial, logits, q_probs, draft_tokens, u_accept,
                                      group == 0, accepted_len, accept_stat, ratio_out);
    if (threadIdx.x == 0) {
      sh_d = dd;
      if (group == 0) decision[srv] = dd;
    }
  }
  __syncthreads();
  const Decision d = sh_d;
  const bool residual = d.q_row >= 0;
  const T* lrow = logits + (size_t)d.row * vocab;
  const T* qrow = residual ? q_probs + (size_t)d.q_row * vocab : nullptr;
  // all loads of the group's tiles are issued before the first is consumed
  float w[kTilesPerGroup][8];
#pragma unroll
  for (int k = 0; k < kTilesPerGroup; ++k) {
    const int tile = group * kTilesPerGroup + k;
    if (tile < n_tiles)
      load_weights8<T, VEC>(lrow, qrow, tile * kTileElems + threadIdx.x * 8, vocab, d.row_max, d.inv_z, residual, w[k]);
  }
#pragma unroll
  for (int k = 0; k < kTilesPerGroup; ++k) {
    const int tile = group * kTilesPerGroup + k;
    if (tile >= n_tiles) break;
    double acc = (double)sum8(w[k]);
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = part[0];
      for (int wv = 1; wv < kTileThreads / 64; ++wv) t += part[wv];
      tile_sums[(size_t)srv * n_tiles + tile] = t;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// pick_token: one workgroup per server.
// ---------------------------------------------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(kTileThreads) void pick_token_kernel(const Decision* __restrict__ decision, int vocab,
                                                                   int n_tiles, const T* __restrict__ logits,
                                                                   const T* __restrict__ q_probs,
                                                                   const double* __restrict__ tile_sums,
                                                                   const float* __restrict__ u_resample,
                                                                   int* __restrict__ next_token) {
  const int srv = blockIdx.x;
  const Decision d = decision[srv];
  bool residual = d.q_row >= 0;
  const T* lrow = logits + (size_t)d.row * vocab;
  const T* qrow = residual ? q_probs + (size_t)d.q_row * vocab : nullptr;
  __shared__ double wave_tot[kTileThreads / 64];
  __shared__ double sh_prefix;
  __shared__ int sh_tile, sh_found, sh_last_pos;
  float w[8];

  // total mass: workgroup scan over the tile sums (fixed order: deterministic)
  const double* sums = tile_sums + (size_t)srv * n_tiles;
  double total = 0.0;
  for (int base = 0; base < n_tiles; base += kTileThreads) {
    const int t = base + threadIdx.x;
    double ex;
    const double incl = block_scan(t < n_tiles ? sums[t] : 0.0, wave_tot, ex);
    if (threadIdx.x == kTileThreads - 1) sh_prefix = incl;
    __syncthreads();
    total += sh_prefix;
    __syncthreads();
  }

  const bool fallback = residual && !(total > 0.0);   // residual without mass: draw from p instead
  if (fallback) {
    residual = false;
    // recompute the total of p tile by tile (rare path, one workgroup walks the row)
    double tot = 0.0;
    for (int t = 0; t < n_tiles; ++t) {
      load_weights8<T, VEC>(lrow, nullptr, t * kTileElems + threadIdx.x * 8, vocab, d.row_max, d.inv_z, false, w);
      double ex;
      double incl = block_scan((double)sum8(w), wave_tot, ex);
      if (threadIdx.x == kTileThreads - 1) sh_prefix = incl;
      __syncthreads();
      tot += sh_prefix;
      __syncthreads();
    }
    total = tot;
  }

  const double target = (double)u_resample[srv] * total;
  if (threadIdx.x == 0) {
    sh_found = -1;
    sh_last_pos = -1;
    sh_tile = n_tiles - 1;
    sh_prefix = 0.0;
  }
  __syncthreads();

  if (!fallback) {
    // the tile in which the running sum crosses the target: exactly one lane sees the crossing
    __shared__ int sh_last_tile;
    __shared__ double sh_carry;
    if (threadIdx.x == 0) {
      sh_tile = -1;
      sh_last_tile = 0;
    }
    __syncthreads();
    double carry = 0.0;
    for (int base = 0; base < n_tiles; base += kTileThreads) {
      const int t = base + threadIdx.x;
      const double v = t < n_tiles ? sums[t] : 0.0;
      double ex;
      const double incl = block_scan(v, wave_tot, ex);
      if ((carry + incl > target) && !(carry + ex > target)) {
        sh_tile = t;
        sh_prefix = carry + ex;
      }
      if (v > 0.0) atomicMax(&sh_last_tile, t);
      if (threadIdx.x == kTileThreads - 1) sh_carry = carry + incl;
      __syncthreads();
      carry = sh_carry;
      const bool done = sh_tile >= 0;
      __syncthreads();
      if (done) break;
    }
    if (sh_tile < 0) {             // rounding left no crossing: the last tile with mass
      carry = 0.0;
      for (int base = 0; base < n_tiles; base += kTileThreads) {
        const int t = base + threadIdx.x;
        double ex;
        const double incl = block_scan(t < n_tiles ? sums[t] : 0.0, wave_tot, ex);
        if (t == sh_last_tile) sh_prefix = carry + ex;
        if (threadIdx.x == kTileThreads - 1) sh_carry = carry + incl;
        __syncthreads();
        carry = sh_carry;
        __syncthreads();
      }
      if (threadIdx.x == 0) sh_tile = sh_last_tile;
      __syncthreads();
    }
  }

  // Walk tiles: a single tile in the normal path, all tiles until found in the fallback path.
  int tile = fallback ? 0 : sh_tile;
  double prefix = fallback ? 0.0 : sh_prefix;
  int last_pos_any = -1;
  for (;;) {
    const int t0 = tile * kTileElems + threadIdx.x * 8;
    load_weights8<T, VEC>(lrow, qrow, t0, vocab, d.row_max, d.inv_z, residual, w);
    double excl;
    const double incl = block_scan((double)sum8(w), wave_tot, excl);
    // exactly one lane sees the running sum cross the target inside its 8 tokens
    if ((prefix + incl > target) && !(prefix + excl > target)) {
      double run = prefix + excl;
      int pick = -1, last = -1;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        run += (double)w[k];
        if (w[k] > 0.f) {
          last = t0 + k;
          if (pick < 0 && run > target) pick = t0 + k;
        }
      }
      sh_found = pick >= 0 ? pick : last;   // lane-local sum order may differ in the last bit
    }
    int lp = -1;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (w[k] > 0.f) lp = t0 + k;
    if (lp >= 0) atomicMax(&sh_last_pos, lp);
    if (threadIdx.x == kTileThreads - 1) sh_prefix = prefix + incl;
    __syncthreads();
    const int found = sh_found;
    prefix = sh_prefix;
    last_pos_any = sh_last_pos;
    __syncthreads();
    if (found >= 0 || !fallback || tile == n_tiles - 1) {
      if (threadIdx.x == 0) next_token[srv] = found >= 0 ? found : max(last_pos_any, 0);
      break;
    }
    ++tile;
  }
}

inline int pick_chunks(int n_rows, int vocab) {
  int want = ceil_div(4096, n_rows > 0 ? n_rows : 1);
  int cap = vocab / 4096 > 0 ? vocab / 4096 : 1;
  int c = want < cap ? want : cap;
  if (c < 1) c = 1;
  if (c > kMaxChunks) c = kMaxChunks;
  return c;
}

struct AcceptPlan {
  int n_chunks, chunk_len, n_tiles;
  size_t bytes;
  float2* partial;
  Decision* decision;
  double* tile_sums;
};

// pack: elements per 16-byte load of the element type (4 for fp32, 8 for bf16); a chunk is a whole number of them
AcceptPlan plan_accept(int n_servers, int n_rows, int vocab, void* workspace, int pack = 4) {
  AcceptPlan p;
  p.n_chunks = pick_chunks(n_rows, vocab);
  p.chunk_len = (ceil_div(vocab, p.n_chunks) + pack - 1) / pack * pack;
  p.n_chunks = ceil_div(vocab, p.chunk_len);
  p.n_tiles = ceil_div(vocab, kTileElems);
  Carver c(workspace);
  p.partial = c.take<float2>((size_t)n_rows * p.n_chunks);
  p.decision = c.take<Decision>(n_servers);
  p.tile_sums = c.take<double>((size_t)n_servers * p.n_tiles);
  p.bytes = c.used();
  return p;
}

template <typename T, bool VEC>
gs_status launch_accept_t(const AcceptPlan& p, int n_servers, int n_rows, const int* cu_rows, int vocab,
                          const T* target_logits, const T* q_probs, const int* draft_tokens, const float* u_accept,
                          const float* u_resample, const gs_accept_out* out, hipStream_t stream,
                          const void* row_stats, int n_stat_blocks) {
  int n_chunks = p.n_chunks;
  if (row_stats) {      // one pair per row, merged from the producer's column-block pairs
    merge_stats_kernel<<<n_rows, 256, 0, stream>>>(static_cast<const float2*>(row_stats), n_stat_blocks, p.partial);
    GS_LAUNCH_CHECK("merge_stats");
    n_chunks = 1;
  } else {
    const unsigned g1 = (unsigned)p.n_chunks * (unsigned)n_rows;
    row_stats_kernel<T, VEC><<<g1, kStatsThreads, 0, stream>>>(target_logits, vocab, p.chunk_len, p.n_chunks, p.partial);
    GS_LAUNCH_CHECK("row_stats");
  }
  const int n_groups = ceil_div(p.n_tiles, kTilesPerGroup);
  const unsigned g2 = (unsigned)n_groups * (unsigned)n_servers;
  draw_tiles_kernel<T, VEC><<<g2, kTileThreads, 0, stream>>>(cu_rows, vocab, n_chunks, p.n_tiles, n_groups, p.partial,
                                                             target_logits, q_probs, draft_tokens, u_accept,
                                                             out->accepted_len, out->accept_stat, out->ratio,
                                                             p.decision, p.tile_sums);
  GS_LAUNCH_CHECK("draw_tiles");
  pick_token_kernel<T, VEC><<<n_servers, kTileThreads, 0, stream>>>(p.decision, vocab, p.n_tiles, target_logits, q_probs,
                                                                    p.tile_sums, u_resample, out->next_token);
  GS_LAUNCH_CHECK("pick_token");
  return GS_OK;
}

}  // namespace

// Enqueues the kernels; arguments already validated.  n_rows = sum(gamma + 1).
// elem: GS_F32 or GS_BF16, the type of target_logits and q_probs.
// row_stats: [n_rows][n_stat_blocks] pairs (max, sum exp) that the producer of the logits already reduced, or
// null: then the logits are read once more for them.
gs_status launch_accept(int n_servers, int n_rows, const int* cu_rows, int vocab, int elem, const void* target_logits,
                        const void* q_probs, const int* draft_tokens, const float* u_accept,
                        const float* u_resample, const gs_accept_out* out, void* workspace, hipStream_t stream,
                        const void* row_stats, int n_stat_blocks) {
  const int pack = elem == GS_BF16 ? 8 : 4;
  const AcceptPlan p = plan_accept(n_servers, n_rows, vocab, workspace, pack);
  const bool vec = (vocab % pack == 0) && (reinterpret_cast<uintptr_t>(target_logits) % 16 == 0) &&
                   (q_probs == nullptr || reinterpret_cast<uintptr_t>(q_probs) % 16 == 0);
#define GS_ACCEPT(T_, VEC_)                                                                                        \
  launch_accept_t<T_, VEC_>(p, n_servers, n_rows, cu_rows, vocab, static_cast<const T_*>(target_logits),           \
                            static_cast<const T_*>(q_probs), draft_tokens, u_accept, u_resample, out, stream,      \
                            row_stats, n_stat_blocks)
  if (elem == GS_BF16) return vec ? GS_ACCEPT(bf16_t, true) : GS_ACCEPT(bf16_t, false);
  return vec ? GS_ACCEPT(float, true) : GS_ACCEPT(float, false);
#undef GS_ACCEPT
}

size_t accept_workspace_bytes(int n_servers, int n_rows, int vocab) {
  const size_t a = plan_accept(n_servers, n_rows, vocab, nullptr, 4).bytes;
  const size_t b = plan_accept(n_servers, n_rows, vocab, nullptr, 8).bytes;
  return a > b ? a : b;
}

}  // namespace gs

extern "C" size_t gs_accept_workspace_bytes(int n_servers, int n_rows, int vocab) {
  if (n_servers <= 0 || n_rows <= 0 || vocab <= 0) return 0;
  return gs::accept_workspace_bytes(n_servers, n_rows, vocab);
}

namespace gs {
namespace {

gs_status accept_entry(int elem, int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                       const void* target_logits, const void* q_probs, const int* draft_tokens,
                       const float* u_accept, const float* u_resample, const gs_accept_out* out, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  if (n_servers <= 0 || vocab <= 0) return fail(GS_EINVAL, "n_servers and vocab must be positive");
  if (!gamma_host || !cu_rows || !target_logits || !u_resample || !out || !workspace)
    return fail(GS_EINVAL, "null argument");
  if (!out->accepted_len || !out->next_token || !out->accept_stat)
    return fail(GS_EINVAL, "accepted_len, next_token and accept_stat outputs are required");
  long n_rows = 0, n_draft = 0;
  for (int i = 0; i < n_servers; ++i) {
    if (gamma_host[i] < 0) return fail(GS_EINVAL, "gamma[%d] = %d is negative", i, gamma_host[i]);
    n_rows += gamma_host[i] + 1;
    n_draft += gamma_host[i];
  }
  if (n_rows > kMaxAcceptRows) return fail(GS_EINVAL, "too many rows (at most %ld)", kMaxAcceptRows);
  if (n_draft > 0 && (!q_probs || !draft_tokens || !u_accept))
    return fail(GS_EINVAL, "q_probs, draft_tokens and u_accept are required when any gamma > 0");
  if (workspace_bytes < accept_workspace_bytes(n_servers, (int)n_rows, vocab))
    return fail(GS_ECAPACITY, "workspace of %zu bytes is smaller than gs_accept_workspace_bytes", workspace_bytes);
  return launch_accept(n_servers, (int)n_rows, cu_rows, vocab, elem, target_logits, q_probs, draft_tokens, u_accept,
                       u_resample, out, workspace, static_cast<hipStream_t>(hip_stream), nullptr, 0);
}

}  // namespace
}  // namespace gs

extern "C" gs_status gs_accept_reject(int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                                      const float* target_logits, const float* q_probs, const int* draft_tokens,
                                      const float* u_accept, const float* u_resample, const gs_accept_out* out,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  return gs::accept_entry(GS_F32, n_servers, gamma_host, cu_rows, vocab, target_logits, q_probs, draft_tokens, u_accept,
                          u_resample, out, workspace, workspace_bytes, hip_stream);
}

extern "C" gs_status gs_accept_reject_bf16(int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                                           const void* target_logits, const void* q_probs, const int* draft_tokens,
                                           const float* u_accept, const float* u_resample, const gs_accept_out* out,
                                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  return gs::accept_entry(GS_BF16, n_servers, gamma_host, cu_rows, vocab, target_logits, q_probs, draft_tokens,
                          u_accept, u_resample, out, workspace, workspace_bytes, hip_stream);
}

// ---------------------------------------------------------------------------------------
// gs_accept_reject_static: the same kernels with their workspace in a device array that is part of the
// library image, for callers that cannot allocate.  The array's name is a host-side stand-in, not a
// device address: its address on the current device is looked up once per device and kept.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[GS_ACCEPT_STATIC_SCRATCH_BYTES];

namespace gs {
namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};     // device address of `scratch` per device, filled on first use

gs_status static_scratch(void** out) {
  int dev = -1;
  GS_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(GS_EUNSUPPORTED, "device index %d is beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    GS_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(GS_EDEVICE, "hipGetSymbolAddress returned a null address for the static scratch");
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return GS_OK;
}

}  // namespace
}  // namespace gs

extern "C" gs_status gs_accept_reject_static(int n_servers, const int* gamma_host, const int* cu_rows, int vocab,
                                             const float* target_logits, const float* q_probs,
                                             const int* draft_tokens, const float* u_accept,
                                             const float* u_resample, const gs_accept_out* out, void* hip_stream) {
  if (n_servers <= 0 || vocab <= 0) return gs::fail(GS_EINVAL, "n_servers and vocab must be positive");
  if (!gamma_host) return gs::fail(GS_EINVAL, "null argument");
  long n_rows = 0;
  for (int i = 0; i < n_servers; ++i) {
    if (gamma_host[i] < 0) return gs::fail(GS_EINVAL, "gamma[%d] = %d is negative", i, gamma_host[i]);
    n_rows += gamma_host[i] + 1;
  }
  if (n_rows > gs::kMaxAcceptRows) return gs::fail(GS_EINVAL, "too many rows");
  const size_t need = gs::accept_workspace_bytes(n_servers, (int)n_rows, vocab);
  if (need > GS_ACCEPT_STATIC_SCRATCH_BYTES)
    return gs::fail(GS_ECAPACITY, "this batch needs %zu bytes of scratch, the static array holds %zu", need,
                    (size_t)GS_ACCEPT_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  const gs_status st = gs::static_scratch(&ws);
  if (st != GS_OK) return st;
  return gs_accept_reject(n_servers, gamma_host, cu_rows, vocab, target_logits, q_probs, draft_tokens, u_accept,
                          u_resample, out, ws, GS_ACCEPT_STATIC_SCRATCH_BYTES, hip_stream);
}
