// Dense projections Y = X * W^T of the decoder (QKV, O, gate/up, down, LM head).
//
// bf16 path (MFMA): the verify step has few rows (tens to a few hundred) against
// matrices of 10^7..10^9 weights, so every weight byte is used by only M rows: the kernel
// is a weight-streaming kernel bound by HBM, and the layout serves the stream:
//   * the weights are stored tile-packed (gs_pack_weight): the 2 KB that one wavefront needs
//     per 64-wide k step for its 16 output columns is contiguous, and the blocks are ordered
//     [k_step][n_tile][half][lane][8 bf16]: at one k step the blocks of neighbouring column tiles
//     follow each other, so the waves of the whole launch, which advance through k at about the
//     same pace, sweep one contiguous band of memory at a time (the access pattern of a plain
//     copy, which keeps DRAM pages open) instead of thousands of unrelated 2 KB pieces.  Each
//     wave issues two fully coalesced 1 KB loads per step, straight into the MFMA B operand (no
//     LDS hop for weights); DEPTH steps are kept in flight
//   * the activations (all M rows of the k step, at most 128) are staged once per workgroup
//     in LDS (padded rows: conflict-free 16-byte reads) and shared by the four waves; their
//     global loads run DEPTH steps ahead as well, so a step never waits on the L2 round trip
//   * K is split across workgroups when N alone gives too few of them to fill 256 CUs; the
//     fp32 partial sums [S][M][N] are summed by the consumer kernel, in a fixed order
//   * the gate/up projection, where it runs without a K split, applies the SwiGLU in its epilogue and
//     stores the bf16 activation instead of fp32 sums (gemm_bf16_gate_up_kernel, GATE_UP of the tall kernel).
// k order inside a step is permuted identically for both operands (lane group g takes
// k = 16g .. 16g+15, first half to the first MFMA, second half to the second), which leaves
// the dot products unchanged.  Measured without the activation side, on the gate/up shape: 6.2 TB/s
// in this order, 5.4 TB/s with each tile's k steps contiguous, 4.4 TB/s for row-major weight rows.
//
// fp32 path: plain LDS-tiled FMA kernel for the small fp32 configuration.
#include "common.h"
#include "device_types.h"

namespace gs {
namespace {

// 16-byte load that does not displace cache lines: weights that a launch reads once (measured on the 8B shape
// at 50 rows: 4.52 instead of 4.56 ms per step)
typedef unsigned int uint4_vec __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
  const uint4_vec v = __builtin_nontemporal_load(reinterpret_cast<const uint4_vec*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int kSkinnyDepth = 4;     // k steps of weights and activations in flight per wave
constexpr int kTargetWorkgroups = 512;   // about two per CU
constexpr int kBK = 64;           // k elements per step
constexpr int kLdsRow = kBK + 8;  // padded LDS row (bf16 elements): 144 bytes

// Merge of two online-softmax pairs (max, sum exp(x - max)).
__device__ __forceinline__ void merge_stat(float& m, float& s, float m2, float s2) {
  const float M = fmaxf(m, m2);
  s = s * __expf(m - M) + s2 * __expf(m2 - M);
  m = M;
}

// Reductions over the 16 lanes of a DPP row (lanes 16 g .. 16 g + 15) with data-parallel-primitive moves, which
// are modifiers of ordinary vector instructions (a shuffle through the LDS crossbar costs an LDS instruction
// each): neighbours in a quad, the other pair of the quad, the mirrored quad of the half row, the mirrored half.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));      // quad_perm(1, 0, 3, 2)
  v = fmaxf(v, dpp_move<0x4E>(v));      // quad_perm(2, 3, 0, 1)
  v = fmaxf(v, dpp_move<0x141>(v));     // row_half_mirror
  return fmaxf(v, dpp_move<0x140>(v));  // row_mirror
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  return v + dpp_move<0x140>(v);
}

// STATS (LM head, one K split): the epilogue also reduces every output row over the workgroup's columns to the
// pair (max, sum exp(y - max)) and stores it at stats[row][column block], so that the vocabulary softmax
// statistics (Section II-A-1) come out of the projection and the logits need not be read again for them.
template <int MT, int DEPTH, int NW, bool STATS = false>
__global__ __launch_bounds__(64 * NW) void gemm_bf16_skinny_kernel(const bf16_t* __restrict__ X,
                                                                   const bf16_t* __restrict__ Wp,
                                                                   float* __restrict__ P, int M, int N, int K,
                                                                   int k_per_split, int m_chunks,
                                                                   float2* __restrict__ stats = nullptr,
                                                                   int n_stat_blocks = 0) {
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][MT * 16 * kLdsRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;
  // More rows than one workgroup takes (MT * 16): the row chunks of one column block are separate
  // workgroups that read the same weights.  Workgroups are handed to the 8 XCDs round robin by
  // their linear index, so the chunks of a column block get indices that are 8 apart: they land on
  // the same XCD one after the other, and all but the first read the weights from that XCD's L2.
  int n_block = blockIdx.x, m_chunk = 0;
  if (m_chunks > 1) {
    const int xcd = blockIdx.x & 7, t = blockIdx.x >> 3;
    m_chunk = t % m_chunks;
    n_block = (t / m_chunks) * 8 + xcd;
    if (n_block * (16 * NW) >= N) return;      // padding of the grid to a multiple of 8 column blocks
  }
  const int n_tile = n_block * NW + wave;
  const int n0 = n_tile * 16;
  const int split = blockIdx.y;
  const int m0 = m_chunk * (MT * 16);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_steps = (k_end - k_begin) / kBK;

  // activation tile: MT*16 rows x 64 k = MT*128 chunks of 16 bytes
  constexpr int kChunks = MT * 128;
  constexpr int kGemmThreads = 64 * NW;
  constexpr int kPasses = (kChunks + kGemmThreads - 1) / kGemmThreads;
  uint4 xreg[DEPTH][kPasses];
  auto load_x = [&](int slot, int step) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * kGemmThreads;
      const int row = ch >> 3, col = (ch & 7) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ch < kChunks && m0 + row < M)
        v = *reinterpret_cast<const uint4*>(X + (size_t)(m0 + row) * K + k_begin + step * kBK + col);
      xreg[slot][p] = v;
    }
  };
  auto store_x = [&](int buf, int slot) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * kGemmThreads;
      const int row = ch >> 3, col = (ch & 7) * 8;
      if (ch < kChunks) *reinterpret_cast<uint4*>(&xs[buf][row * kLdsRow + col]) = xreg[slot][p];
    }
  };

  // packed weights: block (n_tile, k_step) is 128 uint4; lane l reads uint4 l (first half of its
  // 16 k values) and uint4 64 + l (second half)
  const size_t w_step_stride = (size_t)(N / 16) * 128;
  const uint4* wbase = reinterpret_cast<const uint4*>(Wp) + (size_t)(k_begin / kBK) * w_step_stride + (size_t)n_tile * 128 + lane;
  uint4 wreg[DEPTH][2];
  auto load_w = [&](int slot, int step) {
    const uint4* p = wbase + (size_t)step * w_step_stride;
    if (m_chunks == 1) {      // read once: do not displace the activations and partial sums in L2
      wreg[slot][0] = stream_load(p);
      wreg[slot][1] = stream_load(p + 64);
    } else {                  // the other row chunks of the column block read the same weights from L2
      wreg[slot][0] = p[0];
      wreg[slot][1] = p[64];
    }
  };

  floatx4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < n_steps) {
      load_w(d, d);
      load_x(d, d);
    }

  for (int base = 0; base < n_steps; base += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int step = base + d;
      if (step < n_steps) {
        const int buf = step & 1;
        store_x(buf, d);
        __syncthreads();
        const uint4 w0 = wreg[d][0], w1 = wreg[d][1];
        if (step + DEPTH < n_steps) {
          load_w(d, step + DEPTH);
          load_x(d, step + DEPTH);
        }
        const bf16x8_t b0 = *reinterpret_cast<const bf16x8_t*>(&w0);
        const bf16x8_t b1 = *reinterpret_cast<const bf16x8_t*>(&w1);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const bf16_t* ap = &xs[buf][(mt * 16 + c) * kLdsRow + g * 16];
          const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(ap);
          const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(ap + 8);
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b0, acc[mt], 0, 0, 0);
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1, acc[mt], 0, 0, 0);
        }
      }
    }
  }

  float* out = P + (size_t)split * M * N;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = m0 + mt * 16 + g * 4 + i;
      if (row < M) out[(size_t)row * N + n0 + c] = acc[mt][i];
    }
  }
  if constexpr (STATS) {
    // lanes (g, 0..15) hold the 16 columns of row mt*16 + g*4 + i: reduce over c, then over the waves
    __shared__ float2 st[NW][MT * 16];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float v = acc[mt][i];
        const float mx = row16_max(v);
        const float e = row16_sum(__expf(v - mx));
        if (c == 0) st[wave][mt * 16 + g * 4 + i] = make_float2(mx, e);
      }
    __syncthreads();
    if (tid < MT * 16 && m0 + tid < M) {
      float m = st[0][tid].x, sum = st[0][tid].y;
#pragma unroll
      for (int w = 1; w < NW; ++w) merge_stat(m, sum, st[w][tid].x, st[w][tid].y);
      stats[(size_t)(m0 + tid) * n_stat_blocks + n_block] = make_float2(m, sum);
    }
  }
}

// Gate/up projection with the SwiGLU in its epilogue (up to 64 rows): act[r][f] = silu(X W_gate^T) * (X W_up^T)
// with W = [gate rows; up rows] ([2F][K], packed).  A wave owns feature tile t of both halves (column tiles
// t and F/16 + t of the packed matrix), so the gate and the up value of an output sit in the same register
// of the same lane; K is not split, so the sums are complete when the loop ends and the fp32 partial result
// ([splits][R][2F], written and read back by a separate kernel otherwise) never exists.  grid F / (16 NW).
template <int MT, int DEPTH, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_bf16_gate_up_kernel(const bf16_t* __restrict__ X,
                                                                    const bf16_t* __restrict__ Wp,
                                                                    bf16_t* __restrict__ act, int M, int F, int K) {
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][MT * 16 * kLdsRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;
  const int f_tile = blockIdx.x * NW + wave;
  const int n_steps = K / kBK;

  constexpr int kChunks = MT * 128;
  constexpr int kGemmThreads = 64 * NW;
  constexpr int kPasses = (kChunks + kGemmThreads - 1) / kGemmThreads;
  uint4 xreg[DEPTH][kPasses];
  auto load_x = [&](int slot, int step) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * kGemmThreads;
      const int row = ch >> 3, col = (ch & 7) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ch < kChunks && row < M) v = *reinterpret_cast<const uint4*>(X + (size_t)row * K + step * kBK + col);
      xreg[slot][p] = v;
    }
  };
  auto store_x = [&](int buf, int slot) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * kGemmThreads;
      const int row = ch >> 3, col = (ch & 7) * 8;
      if (ch < kChunks) *reinterpret_cast<uint4*>(&xs[buf][row * kLdsRow + col]) = xreg[slot][p];
    }
  };
  const size_t w_step_stride = (size_t)(2 * F / 16) * 128;
  const uint4* wgate = reinterpret_cast<const uint4*>(Wp) + (size_t)f_tile * 128 + lane;
  const uint4* wup = wgate + (size_t)(F / 16) * 128;
  uint4 wreg[DEPTH][2][2];
  auto load_w = [&](int slot, int step) {
    const size_t o = (size_t)step * w_step_stride;
    wreg[slot][0][0] = stream_load(wgate + o);
    wreg[slot][0][1] = stream_load(wgate + o + 64);
    wreg[slot][1][0] = stream_load(wup + o);
    wreg[slot][1][1] = stream_load(wup + o + 64);
  };
  floatx4_t acc_g[MT], acc_u[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc_g[mt] = acc_u[mt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < n_steps) {
      load_w(d, d);
      load_x(d, d);
    }
  for (int base = 0; base < n_steps; base += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int step = base + d;
      if (step < n_steps) {
        const int buf = step & 1;
        store_x(buf, d);
        __syncthreads();
        const uint4 g0 = wreg[d][0][0], g1 = wreg[d][0][1], u0 = wreg[d][1][0], u1 = wreg[d][1][1];
        if (step + DEPTH < n_steps) {
          load_w(d, step + DEPTH);
          load_x(d, step + DEPTH);
        }
        const bf16x8_t bg0 = *reinterpret_cast<const bf16x8_t*>(&g0), bg1 = *reinterpret_cast<const bf16x8_t*>(&g1);
        const bf16x8_t bu0 = *reinterpret_cast<const bf16x8_t*>(&u0), bu1 = *reinterpret_cast<const bf16x8_t*>(&u1);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const bf16_t* ap = &xs[buf][(mt * 16 + c) * kLdsRow + g * 16];
          const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(ap);
          const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(ap + 8);
          acc_g[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bg0, acc_g[mt], 0, 0, 0);
          acc_u[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bu0, acc_u[mt], 0, 0, 0);
          acc_g[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bg1, acc_g[mt], 0, 0, 0);
          acc_u[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bu1, acc_u[mt], 0, 0, 0);
        }
      }
    }
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = mt * 16 + g * 4 + i;
      const float gt = acc_g[mt][i];
      if (row < M) act[(size_t)row * F + f_tile * 16 + c] = float_to_bf16(gt / (1.0f + expf(-gt)) * acc_u[mt][i]);
    }
  }
}

// More than 64 rows (a few hundred per step with tens of draft servers): the same streaming design
// with a taller and wider wave tile.  A wave owns NT column tiles and all MT * 16 rows of its row
// chunk, so every activation fragment read from LDS feeds NT MFMAs and every weight fragment MT of
// them; a workgroup covers NT * 64 columns.  Two shapes are used: (MT <= 10, NT = 2, two steps of
// prefetch) while the weight stream still matters (up to a few hundred rows), and (MT = 8, NT = 4, no
// register prefetch: the second wave on each SIMD hides the latency) for row counts where the MFMA
// pipes are the bound.  Both fit two waves per SIMD.
// Row chunks of one column block are separate workgroups that read the same weights: workgroups are
// handed to the 8 XCDs round robin by their linear index, so the chunks of a column block get indices
// that are 8 apart and land on the same XCD one after the other, and all but the first find the weights
// in that XCD's L2.  grid (ceil(N / (64 NT) / 8) * 8 * m_chunks, S).
// GATE_UP (NT = 2, one K split): the wave's two column tiles are feature tile t of the gate half and of the
// up half of a [2F][K] matrix, and the epilogue stores act[r][f] = silu(gate) * up as bf16 ([M][N/2], at P)
// instead of the fp32 sums.
// STATS: as in the skinny kernel, (max, sum exp) of every row over the workgroup's 64 NT columns.
template <int MT, int NT, int DEPTH, bool GATE_UP = false, bool STATS = false>
__global__ __launch_bounds__(256, 2) void gemm_bf16_tall_kernel(const bf16_t* __restrict__ X,
                                                                const bf16_t* __restrict__ Wp,
                                                                float* __restrict__ P, int M, int N, int K,
                                                                int k_per_split, int m_chunks,
                                                                float2* __restrict__ stats = nullptr,
                                                                int n_stat_blocks = 0) {
  static_assert(!GATE_UP || NT % 2 == 0, "gate and up tile of every feature tile");
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][MT * 16 * kLdsRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;
  const int xcd = blockIdx.x & 7, t = blockIdx.x >> 3;
  const int m_chunk = t % m_chunks;
  const int n_block = (t / m_chunks) * 8 + xcd;
  if (n_block * (64 * NT) >= N) return;        // padding of the grid to a multiple of 8 column blocks
  // first column tile of the wave; with GATE_UP its tiles are NT/2 neighbouring feature tiles of the gate
  // half followed by the same ones of the up half (N/32 tiles further)
  const int n_tile0 = GATE_UP ? (n_block * 4 + wave) * (NT / 2) : (n_block * 4 + wave) * NT;
  auto tile_offset = [&](int nt) { return GATE_UP ? (nt % (NT / 2)) + (nt / (NT / 2)) * (N / 32) : nt; };
  const int split = blockIdx.y;
  const int m0 = m_chunk * (MT * 16);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_steps = (k_end - k_begin) / kBK;

  constexpr int kChunks = MT * 128;
  constexpr int kPasses = (kChunks + 255) / 256;
  uint4 xreg[DEPTH][kPasses];
  auto load_x = [&](int slot, int step) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * 256;
      const int row = ch >> 3, col = (ch & 7) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ch < kChunks && m0 + row < M)
        v = *reinterpret_cast<const uint4*>(X + (size_t)(m0 + row) * K + k_begin + step * kBK + col);
      xreg[slot][p] = v;
    }
  };
  auto store_x = [&](int buf, int slot) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * 256;
      const int row = ch >> 3, col = (ch & 7) * 8;
      if (ch < kChunks) *reinterpret_cast<uint4*>(&xs[buf][row * kLdsRow + col]) = xreg[slot][p];
    }
  };
  const size_t w_step_stride = (size_t)(N / 16) * 128;
  const uint4* wbase = reinterpret_cast<const uint4*>(Wp) + (size_t)(k_begin / kBK) * w_step_stride + (size_t)n_tile0 * 128 + lane;
  uint4 wreg[DEPTH][NT][2];
  auto load_w = [&](int slot, int step) {
    const uint4* p = wbase + (size_t)step * w_step_stride;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      wreg[slot][nt][0] = p[(size_t)tile_offset(nt) * 128];
      wreg[slot][nt][1] = p[(size_t)tile_offset(nt) * 128 + 64];
    }
  };

  floatx4_t acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < n_steps) {
      load_w(d, d);
      load_x(d, d);
    }
  for (int base = 0; base < n_steps; base += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int step = base + d;
      if (step < n_steps) {
        const int buf = step & 1;
        store_x(buf, d);
        __syncthreads();
        if (step + DEPTH < n_steps) load_x(d, step + DEPTH);
        bf16x8_t b[NT][2];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          b[nt][0] = *reinterpret_cast<const bf16x8_t*>(&wreg[d][nt][0]);
          b[nt][1] = *reinterpret_cast<const bf16x8_t*>(&wreg[d][nt][1]);
        }
        if (step + DEPTH < n_steps) load_w(d, step + DEPTH);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const bf16_t* ap = &xs[buf][(mt * 16 + c) * kLdsRow + g * 16];
          const bf16x8_t a0 = *reinterpret_cast<const bf16x8_t*>(ap);
          const bf16x8_t a1 = *reinterpret_cast<const bf16x8_t*>(ap + 8);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b[nt][0], acc[mt][nt], 0, 0, 0);
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b[nt][1], acc[mt][nt], 0, 0, 0);
          }
        }
      }
    }
  }

  if constexpr (GATE_UP) {
    bf16_t* act = reinterpret_cast<bf16_t*>(P);
    const int F = N / 2;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = m0 + mt * 16 + g * 4 + i;
        if (row < M) {
#pragma unroll
          for (int ft = 0; ft < NT / 2; ++ft) {
            const float gt = acc[mt][ft][i];
            act[(size_t)row * F + (n_tile0 + ft) * 16 + c] = float_to_bf16(gt / (1.0f + expf(-gt)) * acc[mt][NT / 2 + ft][i]);
          }
        }
      }
    return;
  }
  float* out = P + (size_t)split * M * N;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = m0 + mt * 16 + g * 4 + i;
      if (row < M) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) out[(size_t)row * N + (n_tile0 + nt) * 16 + c] = acc[mt][nt][i];
      }
    }
  if constexpr (STATS) {
    __shared__ float2 st[4][MT * 16];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float mx = acc[mt][0][i];
#pragma unroll
        for (int nt = 1; nt < NT; ++nt) mx = fmaxf(mx, acc[mt][nt][i]);
        mx = row16_max(mx);
        float e = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) e += __expf(acc[mt][nt][i] - mx);
        e = row16_sum(e);
        if (c == 0) st[wave][mt * 16 + g * 4 + i] = make_float2(mx, e);
      }
    __syncthreads();
    for (int r = tid; r < MT * 16; r += 256)
      if (m0 + r < M) {
        float m = st[0][r].x, sum = st[0][r].y;
#pragma unroll
        for (int w = 1; w < 4; ++w) merge_stat(m, sum, st[w][r].x, st[w][r].y);
        stats[(size_t)(m0 + r) * n_stat_blocks + n_block] = make_float2(m, sum);
      }
  }
}

// fp32: 64x64 output tile, k step 16, each of 256 threads owns a 4x4 block.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                       float* __restrict__ Y, int M, int N, int K) {
  __shared__ float xs[16][64 + 1], ws[16][64 + 1];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int e = tid; e < 64 * 16; e += 256) {
      const int r = e >> 4, kk = e & 15;
      xs[kk][r] = (m0 + r < M && k0 + kk < K) ? X[(size_t)(m0 + r) * K + k0 + kk] : 0.f;
      ws[kk][r] = (n0 + r < N && k0 + kk < K) ? W[(size_t)(n0 + r) * K + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = xs[kk][ty * 4 + i];
        b[i] = ws[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = m0 + ty * 4 + i, cc = n0 + tx * 4 + j;
      if (r < M && cc < N) Y[(size_t)r * N + cc] = acc[i][j];
    }
}

// Row-major [N][K] bf16 -> tile-packed [K/64][N/16][2][64][8]: one thread moves one 16-byte piece.
__global__ __launch_bounds__(256) void pack_weight_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                          int N, int K) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;      // destination uint4 index
  const size_t total = (size_t)N * K / 8;
  if (idx >= total) return;
  const int lane = (int)(idx & 63), half = (int)((idx >> 6) & 1);
  const size_t block = idx >> 7;
  const int n_tiles = N / 16;
  const int n_tile = (int)(block % n_tiles), k_step = (int)(block / n_tiles);
  const int g = lane >> 4, c = lane & 15;
  const size_t row = (size_t)n_tile * 16 + c;
  const int k = k_step * kBK + g * 16 + half * 8;
  dst[idx] = src[(row * K + k) / 8];
}

}  // namespace

gs_status launch_pack_weight(const void* src, void* dst, int N, int K, hipStream_t stream) {
  const size_t total = (size_t)N * K / 8;
  pack_weight_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(static_cast<const uint4*>(src),
                                                                          static_cast<uint4*>(dst), N, K);
  GS_LAUNCH_CHECK("pack_weight");
  return GS_OK;
}

// Which bf16 kernel serves a shape, and how the launch is cut.
struct GemmPlan {
  bool tall;      // gemm_bf16_tall_kernel (more than 64 rows, N a multiple of 128)
  int waves;      // skinny: waves per workgroup (4 or 8)
  int mt;         // row tiles per workgroup
  int nt;         // tall: column tiles per wave (2 or 4)
  int m_chunks;   // row chunks (separate workgroups)
  int splits;     // K splits
  int k_per;      // k elements per split (multiple of 64)
};

static GemmPlan gemm_plan(int M, int N, int K) {
  GemmPlan p;
  const int tiles = ceil_div(M, 16);
  p.tall = tiles > 4 && N % 128 == 0;
  p.nt = 1;
  int n_blocks;
  if (p.tall && tiles >= 40 && N % 256 == 0) {        // 640 rows and more: MFMA-bound shape
    p.waves = 4;
    p.nt = 4;
    p.mt = 8;
    p.m_chunks = ceil_div(tiles, 8);
    n_blocks = N / 256;
  } else if (p.tall) {
    p.waves = 4;
    p.nt = 2;
    p.m_chunks = ceil_div(tiles, 10);
    const int per = ceil_div(tiles, p.m_chunks);      // 3 .. 10 row tiles per chunk
    p.mt = per <= 6 ? 6 : per <= 8 ? 8 : 10;
    p.m_chunks = ceil_div(tiles, p.mt);
    n_blocks = N / 128;
  } else {
    // wide matrices get 8 waves (128 columns per workgroup), which halves the number of times the
    // activation rows are re-read from L2; narrower ones keep 4 so that the launch still has
    // enough workgroups
    p.waves = (N % 128 == 0 && N / 128 >= 192) ? 8 : 4;
    p.mt = tiles <= 1 ? 1 : tiles <= 2 ? 2 : tiles <= 4 ? 4 : 8;
    p.m_chunks = ceil_div(tiles, p.mt);
    n_blocks = N / (16 * p.waves);
  }
  const int wgs = n_blocks * p.m_chunks;
  int want = (kTargetWorkgroups + wgs / 2) / wgs;                // about two workgroups per CU
  const int max_s = K / 512 > 0 ? K / 512 : 1;             // at least 8 steps per split
  int s = want < max_s ? want : max_s;
  if (s < 1) s = 1;
  p.k_per = ceil_div(ceil_div(K, s), kBK) * kBK;
  p.splits = ceil_div(K, p.k_per);
  return p;
}

int gemm_w4_splits(int M, int N, int K);
gs_status launch_gemm_w4(const void* X, const void* Wpacked, float* P, int M, int N, int K, hipStream_t stream);

// Number of K splits the projection kernel will use for this shape (1 for fp32).
int gemm_splits(int dtype, int M, int N, int K) {
  if (M <= 0) return 1;
  if (dtype == GS_W4) return gemm_w4_splits(M, N, K);
  if (dtype != GS_BF16) return 1;
  return gemm_plan(M, N, K).splits;
}

template <int NW>
static void launch_skinny(const GemmPlan& p, const bf16_t* x, const bf16_t* w, float* P, int M, int N, int K,
                          hipStream_t stream) {
  const int n_blocks = N / (16 * NW);
  const int gx = p.m_chunks > 1 ? ceil_div(n_blocks, 8) * 8 * p.m_chunks : n_blocks;
  const dim3 grid(gx, p.splits, 1);
  switch (p.mt) {
    case 1: gemm_bf16_skinny_kernel<1, kSkinnyDepth, NW><<<grid, 64 * NW, 0, stream>>>(x, w, P, M, N, K, p.k_per, 1); break;
    case 2: gemm_bf16_skinny_kernel<2, kSkinnyDepth, NW><<<grid, 64 * NW, 0, stream>>>(x, w, P, M, N, K, p.k_per, 1); break;
    case 4: gemm_bf16_skinny_kernel<4, kSkinnyDepth, NW><<<grid, 64 * NW, 0, stream>>>(x, w, P, M, N, K, p.k_per, 1); break;
    default:
      gemm_bf16_skinny_kernel<8, kSkinnyDepth, NW><<<grid, 64 * NW, 0, stream>>>(x, w, P, M, N, K, p.k_per, p.m_chunks);
  }
}

static void launch_tall(const GemmPlan& p, const bf16_t* x, const bf16_t* w, float* P, int M, int N, int K,
                        hipStream_t stream) {
  const dim3 grid(ceil_div(N / (64 * p.nt), 8) * 8 * p.m_chunks, p.splits, 1);
  if (p.nt == 4) {
    gemm_bf16_tall_kernel<8, 4, 1><<<grid, 256, 0, stream>>>(x, w, P, M, N, K, p.k_per, p.m_chunks);
    return;
  }
  switch (p.mt) {
    case 6: gemm_bf16_tall_kernel<6, 2, 2><<<grid, 256, 0, stream>>>(x, w, P, M, N, K, p.k_per, p.m_chunks); break;
    case 8: gemm_bf16_tall_kernel<8, 2, 2><<<grid, 256, 0, stream>>>(x, w, P, M, N, K, p.k_per, p.m_chunks); break;
    default: gemm_bf16_tall_kernel<10, 2, 2><<<grid, 256, 0, stream>>>(x, w, P, M, N, K, p.k_per, p.m_chunks);
  }
}

// Gate/up with the SwiGLU fused: 4 waves (64 features per workgroup; 224 workgroups for F = 14336, each wave
// streaming 256 KB without a K split), weights fetched 6 steps ahead (with 4 the unsplit kernel is 4.5 us
// slower than the split one on the 8B shape, with 6 it is 1.3 us slower and the 6 us of the separate SwiGLU
// kernel and its launch boundary are gone; 2 waves double the activation re-reads, 8 leave half the CUs idle).
constexpr int kGateUpWaves = 4;
constexpr int kGateUpDepth = 6;

// Whether the gate/up projection of this shape runs with the SwiGLU fused: bf16, and either up to 64 rows or
// a shape that the tall kernel serves without a K split anyway.
bool gate_up_fused(int dtype, int M, int F, int K) {
  if (dtype != GS_BF16 || M <= 0 || F % (16 * kGateUpWaves) != 0 || K % kBK != 0) return false;
  if (M <= 64) return true;
  const GemmPlan p = gemm_plan(M, 2 * F, K);
  return p.tall && p.splits == 1;
}

// act [M][F] (bf16) = silu(X Wg^T) * (X Wu^T), W = [Wg; Wu] packed; only for shapes gate_up_fused accepts.
gs_status launch_gemm_gate_up(const void* X, const void* W, void* act, int M, int F, int K, hipStream_t stream) {
  constexpr int NW = kGateUpWaves, D = kGateUpDepth;
  const bf16_t* x = static_cast<const bf16_t*>(X);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  bf16_t* a = static_cast<bf16_t*>(act);
  const int tiles = ceil_div(M, 16);
  if (tiles > 4) {      // tall kernel, one K split, gate and up tile per wave
    const GemmPlan p = gemm_plan(M, 2 * F, K);
    const dim3 grid(ceil_div(2 * F / (64 * p.nt), 8) * 8 * p.m_chunks, 1, 1);
    float* out = static_cast<float*>(act);
    if (p.nt == 4) {
      gemm_bf16_tall_kernel<8, 4, 1, true><<<grid, 256, 0, stream>>>(x, w, out, M, 2 * F, K, K, p.m_chunks);
      GS_LAUNCH_CHECK("gemm_gate_up_tall");
      return GS_OK;
    }
    switch (p.mt) {
      case 6: gemm_bf16_tall_kernel<6, 2, 2, true><<<grid, 256, 0, stream>>>(x, w, out, M, 2 * F, K, K, p.m_chunks); break;
      case 8: gemm_bf16_tall_kernel<8, 2, 2, true><<<grid, 256, 0, stream>>>(x, w, out, M, 2 * F, K, K, p.m_chunks); break;
      default: gemm_bf16_tall_kernel<10, 2, 2, true><<<grid, 256, 0, stream>>>(x, w, out, M, 2 * F, K, K, p.m_chunks);
    }
    GS_LAUNCH_CHECK("gemm_gate_up_tall");
    return GS_OK;
  }
  const int grid = F / (16 * NW);
  if (tiles <= 1) gemm_bf16_gate_up_kernel<1, D, NW><<<grid, 64 * NW, 0, stream>>>(x, w, a, M, F, K);
  else if (tiles <= 2) gemm_bf16_gate_up_kernel<2, D, NW><<<grid, 64 * NW, 0, stream>>>(x, w, a, M, F, K);
  else gemm_bf16_gate_up_kernel<4, D, NW><<<grid, 64 * NW, 0, stream>>>(x, w, a, M, F, K);
  GS_LAUNCH_CHECK("gemm_gate_up");
  return GS_OK;
}

// Number of column blocks per row of the statistics that launch_gemm_stats writes for this shape, or 0 where
// the projection of this shape does not emit them (fp32 and 4-bit models, shapes that need a K split).
int gemm_stat_blocks(int dtype, int M, int N, int K) {
  if (dtype != GS_BF16 || M <= 0) return 0;
  const GemmPlan p = gemm_plan(M, N, K);
  if (p.splits != 1) return 0;
  return p.tall ? N / (64 * p.nt) : N / (16 * p.waves);
}

// Y [M][N] = X W^T (one K split) and stats [M][gemm_stat_blocks] = per row and column block (max, sum exp(y - max)).
gs_status launch_gemm_stats(const void* X, const void* W, float* Y, void* stats, int M, int N, int K,
                            hipStream_t stream) {
  const GemmPlan p = gemm_plan(M, N, K);
  const bf16_t* x = static_cast<const bf16_t*>(X);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  float2* st = static_cast<float2*>(stats);
  const int nb = gemm_stat_blocks(GS_BF16, M, N, K);
  if (nb == 0) return fail(GS_EUNSUPPORTED, "this projection shape does not emit softmax statistics");
  if (p.tall) {
    const dim3 grid(ceil_div(N / (64 * p.nt), 8) * 8 * p.m_chunks, 1, 1);
    if (p.nt == 4) gemm_bf16_tall_kernel<8, 4, 1, false, true><<<grid, 256, 0, stream>>>(x, w, Y, M, N, K, p.k_per, p.m_chunks, st, nb);
    else if (p.mt == 6) gemm_bf16_tall_kernel<6, 2, 2, false, true><<<grid, 256, 0, stream>>>(x, w, Y, M, N, K, p.k_per, p.m_chunks, st, nb);
    else if (p.mt == 8) gemm_bf16_tall_kernel<8, 2, 2, false, true><<<grid, 256, 0, stream>>>(x, w, Y, M, N, K, p.k_per, p.m_chunks, st, nb);
    else gemm_bf16_tall_kernel<10, 2, 2, false, true><<<grid, 256, 0, stream>>>(x, w, Y, M, N, K, p.k_per, p.m_chunks, st, nb);
  } else {
    const int n_blocks = N / (16 * p.waves);
    const int gx = p.m_chunks > 1 ? ceil_div(n_blocks, 8) * 8 * p.m_chunks : n_blocks;
    const dim3 grid(gx, 1, 1);
    const int mc = p.mt == 8 ? p.m_chunks : 1;
#define GS_SKINNY_STATS(MT_, NW_) \
  gemm_bf16_skinny_kernel<MT_, kSkinnyDepth, NW_, true><<<grid, 64 * NW_, 0, stream>>>(x, w, Y, M, N, K, p.k_per, mc, st, nb)
    if (p.waves == 8) {
      switch (p.mt) {
        case 1: GS_SKINNY_STATS(1, 8); break;
        case 2: GS_SKINNY_STATS(2, 8); break;
        case 4: GS_SKINNY_STATS(4, 8); break;
        default: GS_SKINNY_STATS(8, 8);
      }
    } else {
      switch (p.mt) {
        case 1: GS_SKINNY_STATS(1, 4); break;
        case 2: GS_SKINNY_STATS(2, 4); break;
        case 4: GS_SKINNY_STATS(4, 4); break;
        default: GS_SKINNY_STATS(8, 4);
      }
    }
#undef GS_SKINNY_STATS
  }
  GS_LAUNCH_CHECK("gemm_bf16_stats");
  return GS_OK;
}

// P [splits][M][N] fp32 partial sums of X [M][K] * W[N][K]^T (W tile-packed for bf16, packed 4-bit for
// GS_W4 with bf16 activations, row-major for fp32).
gs_status launch_gemm(int dtype, const void* X, const void* W, float* P, int M, int N, int K, hipStream_t stream) {
  if (M <= 0) return GS_OK;
  if (dtype == GS_W4) return launch_gemm_w4(X, W, P, M, N, K, stream);
  if (dtype == GS_BF16) {
    const GemmPlan p = gemm_plan(M, N, K);
    const bf16_t* x = static_cast<const bf16_t*>(X);
    const bf16_t* w = static_cast<const bf16_t*>(W);
    if (p.tall) launch_tall(p, x, w, P, M, N, K, stream);
    else if (p.waves == 8) launch_skinny<8>(p, x, w, P, M, N, K, stream);
    else launch_skinny<4>(p, x, w, P, M, N, K, stream);
    GS_LAUNCH_CHECK("gemm_bf16");
  } else {
    gemm_f32_kernel<<<dim3(ceil_div(N, 64), ceil_div(M, 64)), 256, 0, stream>>>(
        static_cast<const float*>(X), static_cast<const float*>(W), P, M, N, K);
    GS_LAUNCH_CHECK("gemm_f32");
  }
  return GS_OK;
}

}  // namespace gs
