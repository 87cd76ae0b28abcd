// Projections with 4-bit weights (weight-only quantisation in groups of 128 inputs, the format family of
// the AWQ checkpoints the paper's 70B verifier uses, Section IV-A): Y = X * W^T with
// W[n][k] = (code[n][k] - zero[n][k/128]) * scale[n][k/128], codes and zeros in 0..15, scales bf16.
//
// Same streaming design as the bf16 kernel, with a quarter of the weight bytes: a wave owns 16 output
// columns and reads, per 64-wide k step, 8 bytes per lane (16 codes of one column) plus one 32-bit word
// with the column's scale and zero point; the codes are turned into bf16 in registers and fed to the MFMA
// as the B operand.  Dequantisation: the code c becomes the bf16 bit pattern 0x4300 + c = 128 + c (exact),
// widened to fp32, then fma(128 + c, scale, -(128 + zero) * scale) = (c - zero) * scale, which is exact in
// fp32 (5 x 8 significant bits), and rounded to bf16 (nearest even) by the packed conversion: every
// dequantised weight is a function of (c, zero, scale) alone, the same on every path.
//
// Packed layout (gs_pack_weight_w4):
//   codes [K/64][N/16][64 lanes][2 words]: lane l = 16 g + c holds column c, inputs 16 g .. 16 g + 15; word 0
//         the first 8, word 1 the last 8; in a word, input 2p sits in bits 4p..4p+3 and input 2p+1 in bits
//         16+4p..16+4p+3, so that (word >> 4p) & 0x000F000F is one bf16 pair's worth of codes
//   meta  [K/128][N] words: bf16 scale in the high half, zero point in the low byte
// Activations go through LDS exactly as in the bf16 kernel.  Rows beyond 64 are served in chunks of 64 by
// separate workgroups (XCD-aware order, see the bf16 kernel); a taller tile is not built for this format.
#include "common.h"
#include "device_types.h"

namespace gs {
namespace {

constexpr int kBK = 64;
constexpr int kLdsRow = kBK + 8;
constexpr int kGroup = 128;
constexpr int kDepth = 4;

struct W4Step {
  uint2 codes;
  uint32_t meta;
};

__device__ __forceinline__ bf16x8_t dequant8(uint32_t word, float scale, float neg_c0) {
  uint4 out;
  uint32_t* o = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t pair = ((word >> (4 * p)) & 0x000F000Fu) | 0x43004300u;     // (128 + c_even, 128 + c_odd) as bf16
    const float lo = fmaf(__uint_as_float(pair << 16), scale, neg_c0);
    const float hi = fmaf(__uint_as_float(pair & 0xffff0000u), scale, neg_c0);
    o[p] = pack_bf16x2(lo, hi);
  }
  return *reinterpret_cast<const bf16x8_t*>(&out);
}

template <int MT, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_w4_skinny_kernel(const bf16_t* __restrict__ X,
                                                                 const uint2* __restrict__ codes,
                                                                 const uint32_t* __restrict__ meta,
                                                                 float* __restrict__ P, int M, int N, int K,
                                                                 int k_per_split, int m_chunks) {
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][MT * 16 * kLdsRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;
  int n_block = blockIdx.x, m_chunk = 0;
  if (m_chunks > 1) {
    const int xcd = blockIdx.x & 7, t = blockIdx.x >> 3;
    m_chunk = t % m_chunks;
    n_block = (t / m_chunks) * 8 + xcd;
    if (n_block * (16 * NW) >= N) return;
  }
  const int n_tile = n_block * NW + wave;
  const int n0 = n_tile * 16;
  const int split = blockIdx.y;
  const int m0 = m_chunk * (MT * 16);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_steps = (k_end - k_begin) / kBK;
  const int step0 = k_begin / kBK;

  constexpr int kThreads = 64 * NW;
  constexpr int kChunks = MT * 128;
  constexpr int kPasses = (kChunks + kThreads - 1) / kThreads;
  uint4 xreg[kDepth][kPasses];
  auto load_x = [&](int slot, int step) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int ch = tid + p * kThreads;
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
      const int ch = tid + p * kThreads;
      const int row = ch >> 3, col = (ch & 7) * 8;
      if (ch < kChunks) *reinterpret_cast<uint4*>(&xs[buf][row * kLdsRow + col]) = xreg[slot][p];
    }
  };
  const size_t code_stride = (size_t)(N / 16) * 64;       // uint2 per k step
  const uint2* cbase = codes + (size_t)step0 * code_stride + (size_t)n_tile * 64 + lane;
  const uint32_t* mbase = meta + n0 + c;
  W4Step wreg[kDepth];
  auto load_w = [&](int slot, int step) {
    wreg[slot].codes = cbase[(size_t)step * code_stride];
    wreg[slot].meta = mbase[(size_t)((step0 + step) >> 1) * N];
  };

  floatx4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int d = 0; d < kDepth; ++d)
    if (d < n_steps) {
      load_w(d, d);
      load_x(d, d);
    }
  for (int base = 0; base < n_steps; base += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const int step = base + d;
      if (step < n_steps) {
        const int buf = step & 1;
        store_x(buf, d);
        __syncthreads();
        const W4Step w = wreg[d];
        if (step + kDepth < n_steps) {
          load_w(d, step + kDepth);
          load_x(d, step + kDepth);
        }
        const float scale = __uint_as_float(w.meta & 0xffff0000u);
        const float neg_c0 = -(128.0f + (float)(w.meta & 0xffu)) * scale;
        const bf16x8_t b0 = dequant8(w.codes.x, scale, neg_c0);
        const bf16x8_t b1 = dequant8(w.codes.y, scale, neg_c0);
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
}

// One thread per packed code word (8 codes of one column) or per meta word.
__global__ __launch_bounds__(256) void pack_w4_kernel(const uint8_t* __restrict__ q, const bf16_t* __restrict__ scales,
                                                      const uint8_t* __restrict__ zeros, uint32_t* __restrict__ codes,
                                                      uint32_t* __restrict__ meta, int N, int K) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t n_code_words = (size_t)N * K / 8;
  const size_t n_meta = (size_t)(K / kGroup) * N;
  if (idx < n_code_words) {
    const int half = (int)(idx & 1), lane = (int)((idx >> 1) & 63);
    const size_t block = idx >> 7;
    const int n_tiles = N / 16;
    const int n_tile = (int)(block % n_tiles), k_step = (int)(block / n_tiles);
    const int g = lane >> 4, c = lane & 15;
    const uint8_t* src = q + (size_t)(n_tile * 16 + c) * K + k_step * kBK + g * 16 + half * 8;
    uint32_t w = 0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      w |= (uint32_t)(src[2 * p] & 15u) << (4 * p);
      w |= (uint32_t)(src[2 * p + 1] & 15u) << (16 + 4 * p);
    }
    codes[idx] = w;
  } else if (idx < n_code_words + n_meta) {
    const size_t j = idx - n_code_words;
    const int grp = (int)(j / N), n = (int)(j % N);
    const size_t s = (size_t)n * (K / kGroup) + grp;
    meta[j] = ((uint32_t)scales[s] << 16) | (uint32_t)(zeros[s] & 15u);
  }
}

}  // namespace

size_t w4_code_bytes(int N, int K) { return (size_t)N * K / 2; }
size_t w4_packed_bytes(int N, int K) { return w4_code_bytes(N, K) + (size_t)(K / kGroup) * N * 4; }

gs_status launch_pack_weight_w4(const void* q, const void* scales, const void* zeros, void* packed, int N, int K,
                                hipStream_t stream) {
  const size_t total = (size_t)N * K / 8 + (size_t)(K / kGroup) * N;
  uint32_t* codes = static_cast<uint32_t*>(packed);
  uint32_t* meta = reinterpret_cast<uint32_t*>(static_cast<char*>(packed) + w4_code_bytes(N, K));
  pack_w4_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(
      static_cast<const uint8_t*>(q), static_cast<const bf16_t*>(scales), static_cast<const uint8_t*>(zeros), codes,
      meta, N, K);
  GS_LAUNCH_CHECK("pack_w4");
  return GS_OK;
}

// Launch shape of the 4-bit kernel: row tiles per workgroup (1, 2 or 4), row chunks of 64, waves, K splits.
struct W4Plan {
  int mt, m_chunks, waves, splits, k_per;
};

static W4Plan w4_plan(int M, int N, int K) {
  W4Plan p;
  const int tiles = ceil_div(M, 16);
  p.mt = tiles <= 1 ? 1 : tiles <= 2 ? 2 : 4;
  p.m_chunks = ceil_div(tiles, p.mt);
  p.waves = (N % 128 == 0 && N / 128 >= 192) ? 8 : 4;
  const int wgs = N / (16 * p.waves) * p.m_chunks;
  int want = (512 + wgs / 2) / wgs;
  const int max_s = K / 512 > 0 ? K / 512 : 1;
  int s = want < max_s ? want : max_s;
  if (s < 1) s = 1;
  p.k_per = ceil_div(ceil_div(K, s), kGroup) * kGroup;      // whole groups per split
  p.splits = ceil_div(K, p.k_per);
  return p;
}

int gemm_w4_splits(int M, int N, int K) { return M <= 0 ? 1 : w4_plan(M, N, K).splits; }

template <int NW>
static void launch_w4(const W4Plan& p, const bf16_t* x, const uint2* codes, const uint32_t* meta, float* P, int M,
                      int N, int K, hipStream_t stream) {
  const int n_blocks = N / (16 * NW);
  const int gx = p.m_chunks > 1 ? ceil_div(n_blocks, 8) * 8 * p.m_chunks : n_blocks;
  const dim3 grid(gx, p.splits, 1);
  switch (p.mt) {
    case 1: gemm_w4_skinny_kernel<1, NW><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks); break;
    case 2: gemm_w4_skinny_kernel<2, NW><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks); break;
    default: gemm_w4_skinny_kernel<4, NW><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
  }
}

// P [splits][M][N] fp32 partial sums of X [M][K] (bf16) * W^T with W given in the packed 4-bit layout.
gs_status launch_gemm_w4(const void* X, const void* Wpacked, float* P, int M, int N, int K, hipStream_t stream) {
  if (M <= 0) return GS_OK;
  const W4Plan p = w4_plan(M, N, K);
  const bf16_t* x = static_cast<const bf16_t*>(X);
  const uint2* codes = static_cast<const uint2*>(Wpacked);
  const uint32_t* meta = reinterpret_cast<const uint32_t*>(static_cast<const char*>(Wpacked) + w4_code_bytes(N, K));
  if (p.waves == 8) launch_w4<8>(p, x, codes, meta, P, M, N, K, stream);
  else launch_w4<4>(p, x, codes, meta, P, M, N, K, stream);
  GS_LAUNCH_CHECK("gemm_w4");
  return GS_OK;
}

}  // namespace gs
