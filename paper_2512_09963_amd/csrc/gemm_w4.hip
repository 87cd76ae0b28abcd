// Projections with 4-bit weights (weight-only quantisation in groups of 128 inputs, the format family of
// the AWQ checkpoints the paper's 70B verifier uses, Section IV-A): Y = X * W^T with
// W[n][k] = (code[n][k] - zero[n][k/128]) * scale[n][k/128], codes and zeros in 0..15, scales bf16.
//
// Same streaming design as the bf16 kernel, with a quarter of the weight bytes, which moves the bound from
// HBM to the dequantisation arithmetic and the MFMA pipe; so the kernel uses the 32x32x16 MFMA (twice the
// issue rate of the 16x16x32 one on this chip): a wave owns 32 output columns and up to 128 rows and reads,
// per 64-wide k step, 16 bytes per lane (32 codes of one column) plus one 32-bit word with the column's
// scale and zero point; the codes are turned into bf16 in registers and fed to the MFMA as the B operand.
// Dequantisation: four codes are spread to the bytes of a word (two mask operations per eight codes), each
// byte is converted to fp32 by the byte-conversion instruction, fma(c, scale, -zero * scale) = (c - zero) *
// scale is exact in fp32 (5 x 8 significant bits), and the packed conversion rounds it to bf16 (nearest
// even): every dequantised weight is a function of (c, zero, scale) alone, the same on every path.
//
// Packed layout (gs_pack_weight_w4):
//   codes [K/64][N/32][64 lanes][4 words]: lane l holds column l%32, and word kg holds inputs
//         16 kg + 8 (l/32) + i, i = 0..7 (the B fragment of k group kg); in a word, codes 0..3 sit in the low
//         nibbles of bytes 0..3 and codes 4..7 in the high nibbles, so that (word & 0x0F0F0F0F) and
//         ((word >> 4) & 0x0F0F0F0F) each hold four codes, one per byte
//   meta  [K/128][N] words: bf16 scale in the high half, zero point in the low byte
// Activations go through LDS exactly as in the bf16 kernels.  Rows beyond 128 are served in chunks of 128 by
// separate workgroups (XCD-aware order, see the bf16 kernel); a taller tile is not built for this format.
#include "common.h"
#include "device_types.h"

namespace gs {
namespace {

constexpr int kBK = 64;
constexpr int kLdsRow = kBK + 8;
constexpr int kGroup = 128;
constexpr int kDepth = 4;

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;

struct W4Step {
  uint4 codes;       // word kg = the 8 codes of k group kg
  uint32_t meta;
};

// word: codes 0..3 in the even nibbles of bytes 0..3, codes 4..7 in the odd nibbles
__device__ __forceinline__ bf16x8_t dequant8(uint32_t word, float scale, float neg_zs) {
  const uint32_t lo4 = word & 0x0F0F0F0Fu, hi4 = (word >> 4) & 0x0F0F0F0Fu;
  float f[8];
  f[0] = (float)(lo4 & 0xffu);
  f[1] = (float)((lo4 >> 8) & 0xffu);
  f[2] = (float)((lo4 >> 16) & 0xffu);
  f[3] = (float)(lo4 >> 24);
  f[4] = (float)(hi4 & 0xffu);
  f[5] = (float)((hi4 >> 8) & 0xffu);
  f[6] = (float)((hi4 >> 16) & 0xffu);
  f[7] = (float)(hi4 >> 24);
  uint4 out;
  out.x = pack_bf16x2(fmaf(f[0], scale, neg_zs), fmaf(f[1], scale, neg_zs));
  out.y = pack_bf16x2(fmaf(f[2], scale, neg_zs), fmaf(f[3], scale, neg_zs));
  out.z = pack_bf16x2(fmaf(f[4], scale, neg_zs), fmaf(f[5], scale, neg_zs));
  out.w = pack_bf16x2(fmaf(f[6], scale, neg_zs), fmaf(f[7], scale, neg_zs));
  return *reinterpret_cast<const bf16x8_t*>(&out);
}

// MT32 row tiles of 32 rows per workgroup (1, 2 or 4), NW waves of 32 columns each.
template <int MT32, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_w4_kernel(const bf16_t* __restrict__ X,
                                                          const uint4* __restrict__ codes,
                                                          const uint32_t* __restrict__ meta,
                                                          float* __restrict__ P, int M, int N, int K,
                                                          int k_per_split, int m_chunks) {
  constexpr int ROWS = MT32 * 32;
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][ROWS * kLdsRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = lane >> 5, c32 = lane & 31;
  int n_block = blockIdx.x, m_chunk = 0;
  if (m_chunks > 1) {
    const int xcd = blockIdx.x & 7, t = blockIdx.x >> 3;
    m_chunk = t % m_chunks;
    n_block = (t / m_chunks) * 8 + xcd;
    if (n_block * (32 * NW) >= N) return;
  }
  const int n_tile = n_block * NW + wave;        // 32-column tile
  const int n0 = n_tile * 32;
  const int split = blockIdx.y;
  const int m0 = m_chunk * ROWS;
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_steps = (k_end - k_begin) / kBK;
  const int step0 = k_begin / kBK;

  constexpr int kThreads = 64 * NW;
  constexpr int kChunks = ROWS * 8;
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
  const size_t code_stride = (size_t)(N / 32) * 64;       // uint4 per k step
  const uint4* cbase = codes + (size_t)step0 * code_stride + (size_t)n_tile * 64 + lane;
  const uint32_t* mbase = meta + n0 + c32;
  W4Step wreg[kDepth];
  auto load_w = [&](int slot, int step) {
    wreg[slot].codes = cbase[(size_t)step * code_stride];
    wreg[slot].meta = mbase[(size_t)((step0 + step) >> 1) * N];
  };

  floatx16_t acc[MT32];
#pragma unroll
  for (int mt = 0; mt < MT32; ++mt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[mt][e] = 0.f;
#pragma unroll
  for (int d = 0; d < kDepth; ++d)
    if (d < n_steps) {
      load_w(d, d);
      load_x(d, d);
    }
  // A fragment of row tile mt, k group kg: row mt*32 + lane%32, 16-byte piece 2 kg + lane/32
  const int a_lane = c32 * kLdsRow + h * 8;
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
        const float neg_zs = -(float)(w.meta & 0xffu) * scale;
        const uint32_t cw[4] = {w.codes.x, w.codes.y, w.codes.z, w.codes.w};
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
          const bf16x8_t b = dequant8(cw[kg], scale, neg_zs);
#pragma unroll
          for (int mt = 0; mt < MT32; ++mt) {
            const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&xs[buf][mt * 32 * kLdsRow + a_lane + kg * 16]);
            acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[mt], 0, 0, 0);
          }
        }
      }
    }
  }
  float* out = P + (size_t)split * M * N;
#pragma unroll
  for (int mt = 0; mt < MT32; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = m0 + mt * 32 + (v >> 2) * 8 + h * 4 + (v & 3);
      if (row < M) out[(size_t)row * N + n0 + c32] = acc[mt][v];
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
    const int kg = (int)(idx & 3), lane = (int)((idx >> 2) & 63);
    const size_t block = idx >> 8;
    const int n_tiles = N / 32;
    const int n_tile = (int)(block % n_tiles), k_step = (int)(block / n_tiles);
    const int h = lane >> 5, c32 = lane & 31;
    const uint8_t* src = q + (size_t)(n_tile * 32 + c32) * K + k_step * kBK + kg * 16 + h * 8;
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w |= (uint32_t)(src[i] & 15u) << (8 * i);            // codes 0..3: even nibbles
      w |= (uint32_t)(src[4 + i] & 15u) << (8 * i + 4);    // codes 4..7: odd nibbles
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

// Launch shape of the 4-bit kernel: 32-row tiles per workgroup (1, 2 or 4), row chunks of 128, waves, K splits.
struct W4Plan {
  int mt32, m_chunks, waves, splits, k_per;
};

static W4Plan w4_plan(int M, int N, int K) {
  W4Plan p;
  p.mt32 = M <= 32 ? 1 : M <= 64 ? 2 : 4;
  p.m_chunks = ceil_div(M, 32 * p.mt32);
  p.waves = (N % 256 == 0 && N / 256 >= 96) ? 8 : (N % 128 == 0 ? 4 : 2);
  const int wgs = N / (32 * p.waves) * p.m_chunks;
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
static void launch_w4(const W4Plan& p, const bf16_t* x, const uint4* codes, const uint32_t* meta, float* P, int M,
                      int N, int K, hipStream_t stream) {
  const int n_blocks = N / (32 * NW);
  const int gx = p.m_chunks > 1 ? ceil_div(n_blocks, 8) * 8 * p.m_chunks : n_blocks;
  const dim3 grid(gx, p.splits, 1);
  if (p.mt32 == 1)
    gemm_w4_kernel<1, NW><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
  else if (p.mt32 == 2)
    gemm_w4_kernel<2, NW><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
  else
    gemm_w4_kernel<4, NW><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
}

// P [splits][M][N] fp32 partial sums of X [M][K] (bf16) * W^T with W given in the packed 4-bit layout.
gs_status launch_gemm_w4(const void* X, const void* Wpacked, float* P, int M, int N, int K, hipStream_t stream) {
  if (M <= 0) return GS_OK;
  const W4Plan p = w4_plan(M, N, K);
  const bf16_t* x = static_cast<const bf16_t*>(X);
  const uint4* codes = static_cast<const uint4*>(Wpacked);
  const uint32_t* meta = reinterpret_cast<const uint32_t*>(static_cast<const char*>(Wpacked) + w4_code_bytes(N, K));
  if (p.waves == 8) launch_w4<8>(p, x, codes, meta, P, M, N, K, stream);
  else if (p.waves == 4) launch_w4<4>(p, x, codes, meta, P, M, N, K, stream);
  else launch_w4<2>(p, x, codes, meta, P, M, N, K, stream);
  GS_LAUNCH_CHECK("gemm_w4");
  return GS_OK;
}

}  // namespace gs
