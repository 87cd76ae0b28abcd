// Projections with 4-bit weights (weight-only quantisation in groups of 128 inputs, the format family of
// the AWQ checkpoints the paper's 70B verifier uses, Section IV-A): Y = X * W^T with
// W[n][k] = (code[n][k] - zero[n][k/128]) * scale[n][k/128], codes and zeros in 0..15, scales bf16.
//
// Same streaming design as the bf16 kernel, with a quarter of the weight bytes, which moves the bound from
// HBM to the dequantisation arithmetic and the MFMA pipe; so the kernel uses the 32x32x16 MFMA (twice the
// issue rate of the 16x16x32 one on this chip): a wave owns 32 output columns and up to 128 rows and reads,
// per 64-wide k step, 16 bytes per lane (32 codes of one column) plus one 32-bit word with the column's
// scale and zero point; the codes are turned into bf16 in registers and fed to the MFMA as the B operand.
// Beyond 64 rows a wave owns two such column tiles, so that an activation fragment read from LDS feeds two MFMAs.
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

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;

struct W4Step {
  uint4 codes;       // word kg = the 8 codes of k group kg
  uint32_t meta;
};

// float(byte B of x): the byte-select forms of the conversion, written out because the compiler otherwise
// extracts each nibble with a bit-field instruction first (two instructions per code instead of one)
template <int B>
__device__ __forceinline__ float byte_to_float(uint32_t x) {
  float f;
  if constexpr (B == 0) asm("v_cvt_f32_ubyte0_e32 %0, %1" : "=v"(f) : "v"(x));
  else if constexpr (B == 1) asm("v_cvt_f32_ubyte1_e32 %0, %1" : "=v"(f) : "v"(x));
  else if constexpr (B == 2) asm("v_cvt_f32_ubyte2_e32 %0, %1" : "=v"(f) : "v"(x));
  else asm("v_cvt_f32_ubyte3_e32 %0, %1" : "=v"(f) : "v"(x));
  return f;
}

// word: codes 0..3 in the even nibbles of bytes 0..3, codes 4..7 in the odd nibbles
__device__ __forceinline__ bf16x8_t dequant8(uint32_t word, float scale, float neg_zs) {
  const uint32_t lo4 = word & 0x0F0F0F0Fu, hi4 = (word >> 4) & 0x0F0F0F0Fu;
  uint4 out;
  out.x = pack_bf16x2(fmaf(byte_to_float<0>(lo4), scale, neg_zs), fmaf(byte_to_float<1>(lo4), scale, neg_zs));
  out.y = pack_bf16x2(fmaf(byte_to_float<2>(lo4), scale, neg_zs), fmaf(byte_to_float<3>(lo4), scale, neg_zs));
  out.z = pack_bf16x2(fmaf(byte_to_float<0>(hi4), scale, neg_zs), fmaf(byte_to_float<1>(hi4), scale, neg_zs));
  out.w = pack_bf16x2(fmaf(byte_to_float<2>(hi4), scale, neg_zs), fmaf(byte_to_float<3>(hi4), scale, neg_zs));
  return *reinterpret_cast<const bf16x8_t*>(&out);
}

// MT32 row tiles of 32 rows per workgroup (1, 2 or 4), NW waves of NT 32-column tiles each.  With one
// column tile per wave every MFMA needs an activation fragment of its own from LDS (1 KB per 32 MFMA
// cycles and wave: the LDS limit at four row tiles); with two, a fragment serves two MFMAs.  DX: steps the
// activation tile is fetched ahead (registers, then LDS); the weights are fetched DW steps ahead.
template <int MT32, int NW, int NT, int DW, int DX>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(MT32 == 4 && NW >= 4 ? 2 : 1))) void gemm_w4_kernel(const bf16_t* __restrict__ X,
                                                          const uint4* __restrict__ codes,
                                                          const uint32_t* __restrict__ meta,
                                                          float* __restrict__ P, int M, int N, int K,
                                                          int k_per_split, int m_chunks) {
  static_assert(DW % DX == 0, "the unrolled ring addresses the activation slots statically");
  constexpr int ROWS = MT32 * 32;
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][ROWS * kLdsRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = lane >> 5, c32 = lane & 31;
  int n_block = blockIdx.x, m_chunk = 0;
  if (m_chunks > 1) {
    const int xcd = blockIdx.x & 7, t = blockIdx.x >> 3;
    m_chunk = t % m_chunks;
    n_block = (t / m_chunks) * 8 + xcd;
    if (n_block * (32 * NW * NT) >= N) return;
  }
  const int n_tile = (n_block * NW + wave) * NT;        // first 32-column tile of this wave
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
  uint4 xreg[DX][kPasses];
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
  W4Step wreg[DW][NT];
  auto load_w = [&](int slot, int step) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      wreg[slot][nt].codes = cbase[(size_t)step * code_stride + nt * 64];
      wreg[slot][nt].meta = mbase[(size_t)((step0 + step) >> 1) * N + nt * 32];
    }
  };

  floatx16_t acc[MT32][NT];
#pragma unroll
  for (int mt = 0; mt < MT32; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mt][nt][e] = 0.f;
#pragma unroll
  for (int d = 0; d < DW; ++d)
    if (d < n_steps) {
      load_w(d, d);
      if (d < DX) load_x(d, d);
    }
  // A fragment of row tile mt, k group kg: row mt*32 + lane%32, 16-byte piece 2 kg + lane/32
  const int a_lane = c32 * kLdsRow + h * 8;
  auto dequant_group = [&](const W4Step (&w)[NT], int kg, bf16x8_t (&b)[NT]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const float scale = __uint_as_float(w[nt].meta & 0xffff0000u);
      const float neg_zs = -(float)(w[nt].meta & 0xffu) * scale;
      const uint32_t cw = kg == 0 ? w[nt].codes.x : kg == 1 ? w[nt].codes.y : kg == 2 ? w[nt].codes.z : w[nt].codes.w;
      b[nt] = dequant8(cw, scale, neg_zs);
    }
  };
  // Software pipeline: the activation fragments (LDS) and the dequantised weights (vector ALU) of k group
  // kg + 1 are produced while the MFMAs of group kg run; the weights of a step's first group are dequantised
  // during the last group of the step before, since they do not wait for the barrier.
  bf16x8_t b_cur[NT];
  if (n_steps > 0) dequant_group(wreg[0], 0, b_cur);
  for (int base = 0; base < n_steps; base += DW) {
#pragma unroll
    for (int d = 0; d < DW; ++d) {
      const int step = base + d;
      if (step < n_steps) {
        const int buf = step & 1;
        store_x(buf, d % DX);
        __syncthreads();
        W4Step w[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) w[nt] = wreg[d][nt];
        if (step + DW < n_steps) load_w(d, step + DW);
        if (step + DX < n_steps) load_x(d % DX, step + DX);
        bf16x8_t a_cur[MT32];
#pragma unroll
        for (int mt = 0; mt < MT32; ++mt)
          a_cur[mt] = *reinterpret_cast<const bf16x8_t*>(&xs[buf][mt * 32 * kLdsRow + a_lane]);
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
          bf16x8_t a_nxt[MT32], b_nxt[NT];
          if (kg < 3) {
#pragma unroll
            for (int mt = 0; mt < MT32; ++mt)
              a_nxt[mt] = *reinterpret_cast<const bf16x8_t*>(&xs[buf][mt * 32 * kLdsRow + a_lane + (kg + 1) * 16]);
            dequant_group(w, kg + 1, b_nxt);
          } else if (step + 1 < n_steps) {
            dequant_group(wreg[(d + 1) % DW], 0, b_nxt);
          }
#pragma unroll
          for (int mt = 0; mt < MT32; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur[mt], b_cur[nt], acc[mt][nt], 0, 0, 0);
#pragma unroll
          for (int mt = 0; mt < MT32; ++mt) a_cur[mt] = a_nxt[mt];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) b_cur[nt] = b_nxt[nt];
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
      if (row < M) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) out[(size_t)row * N + n0 + nt * 32 + c32] = acc[mt][nt][v];
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

// Launch shape of the 4-bit kernel: 32-row tiles per workgroup (1, 2 or 4), row chunks of 128, waves, column
// tiles per wave, K splits.
struct W4Plan {
  int mt32, m_chunks, waves, nt, splits, k_per;
};

static W4Plan w4_plan(int M, int N, int K) {
  W4Plan p;
  p.mt32 = M <= 32 ? 1 : M <= 64 ? 2 : 4;
  p.m_chunks = ceil_div(M, 32 * p.mt32);
  p.nt = 1;
  if (p.mt32 == 4 && N % 512 == 0 && N / 512 >= 96) {
    p.waves = 8; p.nt = 2;
  } else if (p.mt32 == 4 && N % 256 == 0) {
    p.waves = 4; p.nt = 2;
  } else {
    p.waves = (N % 256 == 0 && N / 256 >= 96) ? 8 : (N % 128 == 0 ? 4 : 2);
  }
  const int wgs = N / (32 * p.waves * p.nt) * p.m_chunks;
  // K splits: enough workgroups to stream from every CU while the weights are the bound (512); one workgroup
  // per CU at four row tiles, where the MFMA work is the bound and every further split only adds an
  // M x N fp32 partial result to write and re-read (measured on the 70B shape: 68 instead of 77 us per launch)
  const int target = p.mt32 == 4 ? 256 : 512;
  int want = (target + wgs / 2) / wgs;
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
  const int n_blocks = N / (32 * NW * p.nt);
  const int gx = p.m_chunks > 1 ? ceil_div(n_blocks, 8) * 8 * p.m_chunks : n_blocks;
  const dim3 grid(gx, p.splits, 1);
  if (p.mt32 == 1)
    gemm_w4_kernel<1, NW, 1, 4, 4><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
  else if (p.mt32 == 2)
    gemm_w4_kernel<2, NW, 1, 4, 4><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
  else if (p.nt == 1)
    gemm_w4_kernel<4, NW, 1, 4, 4><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
  else
    gemm_w4_kernel<4, NW, 2, 2, (NW >= 8 ? 2 : 1)><<<grid, 64 * NW, 0, stream>>>(x, codes, meta, P, M, N, K, p.k_per, p.m_chunks);
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
