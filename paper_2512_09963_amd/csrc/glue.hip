// Row-wise kernels between the projections of the decoder: embedding gather,
// residual add + RMSNorm (also sums the split-K partials of the preceding projection),
// rotary embedding + KV-page append, SwiGLU.  All arithmetic is fp32; T is the storage
// type of the tensors fed to the next projection and of the KV pages (float or bf16).
#include "common.h"
#include "device_types.h"

namespace gs {
namespace {

// Sum over the workgroup (any multiple of 64 threads up to 1024), fixed order.
__device__ __forceinline__ float block_sum(float v, float* sh /*[16]*/) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
  const int n_waves = blockDim.x >> 6;
  for (int w = 0; w < n_waves; ++w) t += sh[w];
  __syncthreads();
  return t;
}

// server that owns target row r: largest i with cu_rows[i] <= r
__device__ __forceinline__ int server_of_row(const int* __restrict__ cu_rows, int n_servers, int r) {
  int lo = 0, hi = n_servers;   // invariant: cu_rows[lo] <= r < cu_rows[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu_rows[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ embed, const int* __restrict__ tokens,
                                                    float* __restrict__ x, int d, int vocab) {
  const int r = blockIdx.x;
  const int tok = min(max(tokens[r], 0), vocab - 1);      // an id outside the vocabulary is never used as an index
  const T* src = embed + (size_t)tok * d;
  for (int i = threadIdx.x; i < d; i += 256) x[(size_t)r * d + i] = Storage<T>::load(src + i);
}

// x[r] += sum_s partial[s][r] (if partial), then h[r] = x[r] * w / sqrt(mean(x[r]^2) + eps).
// One workgroup per row, one float4 per lane and pass; the loads of the S partials are
// independent, so they are issued back to back (d % 4 == 0).  The first two passes of a row (all of it for
// d <= 8192 at 1024 lanes) stay in registers between the sum of squares and the scaling, and the norm
// weights are fetched before the reduction, so the second phase touches no memory but its stores.
template <typename T>
__global__ __launch_bounds__(1024) void add_rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ partial,
                                                           int n_splits, int n_rows, const float* __restrict__ w,
                                                           float eps, T* __restrict__ h, int d) {
  __shared__ float sh[16];
  const int r = blockIdx.x;
  float4* xr = reinterpret_cast<float4*>(x + (size_t)r * d);
  const int d4 = d >> 2;
  const size_t split_stride = (size_t)n_rows * d4;
  const float4* pr = reinterpret_cast<const float4*>(partial) + (size_t)r * d4;
  const float4* wr = reinterpret_cast<const float4*>(w);
  // element i of the row with the partial sums added (and stored back to the residual stream)
  auto fetch = [&](int i) {
    float4 v = xr[i];
    if (partial) {
      float4 a0 = make_float4(0.f, 0.f, 0.f, 0.f), a1 = a0;
      int s = 0;
      for (; s + 4 <= n_splits; s += 4) {
        const float4 p0 = pr[(size_t)s * split_stride + i], p1 = pr[(size_t)(s + 1) * split_stride + i];
        const float4 p2 = pr[(size_t)(s + 2) * split_stride + i], p3 = pr[(size_t)(s + 3) * split_stride + i];
        a0.x += p0.x + p1.x; a0.y += p0.y + p1.y; a0.z += p0.z + p1.z; a0.w += p0.w + p1.w;
        a1.x += p2.x + p3.x; a1.y += p2.y + p3.y; a1.z += p2.z + p3.z; a1.w += p2.w + p3.w;
      }
      for (; s < n_splits; ++s) {
        const float4 p0 = pr[(size_t)s * split_stride + i];
        a0.x += p0.x; a0.y += p0.y; a0.z += p0.z; a0.w += p0.w;
      }
      v.x += a0.x + a1.x; v.y += a0.y + a1.y; v.z += a0.z + a1.z; v.w += a0.w + a1.w;
      xr[i] = v;
    }
    return v;
  };
  auto squares = [](const float4& v) { return (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w); };
  auto emit = [&](int i, const float4& v, const float4& ww, float inv) {
    T* dst = h + (size_t)r * d + 4 * i;
    Storage<T>::store(dst + 0, v.x * inv * ww.x);
    Storage<T>::store(dst + 1, v.y * inv * ww.y);
    Storage<T>::store(dst + 2, v.z * inv * ww.z);
    Storage<T>::store(dst + 3, v.w * inv * ww.w);
  };
  const int bd = blockDim.x;
  const int i0 = threadIdx.x, i1 = threadIdx.x + bd;
  const bool has0 = i0 < d4, has1 = i1 < d4;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 v0 = zero, v1 = zero, w0 = zero, w1 = zero;
  float ss = 0.f;
  if (has0) {
    w0 = wr[i0];
    v0 = fetch(i0);
    ss += squares(v0);
  }
  if (has1) {
    w1 = wr[i1];
    v1 = fetch(i1);
    ss += squares(v1);
  }
  for (int i = i1 + bd; i < d4; i += bd) ss += squares(fetch(i));     // rows wider than two passes
  const float tot = block_sum(ss, sh);
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  if (has0) emit(i0, v0, w0, inv);
  if (has1) emit(i1, v1, w1, inv);
  for (int i = i1 + bd; i < d4; i += bd) emit(i, xr[i], wr[i], inv);
}

// Per-row facts that every layer of a step shares: where the row's K/V go (page, slot), how many keys
// its server has after the append, and the rotary sine/cosine of its position.  rope [R][hd/2] (cos, sin).  The angle pos * theta^(-2i/hd)
// reaches thousands of radians: it is formed in double, so that the rotated values agree with a
// float64 evaluation to fp32 rounding.  grid R, block hd/2.
__global__ void row_meta_kernel(const int* __restrict__ cu_rows, const int* __restrict__ ctx_len, int n_servers,
                                const int* __restrict__ block_table, int max_blocks, int page_size, int hd,
                                double log2_theta, int4* __restrict__ row_slot, float2* __restrict__ rope) {
  const int r = blockIdx.x, i = threadIdx.x;
  const int srv = server_of_row(cu_rows, n_servers, r);
  const int pos = ctx_len[srv] + (r - cu_rows[srv]);
  if (i == 0)      // (page, slot) of the row's own K/V, keys of its server after the append, server
    row_slot[r] = make_int4(block_table[(size_t)srv * max_blocks + pos / page_size], pos % page_size,
                            ctx_len[srv] + (cu_rows[srv + 1] - cu_rows[srv]), srv);
  const double inv_freq = exp2(-2.0 * (double)i / (double)hd * log2_theta);
  double sn, cs;
  sincos((double)pos * inv_freq, &sn, &cs);
  rope[(size_t)r * (hd >> 1) + i] = make_float2((float)cs, (float)sn);
}

// Sums the QKV partials, rotates Q and K at the row's position, stores Q [R][H][hd] and
// appends K ([page][H_kv][slot][hd]) and V ([page][H_kv][hd][slot]) to the layer's pages.
// grid (R, (H + 2 H_kv) * hd/2 / 256): a thread owns the element pair (i, i + hd/2) of one head.
template <typename T>
__global__ __launch_bounds__(256) void rope_append_kernel(const float* __restrict__ qkv, int n_splits, int n_rows,
                                                          const int4* __restrict__ row_slot,
                                                          const float2* __restrict__ rope, int page_size,
                                                          int n_heads, int n_kv, int hd, T* __restrict__ q_out,
                                                          T* __restrict__ k_pages, T* __restrict__ v_pages) {
  const int r = blockIdx.x;
  const int half = hd >> 1;
  const int item = blockIdx.y * 256 + threadIdx.x;
  const int head = item / half, i = item - head * half;
  if (head >= n_heads + 2 * n_kv) return;
  const int width = (n_heads + 2 * n_kv) * hd;
  const size_t split_stride = (size_t)n_rows * width;
  const float* src = qkv + (size_t)r * width + head * hd + i;
  float a = 0.f, b = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    a += src[(size_t)s * split_stride];
    b += src[(size_t)s * split_stride + half];
  }
  const int4 ps = row_slot[r];
  if (head < n_heads + n_kv) {
    const float2 cs = rope[(size_t)r * half + i];
    const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
    T* dst = (head < n_heads) ? q_out + ((size_t)r * n_heads + head) * hd
                              : k_pages + (((size_t)ps.x * n_kv + (head - n_heads)) * page_size + ps.y) * hd;
    Storage<T>::store(dst + i, ra);
    Storage<T>::store(dst + i + half, rb);
  } else {
    T* dst = v_pages + ((size_t)ps.x * n_kv + (head - n_heads - n_kv)) * hd * page_size + ps.y;
    Storage<T>::store(dst + (size_t)i * page_size, a);
    Storage<T>::store(dst + (size_t)(i + half) * page_size, b);
  }
}

// act[r][f] = silu(gate) * up with gate = sum_s gu[s][r][f], up = sum_s gu[s][r][F + f].
// VEC: four features per lane (F % 4 == 0).
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ gu, int n_splits, int n_rows, int F,
                                                     T* __restrict__ act) {
  constexpr int W = VEC ? 4 : 1;
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * W;
  if (idx >= (size_t)n_rows * F) return;
  const int r = (int)(idx / F), f = (int)(idx - (size_t)r * F);
  float gt[W], up[W];
#pragma unroll
  for (int k = 0; k < W; ++k) gt[k] = up[k] = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float* row = gu + ((size_t)s * n_rows + r) * 2 * F;
    if constexpr (VEC) {
      const float4 g4 = *reinterpret_cast<const float4*>(row + f);
      const float4 u4 = *reinterpret_cast<const float4*>(row + F + f);
      gt[0] += g4.x; gt[1] += g4.y; gt[2] += g4.z; gt[3] += g4.w;
      up[0] += u4.x; up[1] += u4.y; up[2] += u4.z; up[3] += u4.w;
    } else {
      gt[0] += row[f];
      up[0] += row[F + f];
    }
  }
#pragma unroll
  for (int k = 0; k < W; ++k) Storage<T>::store(act + idx + k, gt[k] / (1.0f + expf(-gt[k])) * up[k]);
}

}  // namespace

#define GS_DISPATCH_T(dtype, ...)                 \
  if ((dtype) == GS_BF16) {                       \
    using T = bf16_t;                             \
    __VA_ARGS__                                   \
  } else {                                        \
    using T = float;                              \
    __VA_ARGS__                                   \
  }

gs_status launch_embed(int dtype, const void* embed, const int* tokens, float* x, int n_rows, int d, int vocab,
                       hipStream_t stream) {
  GS_DISPATCH_T(dtype, embed_kernel<T><<<n_rows, 256, 0, stream>>>(static_cast<const T*>(embed), tokens, x, d, vocab);)
  GS_LAUNCH_CHECK("embed");
  return GS_OK;
}

gs_status launch_add_rmsnorm(int dtype, float* x, const float* partial, int n_splits, int n_rows, const float* w,
                             float eps, void* h, int d, hipStream_t stream) {
  int threads = ceil_div(d / 4, 64) * 64;
  if (threads > 1024) threads = 1024;
  GS_DISPATCH_T(dtype, add_rmsnorm_kernel<T><<<n_rows, threads, 0, stream>>>(x, partial, n_splits, n_rows, w, eps,
                                                                            static_cast<T*>(h), d);)
  GS_LAUNCH_CHECK("add_rmsnorm");
  return GS_OK;
}

gs_status launch_row_meta(const int* cu_rows, const int* ctx_len, int n_servers, int n_rows, const int* block_table,
                          int max_blocks, int page_size, int hd, float rope_theta, void* row_slot, void* rope,
                          hipStream_t stream) {
  row_meta_kernel<<<n_rows, hd / 2, 0, stream>>>(cu_rows, ctx_len, n_servers, block_table, max_blocks, page_size, hd,
                                                 log2((double)rope_theta), static_cast<int4*>(row_slot),
                                                 static_cast<float2*>(rope));
  GS_LAUNCH_CHECK("row_meta");
  return GS_OK;
}

gs_status launch_rope_append(int dtype, const float* qkv, int n_splits, int n_rows, const void* row_slot,
                             const void* rope, int page_size, int n_heads, int n_kv, int hd, void* q_out,
                             void* k_pages, void* v_pages, hipStream_t stream) {
  const dim3 grid(n_rows, ceil_div((n_heads + 2 * n_kv) * (hd / 2), 256));
  GS_DISPATCH_T(dtype, rope_append_kernel<T><<<grid, 256, 0, stream>>>(
                           qkv, n_splits, n_rows, static_cast<const int4*>(row_slot),
                           static_cast<const float2*>(rope), page_size, n_heads, n_kv, hd, static_cast<T*>(q_out),
                           static_cast<T*>(k_pages), static_cast<T*>(v_pages));)
  GS_LAUNCH_CHECK("rope_append");
  return GS_OK;
}

gs_status launch_swiglu(int dtype, const float* gu, int n_splits, int n_rows, int F, void* act, hipStream_t stream) {
  const size_t total = (size_t)n_rows * F;
  if (F % 4 == 0) {
    const int blocks = (int)((total / 4 + 255) / 256);
    GS_DISPATCH_T(dtype, swiglu_kernel<T, true><<<blocks, 256, 0, stream>>>(gu, n_splits, n_rows, F, static_cast<T*>(act));)
  } else {
    const int blocks = (int)((total + 255) / 256);
    GS_DISPATCH_T(dtype, swiglu_kernel<T, false><<<blocks, 256, 0, stream>>>(gu, n_splits, n_rows, F, static_cast<T*>(act));)
  }
  GS_LAUNCH_CHECK("swiglu");
  return GS_OK;
}

}  // namespace gs
