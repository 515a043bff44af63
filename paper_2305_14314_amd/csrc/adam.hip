// Optimizer step for the LoRA parameters (arXiv 2305.14314, hyperparameter appendix: Adam with beta2 = 0.999 and a
// maximum gradient norm of 0.3; Section 3, "Paged Optimizers": the state this step reads and writes is what the paper
// pages -- here it stays in HBM, in buffers the caller owns).  The update rule itself is the published algorithm
// (Kingma & Ba 2015, Algorithm 1) with bias correction and, optionally, decoupled weight decay.
//
// Two kernels, both pure streams:
//   sqnorm_kernel   sum of squares of a gradient buffer in double precision, added to a device double
//   adam_kernel     per element, every operation a separately rounded fp32 operation in a fixed order:
//                     g' = coef * g;  m = b1 m + (1 - b1) g';  v = b2 v + (1 - b2) g' g'
//                     p = p - (lr wd) p  [wd != 0];  p = p - lr * (m / bc1) / (sqrt(v / bc2) + eps)
//                   writes p, m, v, the bf16 copy of p that the linear layers read, and zeroes g when asked to.
// 34 bytes of HBM traffic per parameter (16 read, 18 written with the bf16 copy and the cleared gradient).
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

namespace {

constexpr int kAdamThreads = 256;
constexpr int kAdamWgsPerCu = 8;

__global__ __launch_bounds__(kAdamThreads) void sqnorm_kernel(const float* __restrict__ g, int64_t n,
                                                              double* __restrict__ out) {
  __shared__ double wsum[kAdamThreads / 64];
  const int64_t n4 = n >> 2, stride = (int64_t)gridDim.x * kAdamThreads;
  double s = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * kAdamThreads + threadIdx.x; i < n4; i += stride) {
    const float4 x = ((const float4*)g)[i];
    s += (double)x.x * (double)x.x + (double)x.y * (double)x.y + (double)x.z * (double)x.z + (double)x.w * (double)x.w;
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {             // the last n % 4 elements
    const double x = (double)g[(n4 << 2) + threadIdx.x];
    s += x * x;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kAdamThreads / 64; ++w) t += wsum[w];
    if (t != 0.0) atomicAdd(out, t);
  }
}

__device__ __forceinline__ void adam_element(float& p, float& m, float& v, float g, const AdamConsts& c, float coef) {
  const float gs = __fmul_rn(g, coef);
  m = __fadd_rn(__fmul_rn(c.b1, m), __fmul_rn(c.omb1, gs));
  v = __fadd_rn(__fmul_rn(c.b2, v), __fmul_rn(c.omb2, __fmul_rn(gs, gs)));
  const float mh = m / c.bc1;                                 // correctly rounded division and square root
  const float vh = v / c.bc2;
  const float d = __fadd_rn(__builtin_sqrtf(vh), c.eps);
  const float u = mh / d;
  if (c.lrwd != 0.0f) p = __fsub_rn(p, __fmul_rn(c.lrwd, p));
  p = __fsub_rn(p, __fmul_rn(c.lr, u));
}

__global__ __launch_bounds__(kAdamThreads) void adam_kernel(float* __restrict__ P, float* __restrict__ Mm,
                                                            float* __restrict__ V, float* __restrict__ G,
                                                            uint16_t* __restrict__ Pb, int64_t n, const AdamConsts c) {
  // the gradient coefficient: grad_scale, times the clipping factor of the global norm when a limit is set
  float coef;
  {
    double k = c.grad_scale;
    if (c.sqnorm != nullptr && c.max_norm > 0.0) {
      const double norm = __builtin_fabs(c.grad_scale) * __builtin_sqrt(*c.sqnorm);
      if (norm > c.max_norm) k = c.grad_scale * (c.max_norm / norm);
    }
    coef = (float)k;
  }
  const int64_t n4 = n >> 2, stride = (int64_t)gridDim.x * kAdamThreads;
  for (int64_t i = (int64_t)blockIdx.x * kAdamThreads + threadIdx.x; i < n4; i += stride) {
    float4 p = ((const float4*)P)[i], m = ((const float4*)Mm)[i], v = ((const float4*)V)[i];
    const float4 g = ((const float4*)G)[i];
    adam_element(p.x, m.x, v.x, g.x, c, coef);
    adam_element(p.y, m.y, v.y, g.y, c, coef);
    adam_element(p.z, m.z, v.z, g.z, c, coef);
    adam_element(p.w, m.w, v.w, g.w, c, coef);
    ((float4*)P)[i] = p; ((float4*)Mm)[i] = m; ((float4*)V)[i] = v;
    if (Pb) {
      uint2 b;
      b.x = (uint32_t)bf16_bits(p.x) | ((uint32_t)bf16_bits(p.y) << 16);
      b.y = (uint32_t)bf16_bits(p.z) | ((uint32_t)bf16_bits(p.w) << 16);
      ((uint2*)Pb)[i] = b;
    }
    if (c.zero_grad) ((float4*)G)[i] = float4{0.f, 0.f, 0.f, 0.f};
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {             // the last n % 4 elements
    const int64_t i = (n4 << 2) + threadIdx.x;
    float p = P[i], m = Mm[i], v = V[i];
    adam_element(p, m, v, G[i], c, coef);
    P[i] = p; Mm[i] = m; V[i] = v;
    if (Pb) Pb[i] = bf16_bits(p);
    if (c.zero_grad) G[i] = 0.0f;
  }
}

unsigned stream_grid(int64_t n) {
  int64_t blocks = ((n >> 2) + kAdamThreads - 1) / kAdamThreads;
  const int64_t cap = 256 * kAdamWgsPerCu;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

}  // namespace

// ---- measurement aid: what plain streams reach on this board ------------------------------------------------------
// mode 0 reads n16 16-byte words (their XOR goes to `sink`, so the loads stay), mode 1 writes them, mode 2 copies
// src to dst.  256 threads, a grid-stride loop with `unroll` independent 16-byte accesses per lane in flight.
template <int MODE>
__global__ __launch_bounds__(256) void hbm_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16,
                                                        uint32_t* __restrict__ sink) {
  constexpr int U = 4;
  const int64_t stride = (int64_t)gridDim.x * 256;
  uint4 x = {0u, 0u, 0u, 0u};
  for (int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x; i0 < n16; i0 += U * stride) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = i0 + u * stride;
      if (MODE != 1) v[u] = src[i < n16 ? i : i0];
      else v[u] = uint4{(uint32_t)i, 1u, 2u, 3u};
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = i0 + u * stride;
      if (MODE == 0) { x.x ^= v[u].x; x.y ^= v[u].y; x.z ^= v[u].z; x.w ^= v[u].w; }
      else if (i < n16) dst[i] = v[u];
    }
  }
  if (MODE == 0 && (x.x ^ x.y ^ x.z ^ x.w) == 0x9e3779b9u) *sink = 1u;   // practically never true: keeps the loads alive
}

hipError_t launch_hbm_probe(int mode, const void* src, void* dst, int64_t bytes, uint32_t* sink, int wgs_per_cu,
                            hipStream_t st) {
  if (mode < 0 || mode > 2 || bytes <= 0 || bytes % 16 != 0 || wgs_per_cu < 1 || wgs_per_cu > 64) return hipErrorInvalidValue;
  const int64_t n16 = bytes / 16;
  const dim3 grid((unsigned)(256 * wgs_per_cu));
  if (mode == 0) hipLaunchKernelGGL(hbm_probe_kernel<0>, grid, dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16, sink);
  else if (mode == 1) hipLaunchKernelGGL(hbm_probe_kernel<1>, grid, dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16, sink);
  else hipLaunchKernelGGL(hbm_probe_kernel<2>, grid, dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16, sink);
  return hipGetLastError();
}

hipError_t launch_grad_sqnorm(const float* g, int64_t n, double* accum, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(sqnorm_kernel, dim3(stream_grid(n)), dim3(kAdamThreads), 0, st, g, n, accum);
  return hipGetLastError();
}

hipError_t launch_adam(float* p, float* m, float* v, float* g, uint16_t* p_bf16, int64_t n, const AdamConsts& c,
                       hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(adam_kernel, dim3(stream_grid(n)), dim3(kAdamThreads), 0, st, p, m, v, g, p_bf16, n, c);
  return hipGetLastError();
}

}  // namespace qlora
