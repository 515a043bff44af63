// k-bit storage of NormalFloat codes for k = 2, 3 (arXiv 2305.14314, Section 3: the k-bit NormalFloat data type has 2^k
// values; a weight then costs k + 0.127 bits).  The 4-bit container every other kernel reads holds such codes with the
// upper bits clear; these two streaming kernels convert between that container and the dense form a weight rests in:
// one bit stream over the flattened weight, code i in bits [k i, k i + k), little-endian.  A lane handles 32 codes:
// 16 bytes of the container against 4 k bytes of the stream, so both sides move whole dwords.
#include "common.hpp"
#include "launch.hpp"

namespace qlora {

namespace {

constexpr int kKbitThreads = 256;

template <int K>
__global__ __launch_bounds__(kKbitThreads) void kbit_pack_kernel(const uint4* __restrict__ packed4,
                                                                 uint32_t* __restrict__ stream, int64_t groups) {
  const int64_t stride = (int64_t)gridDim.x * kKbitThreads;
  for (int64_t g = (int64_t)blockIdx.x * kKbitThreads + threadIdx.x; g < groups; g += stride) {
    const uint4 v = packed4[g];
    const uint32_t in[4] = {v.x, v.y, v.z, v.w};
    uint32_t out[K];
#pragma unroll
    for (int w = 0; w < K; ++w) out[w] = 0u;
#pragma unroll
    for (int j = 0; j < 32; ++j) {                           // code j: nibble j of the 16 bytes
      const uint32_t c = (in[j >> 3] >> (4 * (j & 7))) & ((1u << K) - 1u);
      const int pos = K * j, w = pos >> 5, sh = pos & 31;
      out[w] |= c << sh;
      if (sh + K > 32) out[w + 1] |= c >> (32 - sh);         // a code that straddles two dwords (k = 3 only)
    }
#pragma unroll
    for (int w = 0; w < K; ++w) stream[g * K + w] = out[w];
  }
}

template <int K>
__global__ __launch_bounds__(kKbitThreads) void kbit_unpack_kernel(const uint32_t* __restrict__ stream,
                                                                   uint4* __restrict__ packed4, int64_t groups) {
  const int64_t stride = (int64_t)gridDim.x * kKbitThreads;
  for (int64_t g = (int64_t)blockIdx.x * kKbitThreads + threadIdx.x; g < groups; g += stride) {
    uint32_t in[K];
#pragma unroll
    for (int w = 0; w < K; ++w) in[w] = stream[g * K + w];
    uint32_t out[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const int pos = K * j, w = pos >> 5, sh = pos & 31;
      uint32_t c = in[w] >> sh;
      if (sh + K > 32) c |= in[w + 1] << (32 - sh);
      out[j >> 3] |= (c & ((1u << K) - 1u)) << (4 * (j & 7));
    }
    packed4[g] = uint4{out[0], out[1], out[2], out[3]};
  }
}

unsigned kbit_grid(int64_t groups) {
  int64_t blocks = (groups + kKbitThreads - 1) / kKbitThreads;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

}  // namespace

hipError_t launch_kbit_pack(const uint8_t* packed4, int64_t elems, int k, uint8_t* stream, hipStream_t st) {
  if (elems <= 0 || elems % 32 != 0) return hipErrorInvalidValue;
  const int64_t groups = elems / 32;
  if (k == 2)
    hipLaunchKernelGGL(kbit_pack_kernel<2>, dim3(kbit_grid(groups)), dim3(kKbitThreads), 0, st, (const uint4*)packed4,
                       (uint32_t*)stream, groups);
  else if (k == 3)
    hipLaunchKernelGGL(kbit_pack_kernel<3>, dim3(kbit_grid(groups)), dim3(kKbitThreads), 0, st, (const uint4*)packed4,
                       (uint32_t*)stream, groups);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_kbit_unpack(const uint8_t* stream, int64_t elems, int k, uint8_t* packed4, hipStream_t st) {
  if (elems <= 0 || elems % 32 != 0) return hipErrorInvalidValue;
  const int64_t groups = elems / 32;
  if (k == 2)
    hipLaunchKernelGGL(kbit_unpack_kernel<2>, dim3(kbit_grid(groups)), dim3(kKbitThreads), 0, st, (const uint32_t*)stream,
                       (uint4*)packed4, groups);
  else if (k == 3)
    hipLaunchKernelGGL(kbit_unpack_kernel<3>, dim3(kbit_grid(groups)), dim3(kKbitThreads), 0, st, (const uint32_t*)stream,
                       (uint4*)packed4, groups);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace qlora
