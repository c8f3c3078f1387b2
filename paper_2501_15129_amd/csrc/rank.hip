// es_rank: centred-rank fitness shaping.  rank_i counts the individuals that precede i in
// the order "fitness ascending, ties by index"; shaped_i = rank_i / (N - 1) - 1/2.
//
// Integer work on an order-preserving key of the binary32 pattern, N^2 comparisons spread
// over N/16 workgroups: 16 lanes (one DPP row) share one individual and split the others.
// Latency-bound (N <= a few thousand): 8 bytes per individual.
#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

__device__ __forceinline__ uint32_t order_key(float f) {
  f = f + 0.0f;                                   // -0 -> +0
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr uint32_t RANK_TILE = 4096;

__global__ __launch_bounds__(256) void rank_kernel(const float* __restrict__ fit, int32_t* __restrict__ rank,
                                                   float* __restrict__ shaped, uint32_t n) {
  __shared__ uint32_t keys[RANK_TILE];
  const uint32_t i = blockIdx.x * 16u + (threadIdx.x >> 4);
  const uint32_t part = threadIdx.x & 15u;
  const uint32_t ki = i < n ? order_key(fit[i]) : 0u;
  uint32_t cnt = 0;
  for (uint32_t base = 0; base < n; base += RANK_TILE) {
    const uint32_t len = min(RANK_TILE, n - base);
    __syncthreads();
    // all loads of this tile are issued before any is used (16 independent loads per thread)
    float f[RANK_TILE / 256];
#pragma unroll
    for (uint32_t r = 0; r < RANK_TILE / 256; ++r) {
      const uint32_t t = threadIdx.x + 256u * r;
      f[r] = t < len ? fit[base + t] : 0.0f;
    }
#pragma unroll
    for (uint32_t r = 0; r < RANK_TILE / 256; ++r) {
      const uint32_t t = threadIdx.x + 256u * r;
      if (t < len) keys[t] = order_key(f[r]);
    }
    __syncthreads();
    uint32_t t = part;
    for (; t + 48u < len; t += 64u) {          // four independent compares per iteration
#pragma unroll
      for (uint32_t r = 0; r < 4; ++r) {
        const uint32_t kj = keys[t + 16u * r];
        const uint32_t j = base + t + 16u * r;
        cnt += (kj < ki || (kj == ki && j < i)) ? 1u : 0u;
      }
    }
    for (; t < len; t += 16u) {
      const uint32_t kj = keys[t];
      const uint32_t j = base + t;
      cnt += (kj < ki || (kj == ki && j < i)) ? 1u : 0u;
    }
  }
  cnt += __shfl_xor(cnt, 8, 64);
  cnt += __shfl_xor(cnt, 4, 64);
  cnt += __shfl_xor(cnt, 2, 64);
  cnt += __shfl_xor(cnt, 1, 64);
  if (part == 0 && i < n) {
    rank[i] = (int32_t)cnt;
    shaped[i] = n > 1 ? ((float)cnt / (float)(n - 1)) - 0.5f : 0.0f;
  }
}

int launch_rank(es_ctx* ctx, const float* fit, int32_t* rank, float* shaped, hipStream_t st) {
  const uint32_t n = ctx->shp.N;
  hipLaunchKernelGGL(rank_kernel, dim3((n + 15) / 16), dim3(256), 0, st, fit, rank, shaped, n);
  return check_launch(ctx, "es_rank");
}

}  // namespace es
