// es_rank: fitness shaping.  OpenES: centred ranks; rank_i counts the individuals that precede i in
// the order "fitness ascending, ties by index"; shaped_i = rank_i / (N - 1) - 1/2.  The selection
// steps of ARS and VanillaES follow further down.
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

// ---- selection steps of the sibling strategies (paper Sec. 4; App. B Tables 5a, 5c) ----
// Populations of these strategies are small (the paper uses 128), so one workgroup does the
// whole step: keys in LDS, each thread ranks its own entries against all others (integer
// compares, bit-exact), binary64 sums are reduced through LDS in a fixed tree order.
constexpr uint32_t SEL_THREADS = 1024;
constexpr uint32_t SEL_MAX = 8192;

__device__ __forceinline__ double block_sum(double v, double* red) {
  red[threadIdx.x] = v;
  __syncthreads();
  for (uint32_t s = SEL_THREADS / 2; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

// ARS (Mania et al. 2018): keep the b best mirrored directions by max(F+, F-); divide the kept
// returns by their standard deviation.
__global__ __launch_bounds__(SEL_THREADS) void rank_ars_kernel(const float* __restrict__ fit, int32_t* __restrict__ rank,
                                                               float* __restrict__ shaped, uint32_t n, uint32_t b) {
  __shared__ uint32_t keys[SEL_MAX / 2];
  __shared__ double red[SEL_THREADS];
  const uint32_t R = n / 2;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS) {
    const uint32_t a0 = order_key(fit[2 * j]), a1 = order_key(fit[2 * j + 1]);
    keys[j] = a0 > a1 ? a0 : a1;
  }
  __syncthreads();
  double sum = 0.0, cnt = 0.0;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS) {
    const uint32_t kj = keys[j];
    uint32_t pos = 0;
    for (uint32_t l = 0; l < R; ++l) {
      const uint32_t kl = keys[l];
      pos += (kl > kj || (kl == kj && l < j)) ? 1u : 0u;
    }
    rank[2 * j] = (int32_t)pos;
    rank[2 * j + 1] = (int32_t)pos;
    if (pos < b) { sum += (double)fit[2 * j] + (double)fit[2 * j + 1]; cnt += 2.0; }
  }
  const double total = block_sum(sum, red), count = block_sum(cnt, red);
  const double mean = count > 0.0 ? total / count : 0.0;
  double var = 0.0;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS) {
    if ((uint32_t)rank[2 * j] < b) {          // this thread's own earlier write
      const double d0 = (double)fit[2 * j] - mean, d1 = (double)fit[2 * j + 1] - mean;
      var += d0 * d0 + d1 * d1;
    }
  }
  const double sigma_r = count > 0.0 ? sqrt(block_sum(var, red) / count) : 0.0;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS) {
    const bool kept = (uint32_t)rank[2 * j] < b && sigma_r > 0.0;
    shaped[2 * j] = kept ? (float)((double)fit[2 * j] / sigma_r) : 0.0f;
    shaped[2 * j + 1] = kept ? (float)((double)fit[2 * j + 1] / sigma_r) : 0.0f;
  }
}

// VanillaES (Chrabaszcz et al. 2018): the mu best offspring get the log-rank recombination weights.
__global__ __launch_bounds__(SEL_THREADS) void rank_vanilla_kernel(const float* __restrict__ fit, int32_t* __restrict__ rank,
                                                                   float* __restrict__ shaped, uint32_t n, uint32_t mu) {
  __shared__ uint32_t keys[SEL_MAX];
  __shared__ double red[SEL_THREADS];
  for (uint32_t i = threadIdx.x; i < n; i += SEL_THREADS) keys[i] = order_key(fit[i]);
  __syncthreads();
  const double top = log((double)mu + 0.5);
  double part = 0.0;
  for (uint32_t k = threadIdx.x + 1; k <= mu; k += SEL_THREADS) part += top - log((double)k);
  const double wsum = block_sum(part, red);
  for (uint32_t i = threadIdx.x; i < n; i += SEL_THREADS) {
    const uint32_t ki = keys[i];
    uint32_t pos = 0;
    for (uint32_t l = 0; l < n; ++l) {
      const uint32_t kl = keys[l];
      pos += (kl > ki || (kl == ki && l < i)) ? 1u : 0u;
    }
    rank[i] = (int32_t)pos;
    shaped[i] = pos < mu ? (float)((top - log((double)pos + 1.0)) / wsum) : 0.0f;
  }
}

// ---- the same two selections for populations in the thousands: the N^2 comparisons spread over the chip ----
// Stage 1 (items / 16 workgroups): position of every item - a mirrored direction keyed by max(F+, F-) for ARS, an
// individual for VanillaES - in descending key order, ties to the lower index; 16 lanes share one item, as in
// rank_kernel.  Stage 2 (one workgroup, O(N) work): the statistics over the kept items and the shaped values.
template <bool PAIRS>
__global__ __launch_bounds__(256) void select_pos_kernel(const float* __restrict__ fit, int32_t* __restrict__ rank,
                                                         uint32_t items) {
  __shared__ uint32_t keys[SEL_MAX];
  for (uint32_t j = threadIdx.x; j < items; j += 256u) {
    if (PAIRS) {
      const uint32_t a0 = order_key(fit[2 * j]), a1 = order_key(fit[2 * j + 1]);
      keys[j] = a0 > a1 ? a0 : a1;
    } else {
      keys[j] = order_key(fit[j]);
    }
  }
  __syncthreads();
  const uint32_t i = blockIdx.x * 16u + (threadIdx.x >> 4);
  const uint32_t part = threadIdx.x & 15u;
  const uint32_t ki = i < items ? keys[i] : 0u;
  uint32_t cnt = 0;
  uint32_t t = part;
  for (; t + 48u < items; t += 64u) {
#pragma unroll
    for (uint32_t r = 0; r < 4; ++r) {
      const uint32_t kl = keys[t + 16u * r], l = t + 16u * r;
      cnt += (kl > ki || (kl == ki && l < i)) ? 1u : 0u;
    }
  }
  for (; t < items; t += 16u) {
    const uint32_t kl = keys[t];
    cnt += (kl > ki || (kl == ki && t < i)) ? 1u : 0u;
  }
  cnt += __shfl_xor(cnt, 8, 64);
  cnt += __shfl_xor(cnt, 4, 64);
  cnt += __shfl_xor(cnt, 2, 64);
  cnt += __shfl_xor(cnt, 1, 64);
  if (part == 0 && i < items) {
    if (PAIRS) { rank[2 * i] = (int32_t)cnt; rank[2 * i + 1] = (int32_t)cnt; }
    else rank[i] = (int32_t)cnt;
  }
}

__global__ __launch_bounds__(SEL_THREADS) void shape_ars_kernel(const float* __restrict__ fit, const int32_t* __restrict__ rank,
                                                                float* __restrict__ shaped, uint32_t n, uint32_t b) {
  __shared__ double red[SEL_THREADS];
  const uint32_t R = n / 2;
  double sum = 0.0, cnt = 0.0;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS)
    if ((uint32_t)rank[2 * j] < b) { sum += (double)fit[2 * j] + (double)fit[2 * j + 1]; cnt += 2.0; }
  const double total = block_sum(sum, red), count = block_sum(cnt, red);
  const double mean = count > 0.0 ? total / count : 0.0;
  double var = 0.0;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS) {
    if ((uint32_t)rank[2 * j] < b) {
      const double d0 = (double)fit[2 * j] - mean, d1 = (double)fit[2 * j + 1] - mean;
      var += d0 * d0 + d1 * d1;
    }
  }
  const double sigma_r = count > 0.0 ? sqrt(block_sum(var, red) / count) : 0.0;
  for (uint32_t j = threadIdx.x; j < R; j += SEL_THREADS) {
    const bool kept = (uint32_t)rank[2 * j] < b && sigma_r > 0.0;
    shaped[2 * j] = kept ? (float)((double)fit[2 * j] / sigma_r) : 0.0f;
    shaped[2 * j + 1] = kept ? (float)((double)fit[2 * j + 1] / sigma_r) : 0.0f;
  }
}

__global__ __launch_bounds__(SEL_THREADS) void shape_vanilla_kernel(const int32_t* __restrict__ rank, float* __restrict__ shaped,
                                                                    uint32_t n, uint32_t mu) {
  __shared__ double red[SEL_THREADS];
  const double top = log((double)mu + 0.5);
  double part = 0.0;
  for (uint32_t k = threadIdx.x + 1; k <= mu; k += SEL_THREADS) part += top - log((double)k);
  const double wsum = block_sum(part, red);
  for (uint32_t i = threadIdx.x; i < n; i += SEL_THREADS) {
    const uint32_t pos = (uint32_t)rank[i];
    shaped[i] = pos < mu ? (float)((top - log((double)pos + 1.0)) / wsum) : 0.0f;
  }
}

constexpr uint32_t SEL_ONE_WORKGROUP_MAX = 512;   // up to here one launch of one workgroup is faster than two launches

int launch_rank(es_ctx* ctx, const float* fit, int32_t* rank, float* shaped, hipStream_t st) {
  const uint32_t n = ctx->shp.N;
  if (ctx->cfg.algorithm == ES_ARS) {
    if (n <= SEL_ONE_WORKGROUP_MAX) {
      hipLaunchKernelGGL(rank_ars_kernel, dim3(1), dim3(SEL_THREADS), 0, st, fit, rank, shaped, n, ctx->cfg.num_elites);
      return check_launch(ctx, "es_rank (ARS)");
    }
    hipLaunchKernelGGL(select_pos_kernel<true>, dim3((n / 2 + 15) / 16), dim3(256), 0, st, fit, rank, n / 2);
    if (int rc = check_launch(ctx, "es_rank (ARS positions)")) return rc;
    hipLaunchKernelGGL(shape_ars_kernel, dim3(1), dim3(SEL_THREADS), 0, st, fit, rank, shaped, n, ctx->cfg.num_elites);
    return check_launch(ctx, "es_rank (ARS statistics)");
  }
  if (ctx->cfg.algorithm == ES_VANILLA) {
    if (n <= SEL_ONE_WORKGROUP_MAX) {
      hipLaunchKernelGGL(rank_vanilla_kernel, dim3(1), dim3(SEL_THREADS), 0, st, fit, rank, shaped, n, ctx->cfg.num_elites);
      return check_launch(ctx, "es_rank (VanillaES)");
    }
    hipLaunchKernelGGL(select_pos_kernel<false>, dim3((n + 15) / 16), dim3(256), 0, st, fit, rank, n);
    if (int rc = check_launch(ctx, "es_rank (VanillaES positions)")) return rc;
    hipLaunchKernelGGL(shape_vanilla_kernel, dim3(1), dim3(SEL_THREADS), 0, st, rank, shaped, n, ctx->cfg.num_elites);
    return check_launch(ctx, "es_rank (VanillaES weights)");
  }
  hipLaunchKernelGGL(rank_kernel, dim3((n + 15) / 16), dim3(256), 0, st, fit, rank, shaped, n);
  return check_launch(ctx, "es_rank");
}

}  // namespace es
