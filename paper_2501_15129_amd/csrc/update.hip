// es_update: search-gradient estimate g = noise^T w / (N sigma) followed by an Adam step
// (paper App. B Table 5b: OpenES with Adam, lr 0.01, weight decay 0.005, noise std 0.02).
//
// Two paths, both deterministic and both streaming the noise matrix exactly once:
//  * large matrices (two kernels): stage 1 below writes binary64 partial rows per chunk of rows,
//    stage 2 adds them and applies Adam - the split keeps >2000 workgroups in flight, which
//    is what the HBM needs at 0.5 GB;
//  * small and medium matrices (one kernel): a workgroup of eight wavefronts owns its columns for
//    ALL rows and applies Adam itself - no partials, one launch (the launch is what costs there).
// A third path serves contexts that store no noise at all (paper Sec. 5.1: perturbations generated
// on the fly): stage 1 recomputes every noise value from the counter stream instead of reading it -
// bound by the integer/floating-point ALUs (one Philox block and two Gaussian transforms per four
// values), with zero noise bytes in HBM - and stage 2 is shared.
//
// Stage 1 streams the noise matrix exactly once (HBM-bound: rows * ld * sizeof(elt) bytes,
// ~1 flop per byte).  A workgroup owns a tile of 64*VEC consecutive columns and one chunk
// of rows; its four wavefronts take every fourth row, each lane loads 16 bytes per row
// (fully coalesced 1 KiB per wavefront) and accumulates in binary64 - the fp64 vector rate
// of this chip is far above what the stream needs, and binary64 sums make the result
// independent of the row split to ~1e-16.  The four wavefronts are combined through LDS in
// a fixed order and written as one binary64 partial row per chunk.
// Stage 2 adds the partials in chunk order and applies Adam in binary64 per parameter.
// No atomics anywhere: reruns are bit-identical.
#include <cmath>

#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

constexpr uint32_t UPD_MAX_ROWS_PER_CHUNK = 1024;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool BF16>
struct NoiseVec;
template <>
struct NoiseVec<true> {
  static constexpr int VEC = 8;
  using Raw = u32x4;
  __device__ static __forceinline__ void unpack(const Raw& r, float (&f)[8]) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xFFFF0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xFFFF0000u);
  }
};
template <>
struct NoiseVec<false> {
  static constexpr int VEC = 4;
  using Raw = f32x4;
  __device__ static __forceinline__ void unpack(const Raw& r, float (&f)[4]) {
    f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
  }
};

// TABLE: the rows are slices of the shared noise table (their starts come from `offs`); a compile-time
// choice, so that the plain matrix path keeps its pointer arithmetic free of LDS look-ups.
template <bool BF16, bool TABLE>
__global__ __launch_bounds__(256) void grad_partial_kernel(const void* __restrict__ noise,
                                                           const uint32_t* __restrict__ offs,
                                                           const float* __restrict__ shaped,
                                                           double* __restrict__ partial, uint32_t rows,
                                                           uint32_t ld, uint32_t rows_per_chunk,
                                                           uint32_t antithetic) {
  using NV = NoiseVec<BF16>;
  constexpr int VEC = NV::VEC;
  using Raw = typename NV::Raw;
  __shared__ double coef[UPD_MAX_ROWS_PER_CHUNK];
  __shared__ uint32_t rowoff[TABLE ? UPD_MAX_ROWS_PER_CHUNK : 1];     // start of each table row in Raw units
  __shared__ double red[4][64 * VEC];

  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t r0 = blockIdx.y * rows_per_chunk;
  const uint32_t r1 = min(rows, r0 + rows_per_chunk);
  const uint32_t col0 = blockIdx.x * (64u * VEC);

  for (uint32_t r = r0 + threadIdx.x; r < r1; r += 256u) {
    coef[r - r0] = antithetic ? (double)shaped[2 * r] - (double)shaped[2 * r + 1] : (double)shaped[r];
    if (TABLE) rowoff[r - r0] = offs[r] / VEC;
  }
  __syncthreads();

  double acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.0;

  const Raw* base = reinterpret_cast<const Raw*>(noise) + ((size_t)col0 / VEC + lane);
  const size_t row_stride = ld / VEC;   // in Raw units
  // matrix rows are read once and never again (non-temporal); table rows overlap and may be read again (cached)
  auto load_row = [&](uint32_t rr) {
    if (TABLE) return base[rowoff[TABLE ? rr - r0 : 0]];
    return __builtin_nontemporal_load(base + (size_t)rr * row_stride);
  };
  uint32_t r = r0 + wave;
  for (; r + 12u < r1; r += 16u) {      // four rows of this wavefront in flight
    Raw q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) q[u] = load_row(r + 4u * u);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float f[VEC];
      NV::unpack(q[u], f);
      const double c = coef[r + 4u * u - r0];
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = fma(c, (double)f[v], acc[v]);
    }
  }
  for (; r < r1; r += 4u) {
    const Raw q = load_row(r);
    float f[VEC];
    NV::unpack(q, f);
    const double c = coef[r - r0];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = fma(c, (double)f[v], acc[v]);
  }

#pragma unroll
  for (int v = 0; v < VEC; ++v) red[wave][lane * VEC + v] = acc[v];
  __syncthreads();
  double* out = partial + (size_t)blockIdx.y * ld + col0;
  for (uint32_t c = threadIdx.x; c < 64u * VEC; c += 256u)
    out[c] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
}

// Stage 1 without a noise matrix: thread = four consecutive columns (one counter block per row),
// workgroup = 1024 columns x one chunk of rows.
__global__ __launch_bounds__(256) void grad_regen_kernel(const float* __restrict__ shaped, double* __restrict__ partial,
                                                         uint32_t rows, uint32_t ld, uint32_t D,
                                                         uint32_t rows_per_chunk, uint32_t antithetic, uint32_t round_bf16,
                                                         uint32_t gen, uint32_t k0, uint32_t k1) {
  __shared__ double coef[UPD_MAX_ROWS_PER_CHUNK];
  const uint32_t r0 = blockIdx.y * rows_per_chunk;
  const uint32_t r1 = min(rows, r0 + rows_per_chunk);
  for (uint32_t r = r0 + threadIdx.x; r < r1; r += 256u)
    coef[r - r0] = antithetic ? (double)shaped[2 * r] - (double)shaped[2 * r + 1] : (double)shaped[r];
  __syncthreads();
  const uint32_t d0 = 4u * (blockIdx.x * 256u + threadIdx.x);
  if (d0 >= D) return;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (uint32_t r = r0; r < r1; ++r) {
    float z[4];
    noise_regen4(r, d0, gen, k0, k1, round_bf16 != 0u, z);
    const double c = coef[r - r0];
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = fma(c, (double)z[k], acc[k]);
  }
  double* out = partial + (size_t)blockIdx.y * ld + d0;       // ld is a multiple of 4: columns D..ld-1 are never read
#pragma unroll
  for (int k = 0; k < 4; ++k) out[k] = acc[k];
}

// The parameter step that follows the noise reduction, per strategy (paper Sec. 4, App. B Table 5):
// OpenES = Adam on -g + weight_decay * theta; ARS and VanillaES = theta + step * g, no optimiser state.
struct AdamArgs {
  double inv_scale;      // the reduced sum is divided by this: N sigma (OpenES), b (ARS), 1 / sigma (VanillaES)
  double lr, b1, b2, eps, wd, corr1, corr2;
  double step;           // additive mode: lr (ARS) or 1 (VanillaES)
  uint32_t additive;     // 0: Adam ; 1: theta += step * g
};

__device__ __forceinline__ void apply_step(const AdamArgs& ad, double sum, uint32_t d, float* __restrict__ theta,
                                           float* __restrict__ m, float* __restrict__ v, float* __restrict__ grad) {
  const double g = sum / ad.inv_scale;
  const double th = (double)theta[d];
  if (grad) grad[d] = (float)g;
  if (ad.additive) {
    theta[d] = (float)(th + ad.step * g);
    return;
  }
  const double gr = -g + ad.wd * th;
  const double mn = ad.b1 * (double)m[d] + (1.0 - ad.b1) * gr;
  const double vn = ad.b2 * (double)v[d] + (1.0 - ad.b2) * gr * gr;
  const double mhat = mn / ad.corr1, vhat = vn / ad.corr2;
  m[d] = (float)mn;
  v[d] = (float)vn;
  theta[d] = (float)(th - ad.lr * mhat / (sqrt(vhat) + ad.eps));
}

__global__ __launch_bounds__(256) void adam_kernel(const double* __restrict__ partial, uint32_t chunks,
                                                   uint32_t ld, uint32_t D, const AdamArgs ad,
                                                   float* __restrict__ theta, float* __restrict__ m,
                                                   float* __restrict__ v, float* __restrict__ grad) {
  const uint32_t d = blockIdx.x * 256u + threadIdx.x;
  if (d >= D) return;
  double g = 0.0;
  for (uint32_t c = 0; c < chunks; ++c) g += partial[(size_t)c * ld + d];
  apply_step(ad, g, d, theta, m, v, grad);
}

constexpr int UPD1_WAVES = 8;        // single-pass kernel: wavefronts per workgroup
constexpr int UPD1_INFLIGHT = 8;     // ... and rows of one wavefront in flight
constexpr uint32_t UPD_COEF_ROWS = 2048;   // row weights staged in LDS per pass


template <bool BF16, bool TABLE>
__global__ __launch_bounds__(64 * UPD1_WAVES) void update_single_pass_kernel(const void* __restrict__ noise,
                                                                const uint32_t* __restrict__ offs,
                                                                const float* __restrict__ shaped, uint32_t rows,
                                                                uint32_t ld, uint32_t D, uint32_t antithetic,
                                                                const AdamArgs ad, float* __restrict__ theta,
                                                                float* __restrict__ m, float* __restrict__ v,
                                                                float* __restrict__ grad) {
  using NQ = NoiseVec<BF16>;
  using Raw = typename NQ::Raw;
  constexpr int VEC = NQ::VEC, UPD_TILE = 64 * VEC;
  __shared__ double coef[UPD_COEF_ROWS];
  __shared__ uint32_t rowoff[TABLE ? UPD_COEF_ROWS : 1];     // shared noise table: start of each row in Raw units
  __shared__ double red[UPD1_WAVES][UPD_TILE];

  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t col0 = blockIdx.x * UPD_TILE;
  const Raw* base = reinterpret_cast<const Raw*>(noise) + ((size_t)col0 / VEC + lane);
  const size_t row_stride = ld / VEC;     // in Raw units
  auto load_row = [&](uint32_t rb, uint32_t r) {     // row rb + r; table rows are placed by rowoff instead
    if (TABLE) return __builtin_nontemporal_load(base + rowoff[TABLE ? r : 0]);
    return __builtin_nontemporal_load(base + (size_t)(rb + r) * row_stride);
  };

  double acc[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] = 0.0;
  for (uint32_t rb = 0; rb < rows; rb += UPD_COEF_ROWS) {
    const uint32_t rn = min(UPD_COEF_ROWS, rows - rb);
    __syncthreads();
    for (uint32_t r = threadIdx.x; r < rn; r += 64u * UPD1_WAVES) {
      coef[r] = antithetic ? (double)shaped[2 * (rb + r)] - (double)shaped[2 * (rb + r) + 1] : (double)shaped[rb + r];
      if (TABLE) rowoff[r] = offs[rb + r] / VEC;
    }
    __syncthreads();
    uint32_t r = wave;
    for (; r + UPD1_WAVES * (UPD1_INFLIGHT - 1) < rn; r += UPD1_WAVES * UPD1_INFLIGHT) {
      Raw q[UPD1_INFLIGHT];
#pragma unroll
      for (int u = 0; u < UPD1_INFLIGHT; ++u)
        q[u] = load_row(rb, r + UPD1_WAVES * u);
#pragma unroll
      for (int u = 0; u < UPD1_INFLIGHT; ++u) {
        float f[VEC];
        NQ::unpack(q[u], f);
        const double c = coef[r + UPD1_WAVES * u];
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] = fma(c, (double)f[k], acc[k]);
      }
    }
    for (; r < rn; r += UPD1_WAVES) {
      const Raw q = load_row(rb, r);
      float f[VEC];
      NQ::unpack(q, f);
      const double c = coef[r];
#pragma unroll
      for (int k = 0; k < VEC; ++k) acc[k] = fma(c, (double)f[k], acc[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) red[wave][lane * VEC + k] = acc[k];
  __syncthreads();

  // Adam on this workgroup's 256 parameters (columns past D are padding)
  for (uint32_t c = threadIdx.x; c < (uint32_t)UPD_TILE; c += 64u * UPD1_WAVES) {
    const uint32_t d = col0 + c;
    if (d >= D) break;
    double g = red[0][c];
#pragma unroll
    for (int w = 1; w < UPD1_WAVES; ++w) g += red[w][c];
    apply_step(ad, g, d, theta, m, v, grad);
  }
}


// Row chunks of the regenerating stage 1: enough workgroups to fill every SIMD several times over.
uint32_t update_chunks_regen(uint32_t rows, uint32_t D) {
  const uint32_t wgs_per_chunk = ((D + 3u) / 4u + 255u) / 256u;
  uint32_t chunks = std::max(1u, std::min(rows, (2048u + wgs_per_chunk - 1u) / wgs_per_chunk));
  while ((rows + chunks - 1) / chunks > UPD_MAX_ROWS_PER_CHUNK) ++chunks;
  return chunks;
}

uint32_t update_chunks(uint32_t rows, uint32_t ld, bool bf16) {
  const uint32_t tile = 64u * (bf16 ? 8u : 4u);
  const uint32_t col_tiles = ld / tile;
  if ((uint64_t)rows * ld * (bf16 ? 2u : 4u) < (256ull << 20)) return 1;     // single-pass kernel
  uint32_t chunks = (2048u + col_tiles - 1) / col_tiles;
  chunks = std::min(chunks, std::max(1u, rows / 16u));
  while ((rows + chunks - 1) / chunks > UPD_MAX_ROWS_PER_CHUNK) ++chunks;
  return chunks;
}

static AdamArgs step_args(const es_ctx* ctx, uint64_t step) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  AdamArgs ad;
  ad.b1 = (double)c.beta1; ad.b2 = (double)c.beta2;
  ad.corr1 = 1.0 - std::pow(ad.b1, (double)step);
  ad.corr2 = 1.0 - std::pow(ad.b2, (double)step);
  ad.lr = (double)c.lr; ad.eps = (double)c.adam_eps; ad.wd = (double)c.weight_decay;
  ad.additive = c.algorithm != ES_OPENES;
  ad.step = c.algorithm == ES_ARS ? (double)c.lr : 1.0;
  ad.inv_scale = c.algorithm == ES_ARS ? (double)c.num_elites
               : c.algorithm == ES_VANILLA ? 1.0 / (double)c.sigma
                                           : (double)s.N * (double)c.sigma;
  return ad;
}

int launch_update(es_ctx* ctx, uint64_t step, const void* noise, const float* shaped, float* theta,
                  float* m, float* v, float* grad, void* ws, hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  const NoiseView nv = noise_view(ctx, noise);
  const bool bf16 = nv.mode == 1;
  const uint32_t chunks = ctx->upd_chunks;
  const AdamArgs ad = step_args(ctx, step);
  noise = nv.base;
  if (nv.mode >= 2) {
    const uint32_t rpc = (s.rows + chunks - 1) / chunks;
    double* partial = static_cast<double*>(ws);
    const dim3 grid(((s.D + 3u) / 4u + 255u) / 256u, chunks);       // one thread per group of four columns
    hipLaunchKernelGGL(grad_regen_kernel, grid, dim3(256), 0, st, shaped, partial, s.rows, s.ld, s.D, rpc, c.antithetic,
                       nv.mode == 3 ? 1u : 0u, ctx->regen_generation, (uint32_t)c.seed, (uint32_t)(c.seed >> 32));
    int rc = check_launch(ctx, "es_update (regenerated gradient partials)");
    if (rc != ES_OK) return rc;
    hipLaunchKernelGGL(adam_kernel, dim3((s.D + 255) / 256), dim3(256), 0, st, partial, chunks, s.ld, s.D, ad,
                       theta, m, v, grad);
    return check_launch(ctx, "es_update (parameter step)");
  }
  const bool table = nv.offs != nullptr;
  if (chunks == 1) {
    const dim3 grid1(s.ld / (64 * (bf16 ? 8 : 4))), block1(64 * UPD1_WAVES);
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, grid1, block1, 0, st, noise, nv.offs, shaped, s.rows, s.ld, s.D, c.antithetic, ad, theta, m, v, grad);
    };
    if (bf16) { if (table) go(update_single_pass_kernel<true, true>); else go(update_single_pass_kernel<true, false>); }
    else { if (table) go(update_single_pass_kernel<false, true>); else go(update_single_pass_kernel<false, false>); }
    return check_launch(ctx, "es_update (single pass)");
  }
  const uint32_t rpc = (s.rows + chunks - 1) / chunks;
  const uint32_t tile = 64u * (bf16 ? 8u : 4u);
  double* partial = static_cast<double*>(ws);
  dim3 grid(s.ld / tile, chunks);
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, grid, dim3(256), 0, st, noise, nv.offs, shaped, partial, s.rows, s.ld, rpc, c.antithetic);
  };
  if (bf16) { if (table) go(grad_partial_kernel<true, true>); else go(grad_partial_kernel<true, false>); }
  else { if (table) go(grad_partial_kernel<false, true>); else go(grad_partial_kernel<false, false>); }
  int rc = check_launch(ctx, "es_update (gradient partials)");
  if (rc != ES_OK) return rc;
  hipLaunchKernelGGL(adam_kernel, dim3((s.D + 255) / 256), dim3(256), 0, st, partial, chunks, s.ld, s.D, ad,
                     theta, m, v, grad);
  return check_launch(ctx, "es_update (parameter step)");
}

}  // namespace es
