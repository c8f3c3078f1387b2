// es_sample_population: the noise matrix of one generation, generated on the fly from a
// counter-based stream (paper Sec. 5.1: perturbations are not read from a pre-built table).
//
// One thread turns one Philox block into four consecutive columns of one row.  The matrix
// is written once, with full-width coalesced vector stores; columns past D are zero.
// Bound: integer/fp ALU work (10 Philox rounds + two Box-Muller evaluations per 4 values),
// then the HBM write of rows * ld elements.
#include <algorithm>

#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <bool BF16>
__global__ __launch_bounds__(256) void sample_kernel(void* __restrict__ noise, uint32_t rows, uint32_t D, uint32_t ld,
                                                     uint32_t gen, uint32_t k0, uint32_t k1) {
  const uint32_t blk = blockIdx.x * 256u + threadIdx.x;   // 4-column block within the row
  if (blk * 4u >= ld) return;
  const uint32_t d0 = blk * 4u;
  // grid.y is capped at the launch limit: populations beyond it take several rows per workgroup
  for (uint32_t row = blockIdx.y; row < rows; row += gridDim.y) {
    float z0 = 0.f, z1 = 0.f, z2 = 0.f, z3 = 0.f;
    if (d0 < D) {
      const Words4 w = philox4x32_10(blk, row, gen, STREAM_NOISE, k0, k1);
      gauss_pair(w.x, w.y, z0, z1);
      gauss_pair(w.z, w.w, z2, z3);
      if (d0 + 1 >= D) z1 = 0.f;
      if (d0 + 2 >= D) z2 = 0.f;
      if (d0 + 3 >= D) z3 = 0.f;
    }
    const size_t off = (size_t)row * ld + d0;
    if (BF16) {
      uint2 v;      // packed hardware convert: round to nearest even, the same result as the integer formula
      v.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{z0, z1}, bf16x2));
      v.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{z2, z3}, bf16x2));
      *reinterpret_cast<uint2*>(static_cast<uint16_t*>(noise) + off) = v;
    } else {
      *reinterpret_cast<float4*>(static_cast<float*>(noise) + off) = make_float4(z0, z1, z2, z3);
    }
  }
}

// The shared noise table (paper Sec. 5.1: the variant with a table built once; Salimans et al. 2017):
// the same work as a noise row, on stream 3, counter (t / 4, 0, 0, 3); one thread = four entries.
template <bool BF16>
__global__ __launch_bounds__(256) void table_kernel(void* __restrict__ table, uint32_t len, uint32_t k0, uint32_t k1) {
  const uint32_t blk = blockIdx.x * 256u + threadIdx.x;
  if (blk * 4u >= len) return;                    // len is a multiple of 8
  const Words4 w = philox4x32_10(blk, 0u, 0u, STREAM_TABLE, k0, k1);
  float z0, z1, z2, z3;
  gauss_pair(w.x, w.y, z0, z1);
  gauss_pair(w.z, w.w, z2, z3);
  const size_t off = (size_t)blk * 4u;
  if (BF16) {
    uint2 v;
    v.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{z0, z1}, bf16x2));
    v.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{z2, z3}, bf16x2));
    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(table) + off) = v;
  } else {
    *reinterpret_cast<float4*>(static_cast<float*>(table) + off) = make_float4(z0, z1, z2, z3);
  }
}

// Where each noise row of this generation starts in the table: 8 * (x mod M), x from stream 4.
__global__ __launch_bounds__(256) void table_offsets_kernel(uint32_t* __restrict__ offs, uint32_t rows, uint32_t M,
                                                            uint32_t gen, uint32_t k0, uint32_t k1) {
  const uint32_t j = blockIdx.x * 256u + threadIdx.x;
  if (j >= rows) return;
  const Words4 w = philox4x32_10(j, gen, 0u, STREAM_OFFSET, k0, k1);
  offs[j] = 8u * (w.x % M);
}

int launch_table(es_ctx* ctx, void* noise, hipStream_t st) {
  const uint32_t len = (uint32_t)ctx->cfg.noise_table_len;
  const uint32_t k0 = (uint32_t)ctx->cfg.seed, k1 = (uint32_t)(ctx->cfg.seed >> 32);
  const dim3 grid((len / 4 + 255) / 256);
  if (ctx->cfg.noise_dtype == 5) hipLaunchKernelGGL(table_kernel<true>, grid, dim3(256), 0, st, noise, len, k0, k1);
  else hipLaunchKernelGGL(table_kernel<false>, grid, dim3(256), 0, st, noise, len, k0, k1);
  return check_launch(ctx, "es_build_noise_table");
}

int launch_table_offsets(es_ctx* ctx, uint32_t gen, void* noise, hipStream_t st) {
  const Shape& s = ctx->shp;
  const NoiseView nv = noise_view(ctx, noise);
  const uint32_t M = (uint32_t)((ctx->cfg.noise_table_len - s.ld) / 8u + 1u);
  hipLaunchKernelGGL(table_offsets_kernel, dim3((s.rows + 255) / 256), dim3(256), 0, st, const_cast<uint32_t*>(nv.offs),
                     s.rows, M, gen, (uint32_t)ctx->cfg.seed, (uint32_t)(ctx->cfg.seed >> 32));
  return check_launch(ctx, "es_sample_population (table offsets)");
}

int launch_sample(es_ctx* ctx, uint32_t gen, void* noise, hipStream_t st) {
  const Shape& s = ctx->shp;
  const uint32_t k0 = (uint32_t)ctx->cfg.seed, k1 = (uint32_t)(ctx->cfg.seed >> 32);
  dim3 grid((s.ld / 4 + 255) / 256, std::min(s.rows, 65535u));
  if (ctx->cfg.noise_dtype == 1)
    hipLaunchKernelGGL(sample_kernel<true>, grid, dim3(256), 0, st, noise, s.rows, s.D, s.ld, gen, k0, k1);
  else
    hipLaunchKernelGGL(sample_kernel<false>, grid, dim3(256), 0, st, noise, s.rows, s.D, s.ld, gen, k0, k1);
  return check_launch(ctx, "es_sample_population");
}

}  // namespace es
