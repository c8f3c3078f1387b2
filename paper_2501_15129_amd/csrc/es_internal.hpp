// Internal declarations shared by the host API and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>

#include "../../include/es.h"

namespace es {

enum RolloutKind : int {
  ROLLOUT_WAVE_LDS = 0,   // one wavefront per (individual, env); weights in LDS
  ROLLOUT_MFMA_REG = 1,   // one workgroup per individual; bf16 weights resident in registers, MFMA
  ROLLOUT_WAVE_REG = 2,   // one wavefront per (individual, env); binary32 weights resident in registers
  ROLLOUT_MFMA_F32 = 3,   // one workgroup per individual; binary32 weights resident in registers, fp32 MFMA
};

struct Shape {
  uint32_t N, E, T, no, nh, na;
  uint32_t D;        // parameter count
  uint32_t m;        // hidden layers (W2, b2 below are the first of the m - 1 hidden-to-hidden layers, stride (nh + 1) nh)
  uint32_t ld;       // noise row stride (elements)
  uint32_t rows;     // noise rows
  // flat offsets of W1,b1,W2,b2,W3,b3
  uint32_t oW1, ob1, oW2, ob2, oW3, ob3;
};

}  // namespace es

struct es_ctx {
  es_config cfg;
  es::Shape shp;
  int rollout_kind;
  int mfma_variant;          // index of the instantiated register-resident kernel, or -1
  int reg_variant;           // index of the register-resident binary32 kernel, or -1
  size_t lds_bytes_wave;     // dynamic LDS of the wave/LDS rollout
  uint32_t upd_chunks;       // row chunks of the update reduction
  uint32_t regen_generation; // regenerated noise: the generation named by the last es_sample_population call
  bool regen_valid;          // ... and whether there has been one
  const float* obs_mean;     // frozen observation statistics (device pointers of the caller), or null
  const float* obs_inv_std;
  size_t workspace_bytes;
  int lds_limit;             // LDS bytes per workgroup on the device seen at es_create
  int num_cus;               // compute units of that device
  std::string kernel_name;
  std::string last_error;
};

namespace es {

constexpr uint32_t NOISE_LD_ALIGN = 512;   // elements
constexpr uint32_t STREAM_NOISE = 1u;
constexpr uint32_t STREAM_RESET = 2u;
constexpr uint32_t STREAM_TABLE = 3u;
constexpr uint32_t STREAM_OFFSET = 4u;

int fail(es_ctx* ctx, int code, const std::string& what);

// Noise storage modes of es_config.noise_dtype as the kernels see them: `mode` 0 / 1 = binary32 / bf16
// elements behind a pointer, 2 / 3 = regenerated; `offs` non-null = rows start at base + offs[row]
// (shared table) instead of base + row * ld.
struct NoiseView {
  const void* base;
  const uint32_t* offs;
  uint32_t mode;
};
inline NoiseView noise_view(const es_ctx* ctx, const void* noise) {
  NoiseView v;
  v.base = noise; v.offs = nullptr; v.mode = ctx->cfg.noise_dtype;
  if (ctx->cfg.noise_dtype >= 4) {
    v.mode = ctx->cfg.noise_dtype - 4;
    const size_t table_bytes = (size_t)ctx->cfg.noise_table_len * (v.mode == 1 ? 2 : 4);
    v.offs = reinterpret_cast<const uint32_t*>(static_cast<const char*>(noise) + table_bytes);
  }
  return v;
}
int check_launch(es_ctx* ctx, const char* what);

// stage launchers (each validates nothing: the API layer has done so)
int launch_sample(es_ctx* ctx, uint32_t gen, void* noise, hipStream_t st);
int launch_table(es_ctx* ctx, void* noise, hipStream_t st);
int launch_table_offsets(es_ctx* ctx, uint32_t gen, void* noise, hipStream_t st);
int launch_rank(es_ctx* ctx, const float* fit, int32_t* rank, float* shaped, hipStream_t st);
int launch_update(es_ctx* ctx, uint64_t step, const void* noise, const float* shaped, float* theta,
                  float* m, float* v, float* grad, void* ws, hipStream_t st);
int launch_rollout_wave(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise,
                        const float* A, const float* B, float* returns, int32_t* ep_len,
                        float* fitness, void* ws, hipStream_t st);
int launch_rollout_mfma(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise,
                        const float* A, const float* B, float* returns, int32_t* ep_len,
                        float* fitness, void* ws, hipStream_t st);
int launch_rollout_reg(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise,
                       const float* A, const float* B, float* returns, int32_t* ep_len,
                       float* fitness, void* ws, hipStream_t st);
int launch_rollout_mfma_f32(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise,
                            const float* A, const float* B, float* returns, int32_t* ep_len,
                            float* fitness, void* ws, hipStream_t st);
bool mfma_f32_fits(const es_config& cfg);         // binary32, 65..256 hidden units, one or two hidden layers, obs <= 64, act <= 16
const char* mfma_f32_variant_name(const es_config& cfg, uint32_t copies);   // copies = episodes evaluated per individual
int launch_fitness(es_ctx* ctx, const float* returns, float* fitness, hipStream_t st);
int reg_variant_for(const es_config& cfg);        // -1 when no one-wavefront register-resident kernel is built for the shape
std::string reg_variant_name(int variant, bool bf16);
int mfma_variant_for(const es_config& cfg);       // -1 when no register-resident kernel fits
const char* mfma_variant_name(int variant);
size_t wave_rollout_lds_bytes(const es_config& cfg);
uint32_t update_chunks(uint32_t rows, uint32_t ld, bool bf16);
uint32_t update_chunks_regen(uint32_t rows, uint32_t D);

}  // namespace es
