// Host side of the C boundary: validation, context, dispatch.  See include/es.h for the
// contract of every entry point.
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "es_internal.hpp"

namespace es {

int fail(es_ctx* ctx, int code, const std::string& what) {
  if (ctx) ctx->last_error = what;
  return code;
}

int check_launch(es_ctx* ctx, const char* what) {
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string(what) + ": " + hipGetErrorString(err));
  return ES_OK;
}

static thread_local std::string g_create_error;

// Scratch of es_update_static: the binary64 partial rows that es_update keeps in the caller's workspace
// live here instead, in device memory that exists from the moment the code object is loaded until the
// process ends, once per GPU.  In host code the array's name is only a handle for hipGetSymbolAddress;
// the device address it yields (one per device) is what kernels and copies are given.
constexpr size_t STATIC_SCRATCH_BYTES = 32u << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];     // device address of `scratch` on each GPU, or null

// Address of this GPU's copy of `scratch` (looked up once per device, with that device current).
static int static_scratch(es_ctx* ctx, void** out) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) { (void)hipGetLastError(); return fail(ctx, ES_EHIP, std::string("es_update_static: hipGetDevice: ") + hipGetErrorString(err)); }
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return fail(ctx, ES_EUNSUPPORTED, "es_update_static: device ordinal beyond 63");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return fail(ctx, ES_EHIP, std::string("es_update_static: hipGetSymbolAddress: ") + hipGetErrorString(err));
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return ES_OK;
}

}  // namespace es

using namespace es;

extern "C" {

const char* es_strerror(int status) {
  switch (status) {
    case ES_OK: return "ES_OK";
    case ES_EINVAL: return "ES_EINVAL: invalid argument";
    case ES_EUNSUPPORTED: return "ES_EUNSUPPORTED: no kernel of this build supports the requested shape or mode";
    case ES_EHIP: return "ES_EHIP: HIP runtime error";
    default: return "unknown es_status";
  }
}

const char* es_last_error(const es_ctx* ctx) { return ctx ? ctx->last_error.c_str() : g_create_error.c_str(); }

int es_create(const es_config* cfg, es_ctx** out) {
  g_create_error.clear();
  if (!cfg || !out) { g_create_error = "es_create: null argument"; return ES_EINVAL; }
  *out = nullptr;
  const es_config& c = *cfg;
  auto bad = [&](const char* why) { g_create_error = std::string("es_create: ") + why; return (int)ES_EINVAL; };
  if (c.pop == 0 || c.envs_per_ind == 0 || c.horizon == 0) return bad("pop, envs_per_ind and horizon must be positive");
  if (c.obs_dim == 0 || c.hid_dim == 0 || c.act_dim == 0) return bad("layer widths must be positive");
  if (c.dtype > 1) return bad("dtype must be 0 or 1");
  if (c.noise_dtype > 5) return bad("noise_dtype must be 0..5");
  if (c.antithetic > 1 || c.out_tanh > 1) return bad("antithetic and out_tanh must be 0 or 1");
  if (c.antithetic && (c.pop & 1u)) return bad("pop must be even with mirrored sampling");
  if (c.hidden_act > 1) return bad("hidden_act must be 0 (tanh) or 1 (ReLU)");
  if (c.env_dtype > 1) return bad("env_dtype must be 0 or 1");
  if (c.algorithm > ES_VANILLA) return bad("algorithm must be ES_OPENES, ES_ARS or ES_VANILLA");
  if (c.algorithm == ES_ARS && (!c.antithetic || c.num_elites < 1 || c.num_elites > c.pop / 2))
    return bad("ES_ARS needs mirrored sampling and 1 <= num_elites <= pop / 2");
  if (c.algorithm == ES_VANILLA && (c.antithetic || c.num_elites < 1 || c.num_elites > c.pop))
    return bad("ES_VANILLA needs antithetic = 0 and 1 <= num_elites <= pop");
  if (c.algorithm != ES_OPENES && c.pop > 8192) return bad("ES_ARS and ES_VANILLA support pop <= 8192");
  if (!(c.sigma >= 0.0f) || !std::isfinite(c.sigma)) return bad("sigma must be finite and >= 0");
  if (std::isnan(c.done_thresh)) return bad("done_thresh is NaN");
  if (!std::isfinite(c.lr) || !std::isfinite(c.weight_decay) || !std::isfinite(c.act_cost)) return bad("non-finite hyper-parameter");
  if (!(c.beta1 >= 0.0f && c.beta1 < 1.0f) || !(c.beta2 >= 0.0f && c.beta2 < 1.0f)) return bad("betas must lie in [0, 1)");
  if (!(c.adam_eps > 0.0f)) return bad("adam_eps must be positive");
  const uint64_t o = c.obs_dim, h = c.hid_dim, a = c.act_dim;
  const uint64_t m = c.num_hidden ? c.num_hidden : 2;
  if (m > 64) return bad("num_hidden must be at most 64");
  const uint64_t D = (o + 1) * h + (m - 1) * (h + 1) * h + (h + 1) * a;
  const uint64_t episodes = (uint64_t)c.envs_per_ind * (c.episodes_per_env ? c.episodes_per_env : 1u);
  if (D > (1ull << 30) || (uint64_t)c.pop * episodes > (1ull << 30) || c.obs_dim > 65535 || c.hid_dim > 65535)
    return bad("shape too large");

  es_ctx* ctx = new (std::nothrow) es_ctx();
  if (!ctx) { g_create_error = "es_create: out of host memory"; return ES_EINVAL; }
  ctx->cfg = c;
  ctx->cfg.num_hidden = (uint32_t)m;
  Shape& s = ctx->shp;
  s.N = c.pop; s.E = (uint32_t)episodes; s.T = c.horizon; s.no = c.obs_dim; s.nh = c.hid_dim; s.na = c.act_dim;
  s.D = (uint32_t)D;
  s.ld = (s.D + NOISE_LD_ALIGN - 1) / NOISE_LD_ALIGN * NOISE_LD_ALIGN;
  s.rows = c.antithetic ? c.pop / 2 : c.pop;
  s.m = (uint32_t)m;
  s.oW1 = 0; s.ob1 = (uint32_t)(h * o); s.oW2 = s.ob1 + (uint32_t)h; s.ob2 = s.oW2 + (uint32_t)(h * h);
  s.oW3 = s.oW2 + (uint32_t)((m - 1) * (h + 1) * h); s.ob3 = s.oW3 + (uint32_t)(a * h);

  int dev = 0, lds = 65536, cus = 256;
  if (hipGetDevice(&dev) == hipSuccess) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0) lds = v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    void* scratch_here = nullptr;
    (void)static_scratch(nullptr, &scratch_here);   // resolve this GPU's scratch of es_update_static now, outside any capture
  } else {
    (void)hipGetLastError();   // no device here (host-only checks): keep the conservative default
  }
  ctx->lds_limit = lds;
  ctx->num_cus = cus;
  ctx->lds_bytes_wave = wave_rollout_lds_bytes(c);
  ctx->mfma_variant = mfma_variant_for(c);
  ctx->reg_variant = reg_variant_for(c);
  if (ctx->reg_variant >= 0) {
    ctx->rollout_kind = ROLLOUT_WAVE_REG;
    ctx->kernel_name = reg_variant_name(ctx->reg_variant, c.dtype == 1);
  } else if (mfma_f32_fits(c)) {
    ctx->rollout_kind = ROLLOUT_MFMA_F32;
    ctx->kernel_name = mfma_f32_variant_name(c, ctx->shp.E);
  } else if (ctx->mfma_variant >= 0) {
    ctx->rollout_kind = ROLLOUT_MFMA_REG;
    ctx->kernel_name = mfma_variant_name(ctx->mfma_variant);
    if (m != 2) ctx->kernel_name += ",depth" + std::to_string(m);
  } else {
    ctx->rollout_kind = ROLLOUT_WAVE_LDS;
    ctx->kernel_name = c.dtype == 1 ? "rollout_wave_lds_bf16" : "rollout_wave_lds_f32";
  }
  if (c.noise_dtype >= 4 && (c.noise_table_len % 8 != 0 || c.noise_table_len < s.ld || c.noise_table_len >= (1ull << 32))) {
    delete ctx;
    return bad("noise_table_len must be a multiple of 8, at least the padded row length, and below 2^32");
  }
  ctx->obs_mean = nullptr;
  ctx->obs_inv_std = nullptr;
  ctx->regen_generation = 0;
  ctx->regen_valid = false;
  const bool regen = c.noise_dtype == 2 || c.noise_dtype == 3, bf16_noise = c.noise_dtype == 1 || c.noise_dtype == 5;
  ctx->upd_chunks = regen ? update_chunks_regen(s.rows, s.D) : update_chunks(s.rows, s.ld, bf16_noise);
  ctx->workspace_bytes = std::max<size_t>(256, (size_t)ctx->upd_chunks * s.ld * sizeof(double));
  *out = ctx;
  return ES_OK;
}

int es_destroy(es_ctx* ctx) {
  delete ctx;
  return ES_OK;
}

size_t es_param_count(const es_ctx* ctx) { return ctx ? ctx->shp.D : 0; }
size_t es_noise_rows(const es_ctx* ctx) { return ctx ? ctx->shp.rows : 0; }
size_t es_noise_ld(const es_ctx* ctx) { return ctx ? ctx->shp.ld : 0; }
size_t es_noise_bytes(const es_ctx* ctx) {
  if (!ctx) return 0;
  const uint32_t nd = ctx->cfg.noise_dtype;
  if (nd == 2 || nd == 3) return 0;                       // regenerated noise is never stored
  if (nd >= 4) return (size_t)ctx->cfg.noise_table_len * (nd == 5 ? 2 : 4) + (size_t)ctx->shp.rows * 4;   // table | row offsets
  return (size_t)ctx->shp.rows * ctx->shp.ld * (nd == 1 ? 2 : 4);
}
size_t es_workspace_bytes(const es_ctx* ctx) { return ctx ? ctx->workspace_bytes : 0; }
const char* es_rollout_kernel(const es_ctx* ctx) { return ctx ? ctx->kernel_name.c_str() : ""; }
const char* es_update_kernel(const es_ctx* ctx) {
  if (!ctx) return "";
  if (ctx->cfg.noise_dtype == 2 || ctx->cfg.noise_dtype == 3) return "grad_regen_kernel+adam_kernel";
  return ctx->upd_chunks == 1 ? "update_single_pass_kernel" : "grad_partial_kernel+adam_kernel";
}

// the kernels read parameters, noise rows and environment matrices with 16-byte vector loads
static bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int es_set_obs_norm(es_ctx* ctx, const float* mean_d, const float* inv_std_d) {
  if (!ctx) return ES_EINVAL;
  if ((mean_d == nullptr) != (inv_std_d == nullptr))
    return fail(ctx, ES_EINVAL, "es_set_obs_norm: mean_d and inv_std_d must both be set or both be null");
  ctx->obs_mean = mean_d;
  ctx->obs_inv_std = inv_std_d;
  return ES_OK;
}

int es_build_noise_table(es_ctx* ctx, void* noise_d, void* stream) {
  if (!ctx) return ES_EINVAL;
  if (ctx->cfg.noise_dtype < 4) return fail(ctx, ES_EINVAL, "es_build_noise_table: this context does not use a noise table");
  if (!noise_d) return fail(ctx, ES_EINVAL, "es_build_noise_table: noise_d is null");
  if (misaligned16(noise_d)) return fail(ctx, ES_EINVAL, "es_build_noise_table: noise_d must be 16-byte aligned");
  return launch_table(ctx, noise_d, static_cast<hipStream_t>(stream));
}

// Argument checks of the four stages, shared by the stage calls and es_generation (which must
// reject a bad argument of a later stage before it has enqueued an earlier one).
static bool regenerated(const es_ctx* ctx) { return ctx->cfg.noise_dtype == 2 || ctx->cfg.noise_dtype == 3; }

static int check_sample(es_ctx* ctx, uint64_t generation, const void* noise_d) {
  if (generation >> 32) return fail(ctx, ES_EINVAL, "es_sample_population: generation must be < 2^32");
  if (!regenerated(ctx) && !noise_d) return fail(ctx, ES_EINVAL, "es_sample_population: noise_d is null");
  if (misaligned16(noise_d)) return fail(ctx, ES_EINVAL, "es_sample_population: noise_d must be 16-byte aligned");
  return ES_OK;
}

static int check_rollout(es_ctx* ctx, uint64_t generation, const float* theta_d, const void* noise_d, const float* A_d,
                         const float* B_d, const float* returns_d, const int32_t* ep_len_d, const float* fitness_d,
                         const void* workspace_d) {
  if (!theta_d || !A_d || !B_d || !returns_d || !ep_len_d || !fitness_d || !workspace_d || (!noise_d && !regenerated(ctx)))
    return fail(ctx, ES_EINVAL, "es_rollout: null device pointer");
  if (generation >> 32) return fail(ctx, ES_EINVAL, "es_rollout: generation must be < 2^32");
  if (misaligned16(theta_d) || misaligned16(noise_d) || misaligned16(A_d) || misaligned16(B_d) || misaligned16(workspace_d))
    return fail(ctx, ES_EINVAL, "es_rollout: theta_d, noise_d, A_d, B_d and workspace_d must be 16-byte aligned");
  if (ctx->rollout_kind == ROLLOUT_WAVE_LDS && ctx->lds_bytes_wave > (size_t)ctx->lds_limit)
    return fail(ctx, ES_EUNSUPPORTED, "es_rollout: perturbed parameters of one individual (" +
                                          std::to_string(ctx->lds_bytes_wave) + " B) exceed the LDS of a workgroup (" +
                                          std::to_string(ctx->lds_limit) + " B) and no register-resident kernel is built for this shape");
  return ES_OK;
}

static int check_rank(es_ctx* ctx, const float* fitness_d, const int32_t* rank_d, const float* shaped_d) {
  if (!fitness_d || !rank_d || !shaped_d) return fail(ctx, ES_EINVAL, "es_rank: null device pointer");
  return ES_OK;
}

static int check_update(es_ctx* ctx, uint64_t adam_step, const void* noise_d, const float* shaped_d, const float* theta_d,
                        const float* m_d, const float* v_d, const void* workspace_d, bool sampled) {
  if (!shaped_d || !theta_d || !workspace_d || (!noise_d && !regenerated(ctx)) ||
      ((!m_d || !v_d) && ctx->cfg.algorithm == ES_OPENES))
    return fail(ctx, ES_EINVAL, "es_update: null device pointer");
  if (misaligned16(noise_d) || misaligned16(workspace_d))
    return fail(ctx, ES_EINVAL, "es_update: noise_d and workspace_d must be 16-byte aligned");
  if (regenerated(ctx) && !sampled)
    return fail(ctx, ES_EINVAL, "es_update: with regenerated noise, es_sample_population must name the generation first");
  if (adam_step < 1 && ctx->cfg.algorithm == ES_OPENES) return fail(ctx, ES_EINVAL, "es_update: adam_step is 1-based");
  if (!(ctx->cfg.sigma > 0.0f)) return fail(ctx, ES_EINVAL, "es_update: sigma must be > 0");
  return ES_OK;
}

static int enqueue_sample(es_ctx* ctx, uint32_t generation, void* noise_d, hipStream_t st) {
  if (regenerated(ctx)) {            // nothing to store: remember which generation es_update regenerates
    ctx->regen_generation = generation;
    ctx->regen_valid = true;
    return ES_OK;
  }
  if (ctx->cfg.noise_dtype >= 4) return launch_table_offsets(ctx, generation, noise_d, st);
  return launch_sample(ctx, generation, noise_d, st);
}

static int enqueue_rollout(es_ctx* ctx, uint32_t generation, const float* theta_d, const void* noise_d, const float* A_d,
                           const float* B_d, float* returns_d, int32_t* ep_len_d, float* fitness_d, void* workspace_d,
                           hipStream_t st) {
  if (ctx->rollout_kind == ROLLOUT_WAVE_REG)
    return launch_rollout_reg(ctx, generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d, st);
  if (ctx->rollout_kind == ROLLOUT_MFMA_F32)
    return launch_rollout_mfma_f32(ctx, generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d, st);
  if (ctx->rollout_kind == ROLLOUT_MFMA_REG)
    return launch_rollout_mfma(ctx, generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d, st);
  return launch_rollout_wave(ctx, generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d, st);
}

int es_sample_population(es_ctx* ctx, uint64_t generation, void* noise_d, void* stream) {
  if (!ctx) return ES_EINVAL;
  if (int rc = check_sample(ctx, generation, noise_d)) return rc;
  return enqueue_sample(ctx, (uint32_t)generation, noise_d, static_cast<hipStream_t>(stream));
}

int es_rollout(es_ctx* ctx, uint64_t generation, const float* theta_d, const void* noise_d, const float* A_d,
               const float* B_d, float* returns_d, int32_t* ep_len_d, float* fitness_d, void* workspace_d,
               void* stream) {
  if (!ctx) return ES_EINVAL;
  if (int rc = check_rollout(ctx, generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d)) return rc;
  return enqueue_rollout(ctx, (uint32_t)generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d,
                         static_cast<hipStream_t>(stream));
}

int es_rank(es_ctx* ctx, const float* fitness_d, int32_t* rank_d, float* shaped_d, void* stream) {
  if (!ctx) return ES_EINVAL;
  if (int rc = check_rank(ctx, fitness_d, rank_d, shaped_d)) return rc;
  return launch_rank(ctx, fitness_d, rank_d, shaped_d, static_cast<hipStream_t>(stream));
}

int es_update(es_ctx* ctx, uint64_t adam_step, const void* noise_d, const float* shaped_d, float* theta_d,
              float* m_d, float* v_d, float* grad_d, void* workspace_d, void* stream) {
  if (!ctx) return ES_EINVAL;
  if (int rc = check_update(ctx, adam_step, noise_d, shaped_d, theta_d, m_d, v_d, workspace_d, ctx->regen_valid)) return rc;
  return launch_update(ctx, adam_step, noise_d, shaped_d, theta_d, m_d, v_d, grad_d, workspace_d,
                       static_cast<hipStream_t>(stream));
}

size_t es_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int es_update_static(es_ctx* ctx, uint64_t adam_step, const void* noise_d, const float* shaped_d, float* theta_d,
                     float* m_d, float* v_d, float* grad_d, void* stream) {
  if (!ctx) return ES_EINVAL;
  if (ctx->workspace_bytes > STATIC_SCRATCH_BYTES)
    return fail(ctx, ES_EUNSUPPORTED, "es_update_static: this shape needs " + std::to_string(ctx->workspace_bytes) +
                                          " B of partial sums, more than the built-in scratch of " +
                                          std::to_string(STATIC_SCRATCH_BYTES) + " B; use es_update with a workspace");
  void* ws = nullptr;
  if (int rc = static_scratch(ctx, &ws)) return rc;
  if (int rc = check_update(ctx, adam_step, noise_d, shaped_d, theta_d, m_d, v_d, ws, ctx->regen_valid)) return rc;
  // every partial row the parameter step reads is written by the reduction kernel of the same call:
  // nothing in the scratch has to start at zero
  return launch_update(ctx, adam_step, noise_d, shaped_d, theta_d, m_d, v_d, grad_d, ws, static_cast<hipStream_t>(stream));
}

int es_generation(es_ctx* ctx, uint64_t generation, uint64_t adam_step, void* noise_d, const float* A_d, const float* B_d,
                  float* theta_d, float* m_d, float* v_d, float* returns_d, int32_t* ep_len_d, float* fitness_d,
                  int32_t* rank_d, float* shaped_d, float* grad_d, void* workspace_d, void* stream) {
  if (!ctx) return ES_EINVAL;
  if (int rc = check_sample(ctx, generation, noise_d)) return rc;
  if (int rc = check_rollout(ctx, generation, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d)) return rc;
  if (int rc = check_rank(ctx, fitness_d, rank_d, shaped_d)) return rc;
  if (int rc = check_update(ctx, adam_step, noise_d, shaped_d, theta_d, m_d, v_d, workspace_d, true)) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint32_t gen = (uint32_t)generation;
  if (int rc = enqueue_sample(ctx, gen, noise_d, st)) return rc;
  if (int rc = enqueue_rollout(ctx, gen, theta_d, noise_d, A_d, B_d, returns_d, ep_len_d, fitness_d, workspace_d, st)) return rc;
  if (int rc = launch_rank(ctx, fitness_d, rank_d, shaped_d, st)) return rc;
  return launch_update(ctx, adam_step, noise_d, shaped_d, theta_d, m_d, v_d, grad_d, workspace_d, st);
}

}  // extern "C"
