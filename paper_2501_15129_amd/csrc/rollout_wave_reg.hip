// es_rollout, register-resident binary32 variant for narrow policies (hidden width <= 64).
//
// Paper Sec. 3.2 / 5.2: population x environment-copy evaluation of a deterministic
// two-hidden-layer MLP policy, fitness = mean undiscounted return.  One wavefront runs one
// (individual, environment copy) episode; lane u owns hidden unit u.  The individual's
// perturbed weights (theta + sign*sigma*eps, fused into the load) and the environment
// matrices live in that lane's registers for all T steps:
//   W1 row u (obs values), W2 row u (hid), W3 column u (act), A row u and B row u (lanes < obs).
// A matrix-vector product is a run of v_readlane (the input element becomes a scalar operand)
// + v_fmac; the narrow action layer is act products per lane followed by DPP wavefront
// reductions whose result is read back as a scalar.  No LDS, no barriers.
// Bound: the dependent instruction chain of one step times T (the workloads that use this
// kernel have 32-256 episodes for 1024 SIMDs).
#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

struct RegArgs {
  const float* theta;
  const void* noise;
  const uint32_t* noise_offs;   // shared noise table: start of every row, else null
  const float* A;
  const float* B;
  const float* obs_mean;     // frozen observation statistics, or null
  const float* obs_inv;
  float* returns;
  int32_t* ep_len;
  uint32_t N, E, T, ld;
  uint32_t gen, k0, k1;
  uint32_t antithetic, out_tanh, noise_mode, hidden_relu;
  float sigma, done_thresh, act_cost;
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_zero(float v) {      // lanes without a source (or masked off) read 0
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, ROW_MASK == 0xF));
}
// Sum over the 64 lanes; the total is read from lane 63 and returned as a wavefront-uniform value.
__device__ __forceinline__ float wave_total(float v) {
  v += dpp_zero<0x111, 0xF>(v);      // row_shr:1
  v += dpp_zero<0x112, 0xF>(v);      // row_shr:2
  v += dpp_zero<0x114, 0xF>(v);      // row_shr:4
  v += dpp_zero<0x118, 0xF>(v);      // row_shr:8   -> lane 15 of every row holds the row total
  v += dpp_zero<0x142, 0xA>(v);      // row_bcast:15 into rows 1 and 3
  v += dpp_zero<0x143, 0xC>(v);      // row_bcast:31 into rows 2 and 3 -> lane 63 holds the total
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_total_max(float v) {   // for non-negative values
  v = fmaxf(v, dpp_zero<0x111, 0xF>(v));
  v = fmaxf(v, dpp_zero<0x112, 0xF>(v));
  v = fmaxf(v, dpp_zero<0x114, 0xF>(v));
  v = fmaxf(v, dpp_zero<0x118, 0xF>(v));
  v = fmaxf(v, dpp_zero<0x142, 0xA>(v));
  v = fmaxf(v, dpp_zero<0x143, 0xC>(v));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ float lane_value(float v, int lane) {   // lane is a compile-time constant after unrolling
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

template <int NO, int NH, int NA>
__global__ __launch_bounds__(64) void rollout_reg_kernel(const RegArgs a) {
  static_assert(NH <= 64 && NO <= 64 && NA <= 64, "one lane per unit");
  constexpr uint32_t oW1 = 0, ob1 = NH * NO, oW2 = ob1 + NH, ob2 = oW2 + NH * NH, oW3 = ob2 + NH, ob3 = oW3 + NA * NH;
  const int u = threadIdx.x;
  const uint32_t i = blockIdx.x / a.E, e = blockIdx.x % a.E;
  const uint32_t row = a.antithetic ? (i >> 1) : i;
  const float scale = (a.antithetic && (i & 1u)) ? -a.sigma : a.sigma;
  const bool hid = u < NH, obs = u < NO;

  const void* nbase = a.noise;      // shared table: this individual's row, addressed as row 0
  uint32_t nrow = row;
  if (a.noise_offs) { nbase = table_row_base(a.noise_mode, a.noise, a.noise_offs, row); nrow = 0u; }
  auto param = [&](uint32_t d) -> float {     // perturbed parameter d of individual i (binary32, one rounding)
    return __fmaf_rn(scale, noise_value(a.noise_mode, nbase, a.ld, nrow, d, a.gen, a.k0, a.k1), a.theta[d]);
  };

  // ---- this lane's weights ----
  float w1[NO], w2[NH], w3[NA], ar[NO], br[NA];
  float b1 = 0.f, b2 = 0.f, b3 = 0.f;
#pragma unroll
  for (int k = 0; k < NO; ++k) w1[k] = hid ? param(oW1 + u * NO + k) : 0.f;
#pragma unroll
  for (int k = 0; k < NH; ++k) w2[k] = hid ? param(oW2 + u * NH + k) : 0.f;
#pragma unroll
  for (int c = 0; c < NA; ++c) w3[c] = hid ? param(oW3 + c * NH + u) : 0.f;     // column u of W3
  if (hid) { b1 = param(ob1 + u); b2 = param(ob2 + u); }
  if (u < NA) b3 = param(ob3 + u);
#pragma unroll
  for (int k = 0; k < NO; ++k) ar[k] = obs ? a.A[u * NO + k] : 0.f;
#pragma unroll
  for (int c = 0; c < NA; ++c) br[c] = obs ? a.B[u * NA + c] : 0.f;

  // frozen observation statistics of lane k's state element (identity when none are set: (s - 0) * 1 = s exactly)
  const float mu = (obs && a.obs_mean) ? a.obs_mean[u] : 0.f;
  const float iv = (obs && a.obs_mean) ? a.obs_inv[u] : 1.f;
  float s = obs ? reset_value((uint32_t)u, e, a.gen, a.k0, a.k1) : 0.f;     // lane k holds s[k]
  float R = 0.f;
  int32_t len = 0;
  const float inv_no = 1.0f / (float)NO;

  for (uint32_t t = 0; t < a.T; ++t) {
    // h1 = tanh(W1 s + b1): two accumulation chains
    const float xp = (s - mu) * iv;      // the policy's input (paper App. B: fixed normalisation statistics)
    float acc0 = b1, acc1 = 0.f;
#pragma unroll
    for (int k = 0; k < NO; ++k) {
      const float sk = lane_value(xp, k);
      if (k & 1) acc1 = __fmaf_rn(w1[k], sk, acc1); else acc0 = __fmaf_rn(w1[k], sk, acc0);
    }
    const float h1 = hid ? (a.hidden_relu ? fmaxf(acc0 + acc1, 0.f) : tanh_fast(acc0 + acc1)) : 0.f;
    // h2 = tanh(W2 h1 + b2): four chains
    float c0 = b2, c1 = 0.f, c2 = 0.f, c3 = 0.f;
#pragma unroll
    for (int k = 0; k < NH; k += 4) {
      c0 = __fmaf_rn(w2[k], lane_value(h1, k), c0);
      if (k + 1 < NH) c1 = __fmaf_rn(w2[k + 1], lane_value(h1, k + 1), c1);
      if (k + 2 < NH) c2 = __fmaf_rn(w2[k + 2], lane_value(h1, k + 2), c2);
      if (k + 3 < NH) c3 = __fmaf_rn(w2[k + 3], lane_value(h1, k + 3), c3);
    }
    const float h2 = hid ? (a.hidden_relu ? fmaxf((c0 + c1) + (c2 + c3), 0.f) : tanh_fast((c0 + c1) + (c2 + c3))) : 0.f;
    // a = tanh(W3 h2 + b3): per-lane products, wavefront reductions, results as uniform scalars
    // the NA totals are gathered into lanes 0..NA-1 (lane c also holds b3[c]) so that one tanh serves all of them
    float pv = 0.f;
#pragma unroll
    for (int c = 0; c < NA; ++c) {
      const float tot = wave_total(w3[c] * h2);
      pv = (u == c) ? tot : pv;
    }
    pv = pv + b3;
    const float tv = a.out_tanh ? tanh_fast(pv) : pv;
    float act[NA];
    float aa = 0.f;
#pragma unroll
    for (int c = 0; c < NA; ++c) {
      act[c] = lane_value(tv, c);
      aa = __fmaf_rn(act[c], act[c], aa);
    }
    // reward from the pre-step state
    const float ss = wave_total(s * s);
    R += __fmaf_rn(-ss, inv_no, 1.0f) - a.act_cost * aa;
    len += 1;
    // s' = tanh(A s + B a)
    float e0 = 0.f, e1 = 0.f;
#pragma unroll
    for (int k = 0; k < NO; ++k) {
      const float sk = lane_value(s, k);
      if (k & 1) e1 = __fmaf_rn(ar[k], sk, e1); else e0 = __fmaf_rn(ar[k], sk, e0);
    }
#pragma unroll
    for (int c = 0; c < NA; ++c) e0 = __fmaf_rn(br[c], act[c], e0);
    s = obs ? tanh_fast(e0 + e1) : 0.f;
    const float mx = wave_total_max(fabsf(s));
    if (mx > a.done_thresh) break;       // uniform: mx is a scalar
  }
  if (u == 0) {
    a.returns[(size_t)i * a.E + e] = R;
    a.ep_len[(size_t)i * a.E + e] = len;
  }
}

struct RegShape { uint32_t no, nh, na; const char* name; };
static const RegShape kRegShapes[] = {
    {11, 32, 3, "rollout_wave_reg_f32<11,32,3>"},
    {17, 64, 6, "rollout_wave_reg_f32<17,64,6>"},
};

int reg_variant_for(const es_config& c) {
  if (c.dtype != 0 || (c.num_hidden != 0 && c.num_hidden != 2)) return -1;
  for (int v = 0; v < 2; ++v)
    if (c.obs_dim == kRegShapes[v].no && c.hid_dim == kRegShapes[v].nh && c.act_dim == kRegShapes[v].na) return v;
  return -1;
}
const char* reg_variant_name(int v) { return (v >= 0 && v < 2) ? kRegShapes[v].name : "none"; }

int launch_rollout_reg(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise, const float* A,
                       const float* B, float* returns, int32_t* ep_len, float* fitness, void* /*ws*/,
                       hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  RegArgs a;
  const NoiseView nv = noise_view(ctx, noise);
  a.theta = theta; a.noise = nv.base; a.noise_offs = nv.offs; a.A = A; a.B = B; a.obs_mean = ctx->obs_mean; a.obs_inv = ctx->obs_inv_std; a.returns = returns; a.ep_len = ep_len;
  a.N = s.N; a.E = s.E; a.T = s.T; a.ld = s.ld;
  a.gen = gen; a.k0 = (uint32_t)c.seed; a.k1 = (uint32_t)(c.seed >> 32);
  a.antithetic = c.antithetic; a.out_tanh = c.out_tanh; a.noise_mode = nv.mode; a.hidden_relu = c.hidden_act == 1;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  const dim3 grid(s.N * s.E), block(64);
  switch (ctx->reg_variant) {
    case 0: hipLaunchKernelGGL((rollout_reg_kernel<11, 32, 3>), grid, block, 0, st, a); break;
    case 1: hipLaunchKernelGGL((rollout_reg_kernel<17, 64, 6>), grid, block, 0, st, a); break;
    default: return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident binary32 variant for this shape");
  }
  int rc = check_launch(ctx, "es_rollout (register-resident f32)");
  if (rc != ES_OK) return rc;
  return launch_fitness(ctx, returns, fitness, st);
}

}  // namespace es
