// es_rollout, register-resident binary32 variant for narrow policies (hidden width <= 64).
//
// Paper Sec. 3.2 / 5.2: population x environment-copy evaluation of a deterministic
// two-hidden-layer MLP policy, fitness = mean undiscounted return.  One wavefront runs one
// (individual, environment copy) episode; lane u owns hidden unit u.  The individual's
// perturbed weights (theta + sign*sigma*eps, fused into the load) and the environment
// matrices live in that lane's registers for all T steps:
//   W1 row u (obs values), a 16-column slice of four W2 rows (hid values) and of one W3 row,
//   A row u and B row u (lanes < obs).
// The obs-wide matrix-vector products are runs of v_readlane (the input element becomes a scalar
// operand) + v_fmac.  The hid x hid layer and the action layer instead broadcast their inputs within
// 16-lane rows by DPP (one instruction per multiply-add: the lane in row r, column c adds up the
// inputs 16 r .. 16 r + 15 for the output units c, c + 16, ...) and add the rows' partial sums with
// row swaps.  The reward norms are DPP wavefront reductions read back as scalars.  No LDS, no barriers.
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

// acc += w[j] * (lane 16*row + j of h), j = 0..15: sixteen multiply-adds whose first operand is broadcast
// within each 16-lane row by the DPP modifier, so no input element has to travel through a scalar register.
// The compiler's hazard checks do not look inside inline assembly: a vector ALU write of `h` must be two
// wait states away from the first DPP read, hence the leading s_nop.
template <int B, int N>
__device__ __forceinline__ float row_bcast_mac16(float acc, float h, const float (&w)[N]) {
  asm volatile(
      "s_nop 1\n\t"
      "v_fmac_f32_dpp %0, %1, %2 row_newbcast:0 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %3 row_newbcast:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %4 row_newbcast:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %5 row_newbcast:3 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %6 row_newbcast:4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %7 row_newbcast:5 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %8 row_newbcast:6 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %9 row_newbcast:7 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %10 row_newbcast:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %11 row_newbcast:9 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %12 row_newbcast:10 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %13 row_newbcast:11 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %14 row_newbcast:12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %15 row_newbcast:13 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %16 row_newbcast:14 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
      "v_fmac_f32_dpp %0, %1, %17 row_newbcast:15 row_mask:0xf bank_mask:0xf bound_ctrl:1"
      : "+v"(acc)
      : "v"(h), "v"(w[B + 0]), "v"(w[B + 1]), "v"(w[B + 2]), "v"(w[B + 3]), "v"(w[B + 4]), "v"(w[B + 5]), "v"(w[B + 6]),
        "v"(w[B + 7]), "v"(w[B + 8]), "v"(w[B + 9]), "v"(w[B + 10]), "v"(w[B + 11]), "v"(w[B + 12]), "v"(w[B + 13]),
        "v"(w[B + 14]), "v"(w[B + 15]));
  return acc;
}
// x + (the same register of the other 16-lane row of the pair / of the other half), via the row-swap instructions
__device__ __forceinline__ float swap16_add(float x, float y) {   // rows (0,1,2,3) <- x0+y... see the caller
  const auto p = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
  return __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
}
__device__ __forceinline__ float swap32_add(float x, float y) {
  const auto p = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
  return __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
}

template <int NO, int NH, int NA>
__global__ __launch_bounds__(64) void rollout_reg_kernel(const RegArgs a) {
  static_assert(NH <= 64 && NO <= 64 && NA <= 64, "one lane per unit");
  static_assert(NH == 32 || NH == 64, "the second layer is tiled over whole 16-lane rows");
  static_assert(NA <= 16, "one 16-lane row of action units");
  constexpr int NQ = NH / 16;      // 16-lane rows that hold hidden units
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
  float w1[NO], w2[NH], w3[16], ar[NO], br[NA];
  float b1 = 0.f, b2 = 0.f, b3 = 0.f;
#pragma unroll
  for (int k = 0; k < NO; ++k) w1[k] = hid ? param(oW1 + u * NO + k) : 0.f;
  // second layer: the lane in row r, column c multiplies the 16 inputs of ITS row (h1[16 r + j]) into partial sums of
  // the output units c, c + 16, ...; w2[16 q + j] = W2[c + 16 q][16 r + j]
  const int lr = u >> 4, lc = u & 15;
#pragma unroll
  for (int qq = 0; qq < NQ; ++qq) {
    const uint32_t d0 = oW2 + (uint32_t)(lc + 16 * qq) * NH + 16u * (uint32_t)lr;     // sixteen consecutive parameters
#pragma unroll
    for (int j = 0; j < 16; ++j) w2[16 * qq + j] = hid ? param(d0 + j) : 0.f;
  }
  // action layer, the same scheme: w3[j] = W3[c][16 r + j] (columns c >= act are zero)
#pragma unroll
  for (int j = 0; j < 16; ++j) w3[j] = (hid && lc < NA) ? param(oW3 + (uint32_t)lc * NH + 16u * (uint32_t)lr + j) : 0.f;
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
    // h2 = tanh(W2 h1 + b2): every lane accumulates over its own row's inputs (row-broadcast DPP multiply-adds),
    // then the rows' partial sums are added and moved to the lane of their unit by two row-swap stages
    const float p0 = row_bcast_mac16<0>(0.f, h1, w2), p1 = row_bcast_mac16<16>(0.f, h1, w2);
    float l2;
    if (NQ == 4) {
      const float p2 = row_bcast_mac16<NQ == 4 ? 32 : 0>(0.f, h1, w2), p3 = row_bcast_mac16<NQ == 4 ? 48 : 0>(0.f, h1, w2);
      l2 = swap16_add(swap32_add(p0, p2), swap32_add(p1, p3));
    } else {
      l2 = swap16_add(p0, p1);
    }
    l2 += b2;
    const float h2 = hid ? (a.hidden_relu ? fmaxf(l2, 0.f) : tanh_fast(l2)) : 0.f;
    // a = tanh(W3 h2 + b3): row-broadcast multiply-adds as above, the four rows' partial sums added by two row swaps;
    // lane c of every row then holds unit c's total, and one tanh serves all units
    float pv = row_bcast_mac16<0>(0.f, h2, w3);
    pv = swap16_add(pv, pv);
    pv = swap32_add(pv, pv);
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
