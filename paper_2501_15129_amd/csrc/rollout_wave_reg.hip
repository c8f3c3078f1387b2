// es_rollout, register-resident kernel for narrow policies (obs, hidden <= 64, act <= 16, two hidden layers), binary32
// or bf16 operands.
//
// Paper Sec. 3.2 / 5.2: population x environment-copy evaluation of a deterministic
// two-hidden-layer MLP policy, fitness = mean undiscounted return.  One wavefront runs one
// (individual, environment copy) episode.  Lane u owns hidden unit u (with at most 16 hidden units every
// 16-lane row owns all of them), and the state vector is spread over the four 16-lane rows of the
// wavefront (element k in row k % 4, column k / 4).  The individual's perturbed weights
// (theta + sign*sigma*eps) pass through LDS once, in coalesced order, and then live in registers for all
// T steps, as do the environment matrices.
// Every matrix-vector product broadcasts its inputs within the 16-lane rows by DPP, fused into the
// multiply-add (v_fmac_f32_dpp ... row_newbcast:j, one instruction per multiply-add, no scalar hop):
// the lane in row r, column c adds up the inputs that live in ITS row into partial sums for the outputs
// that belong to ITS column (hidden units c, c + 16, ...; state elements 4 c .. 4 c + 3), and two
// row-swap stages (v_permlane32_swap, v_permlane16_swap + add) add the four rows' partial sums and
// leave each output's total in the lane that owns it.  A step is one straight-line block: no LDS, no
// barriers, no masks (lanes without a unit have zero weights, and tanh and ReLU map 0 to 0), the return is
// accumulated per lane and reduced after the last step, termination is one compare whose mask is the
// branch condition.
// The run lengths (inputs per row, rows of hidden units, action width) are compile-time: exact for the
// benchmark shapes 11-32-3 and 17-64-6, whose activations and observation statistics are compile-time
// variants too, and rounded up to a few classes for every other shape (padding has zero weights), where
// the activations are chosen by branch-free selects.
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
  uint32_t N, E, T, ld, D;
  uint32_t no, nh, na;
  uint32_t oW1, ob1, oW2, ob2, oW3, ob3;
  uint32_t gen, k0, k1;
  uint32_t antithetic, noise_mode, hidden_relu, out_tanh;
  uint32_t env_f32;          // bf16 operands: keep the environment's products binary32
  float sigma, done_thresh, act_cost;
};

#include "dpp_runs.inc"

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_zero(float v) {      // lanes without a source (or masked off) read 0
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, ROW_MASK == 0xF));
}
// x + y after a row swap: permlane16_swap exchanges the odd rows of x with the even rows of y, permlane32_swap the
// upper two rows of x with the lower two of y
__device__ __forceinline__ float swap16_add(float x, float y) {
  const auto p = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
  return __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
}
__device__ __forceinline__ float swap32_add(float x, float y) {
  const auto p = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
  return __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
}
// out[row q] = sum over the four rows of x_q: two row-swap stages
__device__ __forceinline__ float rows_transpose_add(float x0, float x1, float x2, float x3) {
  return swap16_add(swap32_add(x0, x2), swap32_add(x1, x3));
}
// the same for two registers whose sums go to rows 0 and 1 (and again to rows 2 and 3)
__device__ __forceinline__ float rows_transpose_add(float x0, float x1) {
  const float t = swap16_add(x0, x1);
  return swap32_add(t, t);
}
// the sum over the four rows, in every row
__device__ __forceinline__ float rows_add(float x) {
  const float t = swap16_add(x, x);
  return swap32_add(t, t);
}
// sum over the lanes of each 16-lane row, result in lane 15 of the row (lanes without a source read 0)
__device__ __forceinline__ float row_total(float v) {
  v += dpp_zero<0x111, 0xF>(v);
  v += dpp_zero<0x112, 0xF>(v);
  v += dpp_zero<0x114, 0xF>(v);
  return v + dpp_zero<0x118, 0xF>(v);
}

// CJ: state elements per row (ceil(obs / 4), or its class); NQ: 16-lane rows of hidden units (1, 2, 4); NAR: action
// run length (act, or its class).  MODE 0..7 = ReLU (4) | tanh on the action layer (2) | observation statistics (1)
// fixed at compile time; MODE < 0: read from the arguments and applied by selects.  BF16: every operand of a product
// (weights, biases, environment matrices, state, activations, action) is rounded to bf16; sums, tanh, reward binary32.
template <int CJ, int NQ, int NAR, int MODE, bool BF16>
__global__ __launch_bounds__(64) void rollout_reg_kernel(const RegArgs a) {
  static_assert(NQ == 1 || NQ == 2 || NQ == 4, "rows of hidden units");
  constexpr bool FIXED = MODE >= 0;
  constexpr bool RELU = FIXED && (MODE & 4), OUT_TANH = FIXED && (MODE & 2), NORM = !FIXED || (MODE & 1);
  extern __shared__ float sp[];      // the individual's perturbed parameters, once
  const int u = threadIdx.x;
  const uint32_t i = blockIdx.x / a.E, e = blockIdx.x % a.E;
  const uint32_t row = a.antithetic ? (i >> 1) : i;
  const float scale = (a.antithetic && (i & 1u)) ? -a.sigma : a.sigma;
  const int no = (int)a.no, nh = (int)a.nh, na = (int)a.na;
  const int lr = u >> 4, lc = u & 15;
  const int ks = 4 * lc + lr;                    // the state element of this lane
  const bool sval = lc < CJ && ks < no;
  const int hu = NQ == 1 ? lc : u;               // the hidden unit of this lane
  const bool hid = hu < nh;
  auto opnd = [](float v) { return BF16 ? bf16_round(v) : v; };      // a value as an operand of a product
  // ... of one of the ENVIRONMENT's products: rounded like the policy's unless the environment stays binary32 (a select,
  // not a branch: the flag is read into a vector register the compiler cannot prove uniform)
  uint32_t envf_l = a.env_f32;
  if (BF16) asm volatile("" : "+v"(envf_l));
  auto opnd_env = [&](float v) { return BF16 ? (envf_l ? v : bf16_round(v)) : v; };

  // ---- perturbed parameters -> LDS (coalesced, binary32, one rounding each) ----
  {
    const void* nbase = a.noise;      // shared table: this individual's row, addressed as row 0
    uint32_t nrow = row;
    if (a.noise_offs) { nbase = table_row_base(a.noise_mode, a.noise, a.noise_offs, row); nrow = 0u; }
    if (a.noise_mode >= 2u) {       // regenerated noise: one counter block gives four consecutive parameters
      for (uint32_t d0 = 4u * (uint32_t)u; d0 < a.D; d0 += 256u) {
        float z[4];
        noise_regen4(row, d0, a.gen, a.k0, a.k1, a.noise_mode == 3u, z);
#pragma unroll
        for (uint32_t k = 0; k < 4u; ++k)
          if (d0 + k < a.D) sp[d0 + k] = opnd(__fmaf_rn(scale, z[k], a.theta[d0 + k]));
      }
    } else {
      for (uint32_t d = (uint32_t)u; d < a.D; d += 64u)
        sp[d] = opnd(__fmaf_rn(scale, noise_value(a.noise_mode, nbase, a.ld, nrow, d, a.gen, a.k0, a.k1), a.theta[d]));
    }
    __syncthreads();
  }

  // ---- this lane's weights ----
  // first layer: partial sums of the units lc, lc + 16, ... over the inputs of row lr: w1[CJ q + j] = W1[lc + 16 q][4 j + lr]
  // second layer and action layer: the same over the 16 hidden units of row lr: w2[16 q + j] = W2[lc + 16 q][16 lr + j],
  //   w3[j] = W3[lc][16 lr + j] (with one row of hidden units every row holds all of them: input j)
  // environment: partial sums of the four state elements of column lc: ar[CJ r + j] = A[4 lc + r][4 j + lr];
  //   action term of this lane's own element: br[c] = B[ks][c]
  float w1[NQ * CJ], w2[NQ * 16], w3[16], ar[4 * CJ], br[NAR];
#pragma unroll
  for (int qq = 0; qq < NQ; ++qq)
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
      const int unit = lc + 16 * qq, k = 4 * j + lr;
      w1[CJ * qq + j] = (unit < nh && k < no) ? sp[a.oW1 + unit * no + k] : 0.f;
    }
#pragma unroll
  for (int qq = 0; qq < NQ; ++qq)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int unit = lc + 16 * qq, k = (NQ == 1 ? 0 : 16 * lr) + j;
      w2[16 * qq + j] = (unit < nh && k < nh) ? sp[a.oW2 + unit * nh + k] : 0.f;
    }
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int k = (NQ == 1 ? 0 : 16 * lr) + j;
    w3[j] = (lc < na && k < nh) ? sp[a.oW3 + lc * nh + k] : 0.f;
  }
  const float b1 = hid ? sp[a.ob1 + hu] : 0.f, b2 = hid ? sp[a.ob2 + hu] : 0.f;
  const float b3 = lc < na ? sp[a.ob3 + lc] : 0.f;            // in every row: the action vector is kept once per row
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
      const int el = 4 * lc + r, k = 4 * j + lr;
      ar[CJ * r + j] = (lc < CJ && el < no && k < no) ? opnd_env(a.A[el * no + k]) : 0.f;
    }
#pragma unroll
  for (int c = 0; c < NAR; ++c) br[c] = (sval && c < na) ? opnd_env(a.B[ks * na + c]) : 0.f;

  // frozen observation statistics of this lane's state element (identity when none are set: (s - 0) * 1 = s exactly)
  const bool stats = a.obs_mean != nullptr;
  const float mu = (NORM && stats && sval) ? a.obs_mean[ks] : 0.f;
  const float iv = (NORM && stats && sval) ? a.obs_inv[ks] : 1.f;
  // run-time activation choices as per-lane values the compiler cannot prove uniform: selects, not branches
  uint32_t relu_l = a.hidden_relu, otanh_l = a.out_tanh;
  if (!FIXED) asm volatile("" : "+v"(relu_l), "+v"(otanh_l));
  auto hidden = [&](float l) {
    if (FIXED) return RELU ? fmaxf(l, 0.f) : tanh_fast(l);
    const float t = tanh_fast(l);
    return relu_l ? fmaxf(l, 0.f) : t;
  };
  float s = sval ? reset_value((uint32_t)ks, e, a.gen, a.k0, a.k1) : 0.f;
  float R = 0.f;                      // per-lane share of the return
  int32_t len = 0;
  const float inv_no = 1.0f / (float)no, quarter_cost = 0.25f * a.act_cost;

  for (uint32_t t = 0; t < a.T; ++t) {
    // h1 = act(W1 s + b1)
    const float xp = opnd(NORM ? (s - mu) * iv : s);      // the policy's input (paper App. B: fixed normalisation statistics)
    float p[NQ];
    row_bcast_dot<NQ, CJ>(p, xp, w1);
    float l1;
    if constexpr (NQ == 4) l1 = rows_transpose_add(p[0], p[1], p[2], p[3]);
    else if constexpr (NQ == 2) l1 = rows_transpose_add(p[0], p[1]);
    else l1 = rows_add(p[0]);
    const float h1 = opnd(hidden(l1 + b1));
    // h2 = act(W2 h1 + b2)
    row_bcast_dot<NQ, 16>(p, h1, w2);
    float l2;
    if constexpr (NQ == 4) l2 = rows_transpose_add(p[0], p[1], p[2], p[3]);
    else if constexpr (NQ == 2) l2 = swap16_add(p[0], p[1]);      // the units' own rows 0 and 1 hold all of their inputs
    else l2 = p[0];                                               // every row holds all inputs
    const float h2 = opnd(hidden(l2 + b2));
    // a = tanh(W3 h2 + b3): column c of every row ends up with unit c's total, one tanh serves all units
    float pa[1];
    row_bcast_dot<1, 16>(pa, h2, w3);
    float pv = NQ == 1 ? pa[0] : rows_add(pa[0]);
    pv = pv + b3;
    float tv;
    if (FIXED) tv = OUT_TANH ? tanh_fast(pv) : pv;      // columns >= act: weights and bias are zero
    else { const float tt = tanh_fast(pv); tv = otanh_l ? tt : pv; }
    // reward from the pre-step state, 1 - |s|^2 / obs - cost |a|^2: a sum over all 64 lanes (the action vector is held
    // once per row, hence the quarter)
    R += __fmaf_rn(-inv_no * s, s, -quarter_cost * (tv * tv));      // this lane's share; the lanes are added after the last step
    len += 1;
    // s' = tanh(A s + B a): partial sums of the four elements of this column over the inputs of this row, rows added
    // and moved to their element's lane; the action term straight from the row's action vector
    float ev[4];
    row_bcast_dot<4, CJ>(ev, opnd_env(s), ar);
    float pre = rows_transpose_add(ev[0], ev[1], ev[2], ev[3]);
    pre = row_bcast_mac<NAR>(pre, opnd_env(tv), br);
    s = tanh_fast(pre);                                  // lanes without a state element: zero weights, tanh(0) = 0
    if (__ballot(fabsf(s) > a.done_thresh) != 0ull) break;       // max |s| > threshold: some lane exceeds it
  }
  R = (float)len + row_total(rows_add(R));      // ends in lane 15
  if (u == 15) {
    a.returns[(size_t)i * a.E + e] = R;
    a.ep_len[(size_t)i * a.E + e] = len;
  }
}

// ---- variants: two exact shapes, and classes for everything else ----
constexpr int REG_EXACT = 2;
struct RegExact { uint32_t no, nh, na; };
static const RegExact kRegExact[REG_EXACT] = {{11, 32, 3}, {17, 64, 6}};
// class variant index = REG_EXACT + 9 * (obs class) + 3 * (hidden class) + (act class)
static int class_of(uint32_t v, uint32_t a, uint32_t b) { return v <= a ? 0 : (v <= b ? 1 : 2); }

int reg_variant_for(const es_config& c) {
  if (c.dtype > 1 || (c.num_hidden != 0 && c.num_hidden != 2)) return -1;
  if (c.obs_dim > 64 || c.hid_dim > 64 || c.act_dim > 16) return -1;
  for (int v = 0; v < REG_EXACT && c.dtype == 0; ++v)
    if (c.obs_dim == kRegExact[v].no && c.hid_dim == kRegExact[v].nh && c.act_dim == kRegExact[v].na) return v;
  return REG_EXACT + 9 * class_of(c.obs_dim, 16, 32) + 3 * class_of(c.hid_dim, 16, 32) + class_of(c.act_dim, 4, 8);
}

std::string reg_variant_name(int v, bool bf16) {
  if (v < 0) return "none";
  if (v < REG_EXACT)
    return "rollout_wave_reg_f32<" + std::to_string(kRegExact[v].no) + "," + std::to_string(kRegExact[v].nh) + "," +
           std::to_string(kRegExact[v].na) + ">";
  v -= REG_EXACT;
  static const char* obs[] = {"16", "32", "64"}, *hid[] = {"16", "32", "64"}, *act[] = {"4", "8", "16"};
  return std::string(bf16 ? "rollout_wave_reg_bf16<obs<=" : "rollout_wave_reg_f32<obs<=") + obs[v / 9] + ",hid<=" + hid[(v / 3) % 3] + ",act<=" + act[v % 3] + ">";
}

template <int CJ, int NQ, int NAR>
static void launch_fixed(int mode, dim3 grid, size_t lds, hipStream_t st, const RegArgs& a) {
  auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, dim3(64), lds, st, a); };
  switch (mode) {
    case 0: go(rollout_reg_kernel<CJ, NQ, NAR, 0, false>); break;
    case 1: go(rollout_reg_kernel<CJ, NQ, NAR, 1, false>); break;
    case 2: go(rollout_reg_kernel<CJ, NQ, NAR, 2, false>); break;
    case 3: go(rollout_reg_kernel<CJ, NQ, NAR, 3, false>); break;
    case 4: go(rollout_reg_kernel<CJ, NQ, NAR, 4, false>); break;
    case 5: go(rollout_reg_kernel<CJ, NQ, NAR, 5, false>); break;
    case 6: go(rollout_reg_kernel<CJ, NQ, NAR, 6, false>); break;
    default: go(rollout_reg_kernel<CJ, NQ, NAR, 7, false>); break;
  }
}
template <int CJ, int NQ, bool BF16>
static void launch_class_act(int act_class, dim3 grid, size_t lds, hipStream_t st, const RegArgs& a) {
  auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, dim3(64), lds, st, a); };
  if (act_class == 0) go(rollout_reg_kernel<CJ, NQ, 4, -1, BF16>);
  else if (act_class == 1) go(rollout_reg_kernel<CJ, NQ, 8, -1, BF16>);
  else go(rollout_reg_kernel<CJ, NQ, 16, -1, BF16>);
}
template <int CJ, bool BF16>
static void launch_class_hid(int hid_class, int act_class, dim3 grid, size_t lds, hipStream_t st, const RegArgs& a) {
  if (hid_class == 0) launch_class_act<CJ, 1, BF16>(act_class, grid, lds, st, a);
  else if (hid_class == 1) launch_class_act<CJ, 2, BF16>(act_class, grid, lds, st, a);
  else launch_class_act<CJ, 4, BF16>(act_class, grid, lds, st, a);
}
template <bool BF16>
static void launch_class(int obs_class, int hid_class, int act_class, dim3 grid, size_t lds, hipStream_t st, const RegArgs& a) {
  if (obs_class == 0) launch_class_hid<4, BF16>(hid_class, act_class, grid, lds, st, a);
  else if (obs_class == 1) launch_class_hid<8, BF16>(hid_class, act_class, grid, lds, st, a);
  else launch_class_hid<16, BF16>(hid_class, act_class, grid, lds, st, a);
}

int launch_rollout_reg(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise, const float* A,
                       const float* B, float* returns, int32_t* ep_len, float* fitness, void* /*ws*/,
                       hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  RegArgs a;
  const NoiseView nv = noise_view(ctx, noise);
  a.theta = theta; a.noise = nv.base; a.noise_offs = nv.offs; a.A = A; a.B = B; a.obs_mean = ctx->obs_mean; a.obs_inv = ctx->obs_inv_std; a.returns = returns; a.ep_len = ep_len;
  a.N = s.N; a.E = s.E; a.T = s.T; a.ld = s.ld; a.D = s.D;
  a.no = s.no; a.nh = s.nh; a.na = s.na;
  a.oW1 = s.oW1; a.ob1 = s.ob1; a.oW2 = s.oW2; a.ob2 = s.ob2; a.oW3 = s.oW3; a.ob3 = s.ob3;
  a.gen = gen; a.k0 = (uint32_t)c.seed; a.k1 = (uint32_t)(c.seed >> 32);
  a.antithetic = c.antithetic; a.noise_mode = nv.mode; a.hidden_relu = c.hidden_act == 1; a.out_tanh = c.out_tanh != 0;
  a.env_f32 = (c.dtype == 1 && c.env_dtype == 1) ? 1u : 0u;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  const dim3 grid(s.N * s.E);
  const size_t lds = (size_t)s.D * sizeof(float);      // at most 65*64 + 65*64 + 65*16 values: 37 KB
  const int mode = (c.hidden_act == 1 ? 4 : 0) | (c.out_tanh ? 2 : 0) | (ctx->obs_mean ? 1 : 0);
  const int v = ctx->reg_variant;
  if (v < 0 || s.no > 64 || s.nh > 64 || s.na > 16 || s.m != 2)
    return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident binary32 variant for this shape");
  if (v == 0) launch_fixed<3, 2, 3>(mode, grid, lds, st, a);
  else if (v == 1) launch_fixed<5, 4, 6>(mode, grid, lds, st, a);
  else {
    const int k = v - REG_EXACT, oc = k / 9, hc = (k / 3) % 3, ac = k % 3;
    if (c.dtype == 1) launch_class<true>(oc, hc, ac, grid, lds, st, a);
    else launch_class<false>(oc, hc, ac, grid, lds, st, a);
  }
  int rc = check_launch(ctx, "es_rollout (register-resident f32)");
  if (rc != ES_OK) return rc;
  return launch_fitness(ctx, returns, fitness, st);
}

}  // namespace es
