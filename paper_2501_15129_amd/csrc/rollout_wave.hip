// es_rollout, general variant: one wavefront per (individual, environment copy).
//
// Paper Sec. 3.2: every individual of the population is evaluated at once, each on several
// parallel environment copies; Sec. 5.2: deterministic two-hidden-layer MLP policy, fitness
// = mean undiscounted episodic return.  This variant handles any layer widths whose
// perturbed weights fit in LDS (binary32, or bf16 bit patterns in bf16 mode): the
// perturbation theta + sign*sigma*eps is fused into the staging pass, so the perturbed
// parameters never exist in HBM, and they stay on chip for all T steps.
//
// Mapping: lane u of the wavefront owns output unit u (u + 64, ... for wider layers) of
// every layer; matrices are stored transposed in LDS with an odd row pitch so that the 64
// lanes read 64 consecutive banks, and the input vector is read as an LDS broadcast.
// Reward norms and the termination test are wavefront shuffle reductions.
// Bound: per-step latency of one wavefront (T dependent steps), not throughput.
#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

struct WaveArgs {
  const float* theta;
  const void* noise;
  const uint32_t* noise_offs;   // shared noise table: start of every row, else null
  const float* A;
  const float* B;
  const float* obs_mean;     // frozen observation statistics, or null
  const float* obs_inv;
  float* returns;
  int32_t* ep_len;
  uint32_t N, E, T, no, nh, na, D, ld, m;
  uint32_t oW1, ob1, oW2, ob2, oW3, ob3;
  uint32_t gen, k0, k1;
  uint32_t antithetic, out_tanh, noise_mode, hidden_relu;
  uint32_t env_f32;          // bf16 operands: the environment's products stay binary32 (its matrices then live among the floats)
  float sigma, done_thresh, act_cost;
};

template <bool BF16>
struct WStore;
template <>
struct WStore<false> {
  using T = float;
  __device__ static __forceinline__ T put(float v) { return v; }
  __device__ static __forceinline__ float get(T v) { return v; }
};
template <>
struct WStore<true> {
  using T = uint16_t;
  __device__ static __forceinline__ T put(float v) { return (uint16_t)bf16_bits(v); }
  __device__ static __forceinline__ float get(T v) { return bf16_to_f32(v); }
};

__host__ __device__ inline uint32_t odd_pitch(uint32_t n) { return n | 1u; }

// LDS carve-up, in elements of the weight type for matrices and floats for the rest.
struct WaveLayout {
  uint32_t p_h, p_a, p_o;                   // pitches
  size_t w1, w2, w3, at, bt, wcount;        // matrix offsets (weight elements)
  size_t b1, b2, b3, s, x, xp, mu, iv, h1, h2, a, qa, fcount;   // float offsets
};
// env_floats: the environment matrices are kept as binary32 among the floats (bf16 policy, binary32 environment)
// instead of among the weight elements.
__host__ __device__ inline WaveLayout wave_layout(uint32_t no, uint32_t nh, uint32_t na, uint32_t m, bool env_floats) {
  WaveLayout L;
  L.p_h = odd_pitch(nh); L.p_a = odd_pitch(na); L.p_o = odd_pitch(no);
  size_t o = 0;
  L.w1 = o; o += (size_t)no * L.p_h;
  L.w2 = o; o += (size_t)(m - 1) * nh * L.p_h;        // the m - 1 hidden-to-hidden matrices, one after the other
  L.w3 = o; o += (size_t)nh * L.p_a;
  if (!env_floats) {
    L.at = o; o += (size_t)no * L.p_o;
    L.bt = o; o += (size_t)na * L.p_o;
  }
  L.wcount = (o + 1) & ~(size_t)1;
  size_t f = 0;
  if (env_floats) {
    L.at = f; f += (size_t)no * L.p_o;
    L.bt = f; f += (size_t)na * L.p_o;
  }
  L.b1 = f; f += nh; L.b2 = f; f += (size_t)(m - 1) * nh; L.b3 = f; f += na;
  L.s = f; f += no; L.x = f; f += no; L.xp = f; f += no; L.mu = f; f += no; L.iv = f; f += no; L.h1 = f; f += nh; L.h2 = f; f += nh;
  L.a = f; f += na; L.qa = f; f += na;
  L.fcount = f;
  return L;
}

size_t wave_rollout_lds_bytes(const es_config& c) {
  const WaveLayout L = wave_layout(c.obs_dim, c.hid_dim, c.act_dim, c.num_hidden ? c.num_hidden : 2, c.dtype == 1 && c.env_dtype == 1);
  return L.fcount * 4 + L.wcount * (c.dtype == 1 ? 2 : 4);
}

template <bool BF16>
__global__ __launch_bounds__(64) void rollout_wave_kernel(const WaveArgs a) {
  using WS = WStore<BF16>;
  using WT = typename WS::T;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const bool envf = BF16 && a.env_f32 != 0u;
  const WaveLayout L = wave_layout(a.no, a.nh, a.na, a.m, envf);
  float* fl = reinterpret_cast<float*>(lds_raw);
  WT* wt = reinterpret_cast<WT*>(lds_raw + L.fcount * 4);
  // the environment's matrices and operands: bf16-rounded like the policy's, or binary32
  auto env_put = [&](size_t off, float v) { if (envf) fl[off] = v; else wt[off] = WS::put(BF16 ? bf16_round(v) : v); };
  auto env_get = [&](size_t off) { return envf ? fl[off] : WS::get(wt[off]); };
  auto env_opnd = [&](float v) { return (BF16 && !envf) ? bf16_round(v) : v; };

  const uint32_t lane = threadIdx.x;
  const uint32_t i = blockIdx.x / a.E, e = blockIdx.x % a.E;
  const uint32_t row = a.antithetic ? (i >> 1) : i;
  const float scale = (a.antithetic && (i & 1u)) ? -a.sigma : a.sigma;
  const uint32_t no = a.no, nh = a.nh, na = a.na;

  // ---- stage the perturbed parameters of individual i (fused perturbation) ----
  const void* nbase = a.noise;      // shared table: this individual's row, addressed as row 0
  uint32_t nrow = row;
  if (a.noise_offs) { nbase = table_row_base(a.noise_mode, a.noise, a.noise_offs, row); nrow = 0u; }
  auto place = [&](uint32_t d, float eps) {
    float v = __fmaf_rn(scale, eps, a.theta[d]);
    if (BF16) v = bf16_round(v);
    if (d < a.ob1) { const uint32_t u = d / no, k = d - u * no; wt[L.w1 + (size_t)k * L.p_h + u] = WS::put(v); }
    else if (d < a.oW2) fl[L.b1 + (d - a.ob1)] = v;
    else if (d < a.oW3) {          // hidden layer l + 2: matrix [nh, nh], then its bias
      const uint32_t per = (nh + 1u) * nh, q = d - a.oW2, l = q / per, r = q - l * per;
      if (r < nh * nh) { const uint32_t u = r / nh, k = r - u * nh; wt[L.w2 + ((size_t)l * nh + k) * L.p_h + u] = WS::put(v); }
      else fl[L.b2 + (size_t)l * nh + (r - nh * nh)] = v;
    }
    else if (d < a.ob3) { const uint32_t q = d - a.oW3, u = q / nh, k = q - u * nh; wt[L.w3 + (size_t)k * L.p_a + u] = WS::put(v); }
    else fl[L.b3 + (d - a.ob3)] = v;
  };
  if (a.noise_mode >= 2u) {       // regenerated noise: one counter block gives four consecutive parameters
    for (uint32_t d0 = 4u * lane; d0 < a.D; d0 += 256u) {
      float z[4];
      noise_regen4(row, d0, a.gen, a.k0, a.k1, a.noise_mode == 3u, z);
#pragma unroll
      for (uint32_t k = 0; k < 4u; ++k)
        if (d0 + k < a.D) place(d0 + k, z[k]);
    }
  } else {
    for (uint32_t d = lane; d < a.D; d += 64u) place(d, noise_value(a.noise_mode, nbase, a.ld, nrow, d, a.gen, a.k0, a.k1));
  }
  for (uint32_t q = lane; q < no * no; q += 64u) {
    const uint32_t k = q / no, j = q - k * no;
    env_put(L.at + (size_t)j * L.p_o + k, a.A[q]);
  }
  for (uint32_t q = lane; q < no * na; q += 64u) {
    const uint32_t k = q / na, c = q - k * na;
    env_put(L.bt + (size_t)c * L.p_o + k, a.B[q]);
  }
  for (uint32_t k = lane; k < no; k += 64u) {
    fl[L.s + k] = reset_value(k, e, a.gen, a.k0, a.k1);
    fl[L.mu + k] = a.obs_mean ? a.obs_mean[k] : 0.0f;        // identity statistics when none are set
    fl[L.iv + k] = a.obs_mean ? a.obs_inv[k] : 1.0f;
  }
  __syncthreads();

  float R = 0.0f;
  int32_t len = 0;
  const float inv_unused = 0.0f; (void)inv_unused;
  for (uint32_t t = 0; t < a.T; ++t) {
    float ss = 0.0f;
    for (uint32_t k = lane; k < no; k += 64u) {
      const float sv = fl[L.s + k];
      ss = __fmaf_rn(sv, sv, ss);
      fl[L.x + k] = env_opnd(sv);             // the environment's operand
      const float pv = (sv - fl[L.mu + k]) * fl[L.iv + k];   // the policy's input (paper App. B: fixed statistics)
      fl[L.xp + k] = BF16 ? bf16_round(pv) : pv;
    }
    __syncthreads();
    for (uint32_t u = lane; u < nh; u += 64u) {
      float acc = fl[L.b1 + u];
      for (uint32_t k = 0; k < no; ++k) acc = __fmaf_rn(WS::get(wt[L.w1 + (size_t)k * L.p_h + u]), fl[L.xp + k], acc);
      const float h = a.hidden_relu ? fmaxf(acc, 0.0f) : tanh_accurate(acc);
      fl[L.h1 + u] = BF16 ? bf16_round(h) : h;
    }
    __syncthreads();
    size_t hin = L.h1, hout = L.h2;       // the further hidden layers alternate between the two buffers
    for (uint32_t l = 0; l + 1 < a.m; ++l) {
      for (uint32_t u = lane; u < nh; u += 64u) {
        float acc = fl[L.b2 + (size_t)l * nh + u];
        for (uint32_t k = 0; k < nh; ++k) acc = __fmaf_rn(WS::get(wt[L.w2 + ((size_t)l * nh + k) * L.p_h + u]), fl[hin + k], acc);
        const float h = a.hidden_relu ? fmaxf(acc, 0.0f) : tanh_accurate(acc);
        fl[hout + u] = BF16 ? bf16_round(h) : h;
      }
      __syncthreads();
      const size_t tmp = hin; hin = hout; hout = tmp;
    }
    float aa = 0.0f;
    for (uint32_t c = lane; c < na; c += 64u) {
      float acc = fl[L.b3 + c];
      for (uint32_t k = 0; k < nh; ++k) acc = __fmaf_rn(WS::get(wt[L.w3 + (size_t)k * L.p_a + c]), fl[hin + k], acc);
      const float av = a.out_tanh ? tanh_accurate(acc) : acc;
      aa = __fmaf_rn(av, av, aa);
      fl[L.qa + c] = env_opnd(av);
    }
    __syncthreads();
    ss = wave_sum(ss);
    aa = wave_sum(aa);
    R += (1.0f - (ss / (float)no)) - a.act_cost * aa;
    len += 1;
    float mx = 0.0f;
    for (uint32_t k = lane; k < no; k += 64u) {
      float acc = 0.0f;
      for (uint32_t j = 0; j < no; ++j) acc = __fmaf_rn(env_get(L.at + (size_t)j * L.p_o + k), fl[L.x + j], acc);
      for (uint32_t c = 0; c < na; ++c) acc = __fmaf_rn(env_get(L.bt + (size_t)c * L.p_o + k), fl[L.qa + c], acc);
      const float sn = tanh_accurate(acc);
      mx = fmaxf(mx, fabsf(sn));
      fl[L.s + k] = sn;
    }
    mx = wave_max(mx);
    __syncthreads();
    if (mx > a.done_thresh) break;
  }
  if (lane == 0) {
    a.returns[(size_t)i * a.E + e] = R;
    a.ep_len[(size_t)i * a.E + e] = len;
  }
}

// fitness_i = mean over the E episodes, summed in index order.
__global__ __launch_bounds__(256) void fitness_kernel(const float* __restrict__ returns, float* __restrict__ fitness,
                                                      uint32_t N, uint32_t E) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= N) return;
  float s = 0.0f;
  for (uint32_t e = 0; e < E; ++e) s += returns[(size_t)i * E + e];
  fitness[i] = (s / (float)E);
}

int launch_fitness(es_ctx* ctx, const float* returns, float* fitness, hipStream_t st) {
  const Shape& s = ctx->shp;
  hipLaunchKernelGGL(fitness_kernel, dim3((s.N + 255) / 256), dim3(256), 0, st, returns, fitness, s.N, s.E);
  return check_launch(ctx, "es_rollout (fitness)");
}

int launch_rollout_wave(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise, const float* A,
                        const float* B, float* returns, int32_t* ep_len, float* fitness, void* /*ws*/,
                        hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  WaveArgs a;
  const NoiseView nv = noise_view(ctx, noise);
  a.theta = theta; a.noise = nv.base; a.noise_offs = nv.offs; a.A = A; a.B = B; a.obs_mean = ctx->obs_mean; a.obs_inv = ctx->obs_inv_std; a.returns = returns; a.ep_len = ep_len;
  a.N = s.N; a.E = s.E; a.T = s.T; a.no = s.no; a.nh = s.nh; a.na = s.na; a.D = s.D; a.ld = s.ld; a.m = s.m;
  a.oW1 = s.oW1; a.ob1 = s.ob1; a.oW2 = s.oW2; a.ob2 = s.ob2; a.oW3 = s.oW3; a.ob3 = s.ob3;
  a.gen = gen; a.k0 = (uint32_t)c.seed; a.k1 = (uint32_t)(c.seed >> 32);
  a.antithetic = c.antithetic; a.out_tanh = c.out_tanh; a.noise_mode = nv.mode; a.hidden_relu = c.hidden_act == 1;
  a.env_f32 = (c.dtype == 1 && c.env_dtype == 1) ? 1u : 0u;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  const size_t lds = ctx->lds_bytes_wave;
  hipError_t err;
  if (c.dtype == 1) {
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(rollout_wave_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(err));
    hipLaunchKernelGGL(rollout_wave_kernel<true>, dim3(s.N * s.E), dim3(64), lds, st, a);
  } else {
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(rollout_wave_kernel<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(err));
    hipLaunchKernelGGL(rollout_wave_kernel<false>, dim3(s.N * s.E), dim3(64), lds, st, a);
  }
  int rc = check_launch(ctx, "es_rollout (wave/LDS)");
  if (rc != ES_OK) return rc;
  return launch_fitness(ctx, returns, fitness, st);
}

}  // namespace es
