// es_rollout, register-resident matrix-core variant for BINARY32 policies with a wide hidden layer.
//
// Paper Sec. 5.1 times OpenES on policies with m hidden layers of 256 units in the framework's default
// precision; Sec. 3.2 / 5.2 define the evaluation (population x environment copies, fitness = mean
// undiscounted return).  A 256-wide two-layer policy is 272-300 KB in binary32: more than the LDS, less than
// the 512 KB register file of a CU.  One workgroup of four wavefronts evaluates one individual on up to 16
// environment copies per pass, every product on the fp32 16x16x4 MFMA (lane (g, n) supplies A[row n][k = g]
// and B[k = g][column n]; the 16 columns are the environment copies):
//
//   * each wavefront owns 64 units (four 16-row tiles) of both hidden layers; its rows of W1 and W2 sit in
//     registers as MFMA A operands for all T steps (W2: 256 registers per lane, in the accumulation half of
//     the file), the perturbation fused into the load;
//   * the K order of a product is free as long as both operands agree, so it is chosen per layer such that a
//     lane's operands are contiguous where they come from: layer 1 and A s read the lane's KPL consecutive
//     state elements of its column from the binary32 state buffer; layer 2 reads 64 consecutive units of h1;
//     the action layer is split along K - every wavefront multiplies the h2 units it has just produced, still
//     in its registers, with its slice of W3, and only the partial sums cross the LDS; B a takes the action
//     from the registers the reduction leaves it in;
//   * three workgroup barriers per step (h1, action partials, new state); the norms for the reward and the
//     termination test are reduced inside a wavefront with the row-swap instructions and across wavefronts
//     through one LDS partial per wavefront, added by every lane in the same order: reruns are bit-identical.
// Bound: the fp32 MFMA pipe (32 cycles per 16x16x4 instruction, 4 (KPL + 64 + 4) + KPL + 4 of them per step).
//
// Up to eight copies per individual (and policies with ONE hidden layer) run on a second kernel further down, built on the
// 4x4x1 shape with four copies per pass: a quarter of the matrix-pipe time when only one to four columns carry episodes.
#include <algorithm>
#include <type_traits>

#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct F32Args {
  const float* theta;
  const void* noise;
  const uint32_t* noise_offs;   // shared noise table: start of every row, else null
  const float* A;
  const float* B;
  const float* obs_mean;        // frozen observation statistics (paper App. B), or null
  const float* obs_inv;
  float* returns;
  int32_t* ep_len;
  float* fitness;
  uint32_t N, E, T, no, nh, na, ld;
  uint32_t oW1, ob1, oW2, ob2, oW3, ob3;
  uint32_t gen, k0, k1;
  uint32_t antithetic, out_tanh, noise_mode;
  float sigma, done_thresh, act_cost;
};

constexpr int NHP = 256;       // padded hidden width
constexpr int NCOL = 16;       // environment copies per pass
constexpr int PH = NHP + 4;    // LDS pitch (floats) of an h1 row: 16-byte reads of 16 lanes hit distinct banks

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
__device__ __forceinline__ void pin_agpr(float& v) { asm volatile("" : "+a"(v)); }
__device__ __forceinline__ void pin_vgpr(float& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ unsigned umax(unsigned a, unsigned b) { return a > b ? a : b; }
__device__ __forceinline__ unsigned abs_bits(float v) { return __builtin_bit_cast(unsigned, v) & 0x7FFFFFFFu; }
// sum / max over the four 16-lane rows of the wavefront (lanes l, l+16, l+32, l+48), result in every row
__device__ __forceinline__ float rows_sum(float v) {
  const unsigned b = __builtin_bit_cast(unsigned, v);
  const auto p = __builtin_amdgcn_permlane16_swap(b, b, false, false);
  const float t = __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
  const unsigned c = __builtin_bit_cast(unsigned, t);
  const auto r = __builtin_amdgcn_permlane32_swap(c, c, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
__device__ __forceinline__ unsigned rows_umax(unsigned b) {
  const auto p = __builtin_amdgcn_permlane16_swap(b, b, false, false);
  const unsigned c = umax((unsigned)p[0], (unsigned)p[1]);
  const auto r = __builtin_amdgcn_permlane32_swap(c, c, false, false);
  return umax((unsigned)r[0], (unsigned)r[1]);
}
__device__ __forceinline__ f32x4 tanh4(f32x4 v) { return f32x4{tanh_fast(v.x), tanh_fast(v.y), tanh_fast(v.z), tanh_fast(v.w)}; }
template <bool RELU>
__device__ __forceinline__ f32x4 hidden4(f32x4 v) {
  if (RELU) return f32x4{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
  return tanh4(v);
}

__device__ __forceinline__ float noise_f32(float e) { return e; }
__device__ __forceinline__ float noise_f32(uint16_t e) { return bf16_to_f32(e); }
// One noise row under any storage mode, and the perturbed parameters of an individual written into an LDS window:
//   win[map(q).dst] = map(q).ok ? fma(scale, noise[map(q).idx], theta[map(q).idx]) : 0     for q = tid, tid + 256, ... < total.
// The loads of eight iterations are issued together and unconditionally (a masked-out element reads parameter 0, which is
// always there) and only then consumed: a load inside the bounds test would be waited for in its own iteration.
struct ParamSrc {
  const float* theta;
  const void* nbase;        // stored noise: the row (table modes: the row's start), else unused
  uint32_t mode, ld, nrow, gen, k0, k1;
  float scale;
  __device__ __forceinline__ float one(uint32_t idx) const {
    return __fmaf_rn(scale, noise_value(mode, nbase, ld, nrow, idx, gen, k0, k1), theta[idx]);
  }
};
struct Slot { int dst; uint32_t idx; bool ok; };
template <class Map>
__device__ __forceinline__ void stage_params(float* win, int total, int tid, const ParamSrc& ps, Map map) {
  constexpr int U = 8;
  auto batch = [&](auto fetch) {
    for (int q0 = tid; q0 < total; q0 += U * 256) {
      float th[U];
      decltype(fetch(0u)) ez[U];
      Slot sl[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int q = q0 + u * 256;
        sl[u] = map(q < total ? q : tid);
        sl[u].ok = sl[u].ok && q < total;
        const uint32_t idx = sl[u].ok ? sl[u].idx : 0u;
        th[u] = ps.theta[idx];
        ez[u] = fetch(idx);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (q0 + u * 256 < total) win[sl[u].dst] = sl[u].ok ? __fmaf_rn(ps.scale, noise_f32(ez[u]), th[u]) : 0.0f;
    }
  };
  if (ps.mode >= 2u) {          // regenerated: arithmetic only
    for (int q = tid; q < total; q += 256) {
      const Slot sl = map(q);
      win[sl.dst] = sl.ok ? ps.one(sl.idx) : 0.0f;
    }
  } else if (ps.mode == 1u) {
    const uint16_t* row = static_cast<const uint16_t*>(ps.nbase) + (size_t)ps.nrow * ps.ld;
    batch([&](uint32_t idx) { return row[idx]; });
  } else {
    const float* row = static_cast<const float*>(ps.nbase) + (size_t)ps.nrow * ps.ld;
    batch([&](uint32_t idx) { return row[idx]; });
  }
}

// KPL: state elements per lane group of the K dimension (padded observation width NOP = 4 KPL: 32 or 64)
template <int KPL>
struct Lds {
  static constexpr int NOP = 4 * KPL;
  static constexpr int PXF = NOP + 4;                      // pitch of a state row (floats)
  static constexpr int OFF_H1 = 0;                         // [copy][PH] f32
  static constexpr int OFF_XF = OFF_H1 + 4 * NCOL * PH;    // [copy][PXF] f32
  static constexpr int OFF_P3 = OFF_XF + 4 * NCOL * PXF;   // action partials [wavefront][copy][16 rows] f32
  static constexpr int OFF_SSP = OFF_P3 + 4 * 4 * NCOL * 16;   // |s'|^2 partials [copy][wavefront]
  static constexpr int OFF_MXP = OFF_SSP + 4 * NCOL * 4;       // max|s'| partials, same layout
  static constexpr int OFF_B1 = OFF_MXP + 4 * NCOL * 4;
  static constexpr int OFF_B2 = OFF_B1 + 4 * NHP;
  static constexpr int OFF_B3 = OFF_B2 + 4 * NHP;
  static constexpr int OFF_MU = OFF_B3 + 4 * 16;
  static constexpr int OFF_IV = OFF_MU + 4 * NOP;
  static constexpr int OFF_SCR = OFF_IV + 4 * NOP;         // scratch for the initial-state norms [16][16]
  static constexpr int OFF_WIN = OFF_SCR + 4 * 256;        // staging window [256][65] f32
  static constexpr int BYTES = OFF_WIN + 4 * NHP * 65;
};

template <int KPL, bool RELU, bool NORM>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void rollout_mfma_f32_kernel(const F32Args a) {
  using L = Lds<KPL>;
  constexpr int NOP = L::NOP, PXF = L::PXF;
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n = lane & 15;
  const int no = (int)a.no, nh = (int)a.nh, na = (int)a.na;
  float* h1s = reinterpret_cast<float*>(lds + L::OFF_H1);
  float* xfs = reinterpret_cast<float*>(lds + L::OFF_XF);
  float* p3s = reinterpret_cast<float*>(lds + L::OFF_P3);
  float* ssps = reinterpret_cast<float*>(lds + L::OFF_SSP);
  unsigned* mxps = reinterpret_cast<unsigned*>(lds + L::OFF_MXP);
  float* b1s = reinterpret_cast<float*>(lds + L::OFF_B1);
  float* b2s = reinterpret_cast<float*>(lds + L::OFF_B2);
  float* b3s = reinterpret_cast<float*>(lds + L::OFF_B3);
  float* mus = reinterpret_cast<float*>(lds + L::OFF_MU);
  float* ivs = reinterpret_cast<float*>(lds + L::OFF_IV);
  const bool env_wave = 16 * w < NOP;                     // this wavefront owns state rows 16w..16w+15

  // ---- environment matrices -> registers (once per workgroup): Af[kk] = A[16w + n][KPL g + kk], Bf[kk] = B[16w + n][4g + kk]
  float Af[KPL], Bf[4];
  {
    const int row = 16 * w + n;
#pragma unroll
    for (int kk = 0; kk < KPL; ++kk) { const int k = KPL * g + kk; Af[kk] = (row < no && k < no) ? a.A[row * no + k] : 0.0f; }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) { const int c = 4 * g + kk; Bf[kk] = (row < no && c < na) ? a.B[row * na + c] : 0.0f; }
  }
  if (NORM) {
    for (int k = tid; k < NOP; k += 256) {
      mus[k] = k < no ? a.obs_mean[k] : 0.0f;
      ivs[k] = k < no ? a.obs_inv[k] : 0.0f;
    }
  }
  const uint32_t per_unit = a.antithetic ? 2u : 1u;
  const uint32_t nblk = (a.E + (uint32_t)NCOL - 1u) / (uint32_t)NCOL;
  const float inv_no = 1.0f / (float)no;

  for (uint32_t i = blockIdx.x; i < a.N; i += gridDim.x) {
    const uint32_t unit = i / per_unit, sub = i - unit * per_unit;
    const float scale = sub ? -a.sigma : a.sigma;
    const void* nbase = a.noise;
    uint32_t nrow = unit;
    if (a.noise_offs) { nbase = table_row_base(a.noise_mode, a.noise, a.noise_offs, unit); nrow = 0u; }
    const ParamSrc ps{a.theta, nbase, a.noise_mode, a.ld, nrow, a.gen, a.k0, a.k1, scale};
    __syncthreads();          // the previous individual's last reads of the bias arrays are done
    // ---- perturbed parameters -> LDS window (coalesced) -> registers, a slab at a time ----
    // The window holds 256 rows x 64 columns (pitch 65).  W2 goes through it in four slabs: slab c = columns
    // 64g + 16c .. + 15 of every lane group g, so that a lane picks its K slots 16c .. 16c + 15 of all four tiles.
    float W1r[4][KPL], W2r[4][64], W3k[16];
    float* win = reinterpret_cast<float*>(lds + L::OFF_WIN);
    constexpr int PWIN = 65;
    stage_params(win, NHP * NOP, tid, ps, [&](int q) {
      const int row = q / NOP, k = q - row * NOP;
      return Slot{row * PWIN + k, a.oW1 + (uint32_t)(row * no + k), row < nh && k < no};
    });
    __syncthreads();
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int kk = 0; kk < KPL; ++kk) W1r[tt][kk] = win[(64 * w + 16 * tt + n) * PWIN + KPL * g + kk];
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      stage_params(win, NHP * 64, tid, ps, [&](int q) {
        const int row = q >> 6, cc = q & 63, k = 64 * (cc >> 4) + 16 * c + (cc & 15);
        return Slot{row * PWIN + cc, a.oW2 + (uint32_t)(row * nh + k), row < nh && k < nh};
      });
      __syncthreads();
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int q = 0; q < 16; ++q) W2r[tt][16 * c + q] = win[(64 * w + 16 * tt + n) * PWIN + 16 * g + q];
      __syncthreads();
    }
    // action layer: K slot (j, g) = unit 64w + 16 (j / 4) + 4g + (j % 4), the order of h2 in the registers
    stage_params(win, 16 * NHP, tid, ps, [&](int q) {
      const int row = q >> 8, u = q & 255;
      return Slot{row * (NHP + 1) + u, a.oW3 + (uint32_t)(row * nh + u), row < na && u < nh};
    });
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) W3k[j] = win[n * (NHP + 1) + 64 * w + 16 * (j >> 2) + 4 * g + (j & 3)];
    stage_params(b1s, NHP, tid, ps, [&](int u) { return Slot{u, a.ob1 + (uint32_t)u, u < nh}; });
    stage_params(b2s, NHP, tid, ps, [&](int u) { return Slot{u, a.ob2 + (uint32_t)u, u < nh}; });
    stage_params(b3s, 16, tid, ps, [&](int c) { return Slot{c, a.ob3 + (uint32_t)c, c < na}; });
    float fit_sum = 0.0f;
    for (uint32_t cb = 0; cb < nblk; ++cb) {
      // ---- initial states of this block of copies, their norms as the partials of "step -1" ----
      __syncthreads();
      {
        const int n0 = tid & 15, kq = tid >> 4;
        const uint32_t e0 = cb * (uint32_t)NCOL + (uint32_t)n0;
        float part = 0.0f;
        for (int k = kq; k < NOP; k += 16) {
          float v = 0.0f;
          if (k < no && e0 < a.E) v = reset_value((uint32_t)k, e0, a.gen, a.k0, a.k1);
          part = __fmaf_rn(v, v, part);
          xfs[n0 * PXF + k] = v;
        }
        float* scratch = reinterpret_cast<float*>(lds + L::OFF_SCR);
        scratch[kq * 16 + n0] = part;
        __syncthreads();
        if (tid < 16) {
          float s = 0.0f;
          for (int r = 0; r < 16; ++r) s += scratch[r * 16 + tid];
          ssps[tid * 4] = s; ssps[tid * 4 + 1] = 0.0f; ssps[tid * 4 + 2] = 0.0f; ssps[tid * 4 + 3] = 0.0f;
          mxps[tid * 4] = 0u; mxps[tid * 4 + 1] = 0u; mxps[tid * 4 + 2] = 0u; mxps[tid * 4 + 3] = 0u;
        }
        __syncthreads();
      }
      const uint32_t e = cb * (uint32_t)NCOL + (uint32_t)n;
      bool alive = e < a.E;
      float Rn = 0.0f, aa_prev = 0.0f, ss_cur = 0.0f;
      int32_t Ln = 0;
      bool first = true;

      for (uint32_t t = 0; t <= a.T; ++t) {
        // ---- phase A: books of the previous step; h1 = act(W1 x + b1); A s ----
        const f32x4 sp4 = *reinterpret_cast<const f32x4*>(ssps + 4 * n);
        const u32x4 mp4 = *reinterpret_cast<const u32x4*>(mxps + 4 * n);
        float xf[KPL], xp[KPL];
#pragma unroll
        for (int j = 0; j < KPL / 4; ++j) {
          const f32x4 v4 = *reinterpret_cast<const f32x4*>(xfs + n * PXF + KPL * g + 4 * j);
          xf[4 * j] = v4.x; xf[4 * j + 1] = v4.y; xf[4 * j + 2] = v4.z; xf[4 * j + 3] = v4.w;
        }
#pragma unroll
        for (int kk = 0; kk < KPL; ++kk) xp[kk] = NORM ? (xf[kk] - mus[KPL * g + kk]) * ivs[KPL * g + kk] : xf[kk];
        f32x4 acc[4];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b1s + 64 * w + 16 * tt + 4 * g);
#pragma unroll
        for (int kk = 0; kk < KPL; ++kk)
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) {
            if (KPL > 8 && tt < 2) pin_agpr(W1r[tt][kk]);      // the wider observation: half of W1 joins W2 in the accumulation half
            acc[tt] = mfma4(W1r[tt][kk], xp[kk], acc[tt]);
          }
        {
          const float ss_new = (sp4.x + sp4.y) + (sp4.z + sp4.w);
          const float mx = __builtin_bit_cast(float, umax(umax(mp4.x, mp4.y), umax(mp4.z, mp4.w)));
          const bool book = !first, add = book && alive;
          const float r = __fmaf_rn(-ss_cur, inv_no, 1.0f) - a.act_cost * aa_prev;
          Rn += add ? r : 0.0f;
          Ln += add ? 1 : 0;
          alive = alive && !(book && mx > a.done_thresh);
          ss_cur = ss_new;
          first = false;
        }
        if (t == a.T || __ballot(alive) == 0ull) break;       // identical in all four wavefronts
        f32x4 accE = f32x4{0.f, 0.f, 0.f, 0.f};
        if (env_wave) {
#pragma unroll
          for (int kk = 0; kk < KPL; ++kk) accE = mfma4(Af[kk], xf[kk], accE);
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const f32x4 h = hidden4<RELU>(acc[tt]);
          *reinterpret_cast<f32x4*>(h1s + n * PH + 64 * w + 16 * tt + 4 * g) = h;
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b2s + 64 * w + 16 * tt + 4 * g);
        __syncthreads();
        // ---- phase B: h2 = act(W2 h1 + b2); K slot (kk, g) = unit 64g + kk: 64 consecutive values of the lane's column ----
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const f32x4 hb = *reinterpret_cast<const f32x4*>(h1s + n * PH + 64 * g + 4 * j);
#pragma unroll
          for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
              // three of the four tiles of W2 live in the accumulation half of the register file (192 of its 256
              // registers; the rest is left to the compiler), the fourth beside everything else in the architectural half
              if (tt < 3) pin_agpr(W2r[tt][4 * j + r]); else pin_vgpr(W2r[tt][4 * j + r]);
              acc[tt] = mfma4(W2r[tt][4 * j + r], hb[r], acc[tt]);
            }
        }
        // this wavefront's K slice of the action layer, from the registers that hold its h2
        // (four partial accumulators: a dependent 16x16x4 MFMA waits out the previous one's eight passes)
        f32x4 p3q[4];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const f32x4 h = hidden4<RELU>(acc[tt]);
#pragma unroll
          for (int r = 0; r < 4; ++r) p3q[r] = mfma4(W3k[4 * tt + r], h[r], tt == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : p3q[r]);
        }
        *reinterpret_cast<f32x4*>(p3s + (w * NCOL + n) * 16 + 4 * g) = (p3q[0] + p3q[1]) + (p3q[2] + p3q[3]);
        __syncthreads();
        // ---- phase D: a = tanh(sum of the partials + b3); s' = tanh(A s + B a); norms ----
        f32x4 v = *reinterpret_cast<const f32x4*>(b3s + 4 * g);
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) v += *reinterpret_cast<const f32x4*>(p3s + (ww * NCOL + n) * 16 + 4 * g);
        {
          const f32x4 tv = tanh4(v);
          const bool squash = a.out_tanh != 0u;
          v = f32x4{squash ? tv.x : v.x, squash ? tv.y : v.y, squash ? tv.z : v.z, squash ? tv.w : v.w};
        }
        float part = v.x * v.x;
        part = __fmaf_rn(v.y, v.y, part); part = __fmaf_rn(v.z, v.z, part); part = __fmaf_rn(v.w, v.w, part);
        aa_prev = rows_sum(part);                  // |a_t|^2 of column n (rows past the action width are exactly zero)
        float ssp = 0.0f;
        unsigned mxp = 0u;
        if (env_wave) {
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) accE = mfma4(Bf[kk], v[kk], accE);       // K slot (kk, g) = action row 4g + kk
          const f32x4 sn = tanh4(accE);
          ssp = sn.x * sn.x;
          ssp = __fmaf_rn(sn.y, sn.y, ssp); ssp = __fmaf_rn(sn.z, sn.z, ssp); ssp = __fmaf_rn(sn.w, sn.w, ssp);
          mxp = umax(umax(abs_bits(sn.x), abs_bits(sn.y)), umax(abs_bits(sn.z), abs_bits(sn.w)));
          *reinterpret_cast<f32x4*>(xfs + n * PXF + 16 * w + 4 * g) = sn;
        }
        ssp = rows_sum(ssp);
        mxp = rows_umax(mxp);
        if (g == 0) { ssps[n * 4 + w] = ssp; mxps[n * 4 + w] = mxp; }
        __syncthreads();
      }
      // ---- outputs of this block of copies ----
      if (w == 0) {
        const uint32_t cnt = min((uint32_t)NCOL, a.E - cb * (uint32_t)NCOL);
        if (g == 0 && (uint32_t)n < cnt) {
          a.returns[(size_t)i * a.E + e] = Rn;
          a.ep_len[(size_t)i * a.E + e] = Ln;
        }
        for (uint32_t r = 0; r < cnt; ++r) fit_sum += __shfl(Rn, (int)r, 64);
      }
    }
    if (tid == 0) a.fitness[i] = fit_sum / (float)a.E;
  }
}


// ---------------------------------------------------------------------------------------------------------------
// Passes of FOUR copies (the paper's timing experiment evaluates one episode per individual, Sec. 5.1): the 4x4x1
// shape.  One v_mfma_f32_4x4x1 is sixteen independent 4x4 outer products: lane 4b + x supplies A_b[row x] and
// B_b[column x] of block b, and holds D_b[rows 0..3][column x] in its four result registers; with cbsz / abid the A
// values of one block are broadcast to a group of 2^cbsz blocks.  Here the activations are the A operand (row =
// copy, broadcast from the block that holds them) and the weights the B operand (column = the lane's own unit), so
//   * a lane owns ONE unit and accumulates that unit's value for the four copies in its four result registers:
//     no padded columns, a quarter of the matrix-pipe time of the 16-column shape;
//   * a wavefront's 64 units of h1 are at once its K slice of layer 2 (the whole kernel is split along K): after
//     the activation a 4x4 transpose inside each lane quad (register index <-> lane in quad) turns "unit per
//     lane, copy per register" into the A operand "copy per lane, unit per register", and h1 never leaves the
//     wavefront.  Layer 2 produces partial sums for all 256 units; they cross the LDS once, every wavefront adds
//     the four partials of its own 64 units in the same order;
//   * the action layer uses groups of four blocks (cbsz = 2): one instruction multiplies four K values with the
//     sixteen action rows, 16 instructions per wavefront, then a sum over the four lane rows and the partials
//     [wavefront][copy][action] through LDS;
//   * the environment step (obs <= 64: one row per lane) is computed by EVERY wavefront for itself from the same
//     operands in the same order: the state, the norms and the books never cross the LDS, and the four wavefronts
//     stay bit-identical.  Two workgroup barriers per step.
constexpr int NCN = 4;          // copies per pass

// compile-time loop: body(std::integral_constant<int, I>) for I = 0 .. N - 1 (the broadcast block of an MFMA is an immediate)
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& body) {
  if constexpr (I < N) {
    body(std::integral_constant<int, I>{});
    static_for<I + 1, N>(body);
  }
}
// A values of block ABID broadcast to all sixteen blocks
template <int ABID>
__device__ __forceinline__ f32x4 mfma1_all(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 4, ABID, 0); }
// ... of block ABID of every group of four blocks to the blocks of that group
template <int ABID>
__device__ __forceinline__ f32x4 mfma1_group(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 2, ABID, 0); }

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// 4x4 transpose inside every quad of lanes: out[j] of lane (b, i) = in[i] of lane (b, j)
__device__ __forceinline__ f32x4 quad_transpose(f32x4 v, bool p, bool q) {
  // exchange across lane bit 0 (partner = lane ^ 1): register pairs (0, 1) and (2, 3)
  const float s01 = dpp_f<0xB1>(p ? v.x : v.y), s23 = dpp_f<0xB1>(p ? v.z : v.w);      // quad_perm [1, 0, 3, 2]
  f32x4 u = f32x4{p ? s01 : v.x, p ? v.y : s01, p ? s23 : v.z, p ? v.w : s23};
  // exchange across lane bit 1 (partner = lane ^ 2): register pairs (0, 2) and (1, 3)
  const float s02 = dpp_f<0x4E>(q ? u.x : u.z), s13 = dpp_f<0x4E>(q ? u.y : u.w);      // quad_perm [2, 3, 0, 1]
  return f32x4{q ? s02 : u.x, q ? s13 : u.y, q ? u.z : s02, q ? u.w : s13};
}
// sum / max over the sixteen blocks of the lanes with the same position in their quad; result in every lane
__device__ __forceinline__ float blocks_sum(float v) {
  v += dpp_f<0x124>(v);        // row_ror 4
  v += dpp_f<0x128>(v);        // row_ror 8
  return rows_sum(v);
}
__device__ __forceinline__ unsigned blocks_umax(unsigned v) {
  v = umax(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x124, 0xF, 0xF, true));
  v = umax(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, true));
  return rows_umax(v);
}

template <int KO>
struct LdsN {
  static constexpr int PWN = NHP + 1;                       // pitch of a window row of 256 columns
  static constexpr int OFF_P2 = 0;                          // layer-2 partials [producer wavefront][unit][copy] f32
  static constexpr int OFF_P3 = OFF_P2 + 4 * 4 * NHP * NCN; // action partials [wavefront][copy][16 rows] f32
  static constexpr int OFF_B1 = OFF_P3 + 4 * 4 * NCN * 16;
  static constexpr int OFF_B2 = OFF_B1 + 4 * NHP;
  static constexpr int OFF_B3 = OFF_B2 + 4 * NHP;
  static constexpr int OFF_WIN = OFF_B3 + 4 * 16;           // staging window: [256][KO + 1], [64][257] or [16][257] f32
  static constexpr int WIN_FLOATS = 64 * PWN > NHP * (KO + 1) ? 64 * PWN : NHP * (KO + 1);
  static constexpr int BYTES = OFF_WIN + 4 * WIN_FLOATS;
};

// KO: padded observation width (16, 32 or 64): the K extent of layer 1 and of A s.  TWO: two hidden layers; with one
// (the paper's depth sweep, Sec. 5.1) layer 1 feeds the action layer directly and a step has a single barrier.
template <int KO, bool RELU, bool NORM, bool TWO>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void rollout_mfma_f32_narrow_kernel(const F32Args a) {
  using L = LdsN<KO>;
  constexpr int PWN = L::PWN;
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = lane >> 2, x = lane & 3;           // block of the 4x4x1 shape, position in the quad
  const bool xp0 = (x & 1) != 0, xp1 = (x & 2) != 0;
  const int no = (int)a.no, nh = (int)a.nh, na = (int)a.na;
  float* p2s = reinterpret_cast<float*>(lds + L::OFF_P2);
  float* p3s = reinterpret_cast<float*>(lds + L::OFF_P3);
  float* b1s = reinterpret_cast<float*>(lds + L::OFF_B1);
  float* b2s = reinterpret_cast<float*>(lds + L::OFF_B2);
  float* b3s = reinterpret_cast<float*>(lds + L::OFF_B3);
  float* win = reinterpret_cast<float*>(lds + L::OFF_WIN);
  const int unit = 64 * w + lane;                    // this lane's unit of both hidden layers

  // ---- environment matrices -> registers (once per workgroup; every wavefront steps the whole environment):
  //      state row = lane: Ae[k] = A[lane][k], Be[c] = B[lane][c]; observation statistics of rows 4 blk .. 4 blk + 3
  float Ae[KO], Be[16];
#pragma unroll
  for (int k = 0; k < KO; ++k) Ae[k] = (lane < no && k < no) ? a.A[lane * no + k] : 0.0f;
#pragma unroll
  for (int c = 0; c < 16; ++c) Be[c] = (lane < no && c < na) ? a.B[lane * na + c] : 0.0f;
  f32x4 mu4 = f32x4{0.f, 0.f, 0.f, 0.f}, iv4 = mu4;        // padded rows get scale 0: their normalised value stays 0
  if (NORM) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = 4 * blk + j;
      mu4[j] = r < no ? a.obs_mean[r] : 0.0f;
      iv4[j] = r < no ? a.obs_inv[r] : 0.0f;
    }
  }
  const uint32_t per_unit = a.antithetic ? 2u : 1u;
  const uint32_t nblk = (a.E + (uint32_t)NCN - 1u) / (uint32_t)NCN;
  const float inv_no = 1.0f / (float)no;

  for (uint32_t i = blockIdx.x; i < a.N; i += gridDim.x) {
    const uint32_t punit = i / per_unit, sub = i - punit * per_unit;
    const float scale = sub ? -a.sigma : a.sigma;
    const void* nbase = a.noise;
    uint32_t nrow = punit;
    if (a.noise_offs) { nbase = table_row_base(a.noise_mode, a.noise, a.noise_offs, punit); nrow = 0u; }
    const ParamSrc ps{a.theta, nbase, a.noise_mode, a.ld, nrow, a.gen, a.k0, a.k1, scale};
    __syncthreads();          // the previous individual's last reads of the bias arrays are done
    // ---- perturbed parameters -> LDS window (coalesced) -> registers ----
    float W1s[KO], W2k[TWO ? 4 : 1][TWO ? 64 : 1], W3k[16];
    stage_params(win, NHP * KO, tid, ps, [&](int q) {
      const int row = q / KO, k = q - row * KO;
      return Slot{row * (KO + 1) + k, a.oW1 + (uint32_t)(row * no + k), row < nh && k < no};
    });
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KO; ++k) W1s[k] = win[unit * (KO + 1) + k];           // W1[unit][k]
    __syncthreads();
    if constexpr (TWO) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {    // rows 64 t .. 64 t + 63 of W2: the lane keeps row 64 t + lane, columns of its wavefront's K slice
        stage_params(win, 64 * NHP, tid, ps, [&](int q) {
          const int r = q >> 8, c = q & 255, row = 64 * t + r;
          return Slot{r * PWN + c, a.oW2 + (uint32_t)(row * nh + c), row < nh && c < nh};
        });
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 64; ++kk) W2k[t][kk] = win[lane * PWN + 64 * w + kk];
        __syncthreads();
      }
    }
    // action layer: lane (group g = blk / 4, ag = blk % 4, x) serves action row 4 ag + x; its K value number 4 a' + j'
    // is unit 64 w + 16 g + 4 a' + j' (block 4 g + a' of the transposed h2, register j')
    stage_params(win, 16 * NHP, tid, ps, [&](int q) {
      const int row = q >> 8, u = q & 255;
      return Slot{row * PWN + u, a.oW3 + (uint32_t)(row * nh + u), row < na && u < nh};
    });
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) W3k[r] = win[(4 * (blk & 3) + x) * PWN + 64 * w + 16 * (blk >> 2) + r];
    stage_params(b1s, NHP, tid, ps, [&](int u) { return Slot{u, a.ob1 + (uint32_t)u, u < nh}; });
    if constexpr (TWO) stage_params(b2s, NHP, tid, ps, [&](int u) { return Slot{u, a.ob2 + (uint32_t)u, u < nh}; });
    stage_params(b3s, 16, tid, ps, [&](int c) { return Slot{c, a.ob3 + (uint32_t)c, c < na}; });
    __syncthreads();
    const float b1u = b1s[unit], b2u = TWO ? b2s[unit] : 0.0f;
    f32x4 b3q = f32x4{0.f, 0.f, 0.f, 0.f};          // biases of action rows 4 blk .. 4 blk + 3 (blocks 0..3 hold the action)
    if (blk < 4) b3q = *reinterpret_cast<const f32x4*>(b3s + 4 * blk);

    float fit_sum = 0.0f;
    for (uint32_t cb = 0; cb < nblk; ++cb) {
      // ---- initial state, transposed: lane (blk, x) holds rows 4 blk .. 4 blk + 3 of copy x ----
      const uint32_t e = cb * (uint32_t)NCN + (uint32_t)x;
      bool alive = e < a.E;
      f32x4 ts;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = 4 * blk + j;
        ts[j] = (r < no && e < a.E) ? reset_value((uint32_t)r, e, a.gen, a.k0, a.k1) : 0.0f;
      }
      float ss_cur;
      {
        float part = ts.x * ts.x;
        part = __fmaf_rn(ts.y, ts.y, part); part = __fmaf_rn(ts.z, ts.z, part); part = __fmaf_rn(ts.w, ts.w, part);
        ss_cur = blocks_sum(part);
      }
      float Rn = 0.0f;
      int32_t Ln = 0;

      for (uint32_t t = 0; t < a.T; ++t) {
        if (__ballot(alive) == 0ull) break;         // identical in all four wavefronts
        // ---- layer 1 and A s: both read the state; K value r sits in block r / 4, register r % 4 ----
        f32x4 tp = ts;
        if (NORM) tp = (ts - mu4) * iv4;
        // (a result is ready for the next instruction on the same accumulator only three to four issue slots later:
        //  every product keeps several partial accumulators and adds them at the end)
        const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
        f32x4 acc1[2] = {f32x4{b1u, b1u, b1u, b1u}, zero4}, accE[4] = {zero4, zero4, zero4, zero4};
        static_for<0, KO>([&](auto rc) {
          constexpr int r = decltype(rc)::value;
          acc1[r % 2] = mfma1_all<r / 4>(tp[r % 4], W1s[r], r == 1 ? zero4 : acc1[r % 2]);
          accE[r % 2] = mfma1_all<r / 4>(ts[r % 4], Ae[r], r < 2 ? zero4 : accE[r % 2]);
        });
        const f32x4 th1 = quad_transpose(hidden4<RELU>(acc1[0] + acc1[1]), xp0, xp1);
        f32x4 th2 = th1;          // one hidden layer: layer 1 is the last
        if constexpr (TWO) {
          // ---- layer 2, this wavefront's K slice: partial sums of all 256 units ----
          f32x4 acc2[4][2];
          static_for<0, 64>([&](auto kc) {
            constexpr int kk = decltype(kc)::value;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
              pin_agpr(W2k[tt][kk]);
              acc2[tt][kk % 2] = mfma1_all<kk / 4>(th1[kk % 4], W2k[tt][kk], kk < 2 ? zero4 : acc2[tt][kk % 2]);
            }
          });
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) *reinterpret_cast<f32x4*>(p2s + ((w * NHP + 64 * tt + lane) * NCN)) = acc2[tt][0] + acc2[tt][1];
          __syncthreads();
          f32x4 v2 = f32x4{b2u, b2u, b2u, b2u};
#pragma unroll
          for (int ww = 0; ww < 4; ++ww) v2 += *reinterpret_cast<const f32x4*>(p2s + ((ww * NHP + unit) * NCN));
          th2 = quad_transpose(hidden4<RELU>(v2), xp0, xp1);
        }
        // ---- action layer, K slice of this wavefront: four K values per instruction ----
        f32x4 acc3p[4];
        static_for<0, 16>([&](auto rc) {
          constexpr int r = decltype(rc)::value;
          acc3p[r % 4] = mfma1_group<r / 4>(th2[r % 4], W3k[r], r < 4 ? zero4 : acc3p[r % 4]);
        });
        f32x4 acc3 = (acc3p[0] + acc3p[1]) + (acc3p[2] + acc3p[3]);
        acc3 = f32x4{rows_sum(acc3.x), rows_sum(acc3.y), rows_sum(acc3.z), rows_sum(acc3.w)};      // over the four groups
        if (lane < 16) {                       // lane = action row; register = copy
#pragma unroll
          for (int c = 0; c < NCN; ++c) p3s[(w * NCN + c) * 16 + lane] = acc3[c];
        }
        __syncthreads();
        // ---- the action, transposed (blocks 0..3: rows 4 blk .. 4 blk + 3 of copy x); reward; environment step ----
        f32x4 ta = f32x4{0.f, 0.f, 0.f, 0.f};
        if (blk < 4) {
          f32x4 v = b3q;
#pragma unroll
          for (int ww = 0; ww < 4; ++ww) v += *reinterpret_cast<const f32x4*>(p3s + (ww * NCN + x) * 16 + 4 * blk);
          const f32x4 tv = tanh4(v);
          const bool squash = a.out_tanh != 0u;
          ta = f32x4{squash ? tv.x : v.x, squash ? tv.y : v.y, squash ? tv.z : v.z, squash ? tv.w : v.w};
        }
        static_for<0, 16>([&](auto rc) {
          constexpr int r = decltype(rc)::value;
          accE[r % 4] = mfma1_all<r / 4>(ta[r % 4], Be[r], (r % 4 >= 2 && r < 4) ? zero4 : accE[r % 4]);
        });
        {
          float part = ta.x * ta.x;
          part = __fmaf_rn(ta.y, ta.y, part); part = __fmaf_rn(ta.z, ta.z, part); part = __fmaf_rn(ta.w, ta.w, part);
          const float aa = blocks_sum(part);           // |a_t|^2 of copy x (rows past the action width are exactly zero)
          const float r = __fmaf_rn(-ss_cur, inv_no, 1.0f) - a.act_cost * aa;
          Rn += alive ? r : 0.0f;
          Ln += alive ? 1 : 0;
        }
        ts = quad_transpose(tanh4((accE[0] + accE[1]) + (accE[2] + accE[3])), xp0, xp1);      // s_{t+1}; rows past the observation width stay exactly zero
        {
          float part = ts.x * ts.x;
          part = __fmaf_rn(ts.y, ts.y, part); part = __fmaf_rn(ts.z, ts.z, part); part = __fmaf_rn(ts.w, ts.w, part);
          ss_cur = blocks_sum(part);
          const unsigned mxb = blocks_umax(umax(umax(abs_bits(ts.x), abs_bits(ts.y)), umax(abs_bits(ts.z), abs_bits(ts.w))));
          alive = alive && !(__builtin_bit_cast(float, mxb) > a.done_thresh);
        }
      }
      // ---- outputs of this block of copies ----
      if (w == 0) {
        const uint32_t cnt = min((uint32_t)NCN, a.E - cb * (uint32_t)NCN);
        if (blk == 0 && (uint32_t)x < cnt) {
          a.returns[(size_t)i * a.E + e] = Rn;
          a.ep_len[(size_t)i * a.E + e] = Ln;
        }
        for (uint32_t r = 0; r < cnt; ++r) fit_sum += __shfl(Rn, (int)r, 64);
      }
    }
    if (tid == 0) a.fitness[i] = fit_sum / (float)a.E;
  }
}

template <int KO, bool RELU, bool NORM, bool TWO>
int launch_narrow_one(es_ctx* ctx, const F32Args& a, hipStream_t st) {
  const void* fn = reinterpret_cast<const void*>(rollout_mfma_f32_narrow_kernel<KO, RELU, NORM, TWO>);
  hipError_t err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LdsN<KO>::BYTES);
  if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(err));
  const uint32_t grid = std::min<uint32_t>(a.N, (uint32_t)std::max(1, ctx->num_cus));      // persistent: one workgroup per CU
  hipLaunchKernelGGL((rollout_mfma_f32_narrow_kernel<KO, RELU, NORM, TWO>), dim3(grid), dim3(256), LdsN<KO>::BYTES, st, a);
  return check_launch(ctx, "es_rollout (fp32 MFMA, four copies)");
}
template <int KO, bool TWO>
int launch_narrow_depth(es_ctx* ctx, const F32Args& a, hipStream_t st) {
  const bool relu = ctx->cfg.hidden_act == 1, norm = ctx->obs_mean != nullptr;
  if (relu) return norm ? launch_narrow_one<KO, true, true, TWO>(ctx, a, st) : launch_narrow_one<KO, true, false, TWO>(ctx, a, st);
  return norm ? launch_narrow_one<KO, false, true, TWO>(ctx, a, st) : launch_narrow_one<KO, false, false, TWO>(ctx, a, st);
}
template <int KO>
int launch_narrow(es_ctx* ctx, const F32Args& a, hipStream_t st) {
  return ctx->shp.m == 1 ? launch_narrow_depth<KO, false>(ctx, a, st) : launch_narrow_depth<KO, true>(ctx, a, st);
}

template <int KPL, bool RELU, bool NORM>
int launch_one(es_ctx* ctx, const F32Args& a, hipStream_t st) {
  const void* fn = reinterpret_cast<const void*>(rollout_mfma_f32_kernel<KPL, RELU, NORM>);
  hipError_t err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, Lds<KPL>::BYTES);
  if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(err));
  const uint32_t grid = std::min<uint32_t>(a.N, (uint32_t)std::max(1, ctx->num_cus));      // persistent: one workgroup per CU
  hipLaunchKernelGGL((rollout_mfma_f32_kernel<KPL, RELU, NORM>), dim3(grid), dim3(256), Lds<KPL>::BYTES, st, a);
  return check_launch(ctx, "es_rollout (fp32 MFMA)");
}
template <int KPL>
int launch_kpl(es_ctx* ctx, const F32Args& a, hipStream_t st) {
  const bool relu = ctx->cfg.hidden_act == 1, norm = ctx->obs_mean != nullptr;
  if (relu) return norm ? launch_one<KPL, true, true>(ctx, a, st) : launch_one<KPL, true, false>(ctx, a, st);
  return norm ? launch_one<KPL, false, true>(ctx, a, st) : launch_one<KPL, false, false>(ctx, a, st);
}

}  // namespace

// Binary32 policies with 65..256 hidden units, one or two hidden layers, obs <= 64, act <= 16.
bool mfma_f32_fits(const es_config& c) {
  const uint32_t m = c.num_hidden ? c.num_hidden : 2;
  return c.dtype == 0 && (m == 1 || m == 2) && c.hid_dim > 64 && c.hid_dim <= (uint32_t)NHP && c.obs_dim <= 64 && c.act_dim <= 16;
}

// up to eight copies per individual: two passes of the four-copy kernel cost less than one pass of sixteen columns;
// a single hidden layer is served by the four-copy kernel whatever the number of copies
static bool narrow_pays(const es_config& c, uint32_t copies) { return copies <= 2u * (uint32_t)NCN || c.num_hidden == 1; }

const char* mfma_f32_variant_name(const es_config& c, uint32_t copies) {
  if (c.num_hidden == 1)
    return c.obs_dim <= 16 ? "rollout_mfma_reg_f32<obs16,hid256,act16,copies4>,depth1"
         : c.obs_dim <= 32 ? "rollout_mfma_reg_f32<obs32,hid256,act16,copies4>,depth1" : "rollout_mfma_reg_f32<obs64,hid256,act16,copies4>,depth1";
  if (narrow_pays(c, copies))
    return c.obs_dim <= 16 ? "rollout_mfma_reg_f32<obs16,hid256,act16,copies4>"
         : c.obs_dim <= 32 ? "rollout_mfma_reg_f32<obs32,hid256,act16,copies4>" : "rollout_mfma_reg_f32<obs64,hid256,act16,copies4>";
  return c.obs_dim <= 32 ? "rollout_mfma_reg_f32<obs32,hid256,act16>" : "rollout_mfma_reg_f32<obs64,hid256,act16>";
}

int launch_rollout_mfma_f32(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise, const float* A,
                            const float* B, float* returns, int32_t* ep_len, float* fitness, void* /*ws*/,
                            hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  if (!mfma_f32_fits(c)) return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no binary32 matrix-core variant for this shape");
  F32Args a;
  const NoiseView nv = noise_view(ctx, noise);
  a.theta = theta; a.noise = nv.base; a.noise_offs = nv.offs; a.A = A; a.B = B; a.obs_mean = ctx->obs_mean; a.obs_inv = ctx->obs_inv_std;
  a.returns = returns; a.ep_len = ep_len; a.fitness = fitness;
  a.N = s.N; a.E = s.E; a.T = s.T; a.no = s.no; a.nh = s.nh; a.na = s.na; a.ld = s.ld;
  a.oW1 = s.oW1; a.ob1 = s.ob1; a.oW2 = s.oW2; a.ob2 = s.ob2; a.oW3 = s.oW3; a.ob3 = s.ob3;
  a.gen = gen; a.k0 = (uint32_t)c.seed; a.k1 = (uint32_t)(c.seed >> 32);
  a.antithetic = c.antithetic; a.out_tanh = c.out_tanh; a.noise_mode = nv.mode;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  if (narrow_pays(c, s.E)) {
    if (s.no <= 16) return launch_narrow<16>(ctx, a, st);
    return s.no <= 32 ? launch_narrow<32>(ctx, a, st) : launch_narrow<64>(ctx, a, st);
  }
  return s.no <= 32 ? launch_kpl<8>(ctx, a, st) : launch_kpl<16>(ctx, a, st);
}

}  // namespace es
