// es_rollout, register-resident MFMA variant for bf16 policies with a wide hidden layer.
//
// Paper Sec. 3.3 (population x environment-copy evaluation) and Sec. 5.1/5.2 (two hidden
// layers of 256 units, fitness = mean undiscounted return).  One workgroup of four
// wavefronts evaluates one individual at a time on up to 16 environment copies per pass:
//
//   * The individual's perturbed bf16 weights never touch HBM: theta + sign*sigma*eps is
//     computed while staging, and the result is parked in the VGPR/AGPR file as MFMA
//     A-operands (16x16x32 bf16 tiles) for all T steps.  A 256-wide policy is 130-270 KB in
//     bf16, more than the 160 KB of LDS, but fits the 512 KB register file of a CU.  The
//     environment matrices A and B (shared by all individuals) are register-resident too.
//   * Each wavefront owns 64 output units (four 16-row tiles) of every wide layer; the
//     environment copies are the 16 columns of the MFMA.  Activations travel between
//     wavefronts as bf16 through LDS ([column][unit], padded pitch, 16-byte reads).
//   * The 256 -> act layer is split along K over the four wavefronts and summed in a fixed
//     order; reward norms and the termination test are shuffle + LDS reductions in a
//     fixed order, so reruns are bit-identical.
//   * The grid is persistent: workgroup b handles noise rows b, b + grid, ...; the two
//     mirrored individuals of a row run back to back.
// Bound: MFMA issue (dense 16x16x32 bf16) plus the tanh epilogue on the vector ALU.
#include "es_device.hpp"
#include "es_internal.hpp"

namespace es {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct MfmaArgs {
  const float* theta;
  const void* noise;
  const float* A;
  const float* B;
  float* returns;
  int32_t* ep_len;
  float* fitness;
  uint32_t N, E, T, no, nh, na, ld;
  uint32_t oW1, ob1, oW2, ob2, oW3, ob3;
  uint32_t gen, k0, k1;
  uint32_t antithetic, out_tanh, noise_bf16;
  float sigma, done_thresh, act_cost;
};

constexpr int NHP = 256;          // padded hidden width handled by this kernel
constexpr int MT_H = NHP / 64;    // 16-row tiles of a wide layer per wavefront
constexpr int KT_H = NHP / 32;    // 32-deep K tiles over the hidden width
constexpr int KS3 = KT_H / 4;     // K tiles of the action layer per wavefront
constexpr int PH = NHP + 8;       // LDS pitch (bf16 elements) of a hidden activation row

#ifndef ES_V256_KTAR
#define ES_V256_KTAR 4
#endif

constexpr int KC = 2;             // K tiles staged per round
constexpr int PW = 32 * KC + 8;   // LDS pitch of the staging window

template <int KT1_, int MT3_, int MTE_, int KTAR_, int NC_>
struct Variant {
  static constexpr int NC = NC_;              // environment copies per pass: 16, or 4 with column compaction
  static constexpr int KT1 = KT1_;            // K tiles over the (padded) observation width
  static constexpr int MT3 = MT3_;            // 16-row tiles of the action layer
  static constexpr int MTE = MTE_;            // 16-row tiles of the next-state vector per wavefront
  static constexpr int KTAR = KTAR_;          // K tiles of the env matrix A held in registers ...
  static constexpr int KTAL = KT1 - KTAR;     // ... and in LDS (when the register file is full)
  static constexpr int KTA = (16 * MT3 + 31) / 32;   // K tiles over the (padded) action width
  static constexpr int NOP = 32 * KT1;        // padded observation width
  static constexpr int NAP = 32 * KTA;        // padded action width as a K dimension
  static constexpr int PX = NOP + 8;          // LDS pitch of a state row
  static constexpr int PA = NAP + 8;          // LDS pitch of an action row
  static constexpr int PAL = 32 * KTAL + 8;   // LDS pitch of the LDS-resident part of A
  // LDS map (bytes).  [0, REGION0) is the staging window, aliased by the rollout buffers.
  static constexpr int OFF_X = 0;
  static constexpr int OFF_H1 = OFF_X + 2 * NC * PX;
  static constexpr int OFF_H2 = OFF_H1 + 2 * NC * PH;
  static constexpr int OFF_QA = OFF_H2 + 2 * NC * PH;
  static constexpr int OFF_P3 = OFF_QA + 2 * NC * PA;
  static constexpr int OFF_RED = OFF_P3 + 4 * MT3 * 64 * 16;
  static constexpr int ROLL_END = OFF_RED + 4 * 16 * 8;
  static constexpr int WIN_BYTES = 2 * 256 * PW;
  static constexpr int REGION0 = ROLL_END > WIN_BYTES ? ROLL_END : WIN_BYTES;
  static constexpr int OFF_AL = REGION0;
  static constexpr int OFF_B1 = OFF_AL + (KTAL ? 2 * 64 * MTE * PAL : 0);
  static constexpr int OFF_B2 = OFF_B1 + 4 * NHP;
  static constexpr int OFF_B3 = OFF_B2 + 4 * NHP;
  static constexpr int OFF_X0 = OFF_B3 + 4 * 16 * MT3;
  static constexpr int OFF_SS0 = OFF_X0 + 2 * NC * PX;
  static constexpr int LDS_BYTES = OFF_SS0 + 4 * 16;
  static_assert(2 * 16 * MT3 * PH <= WIN_BYTES, "the action layer is staged in one piece");
  static_assert(64 * MTE >= NOP, "the four wavefronts must cover the padded state");
  static_assert(64 * MTE <= 256, "staging window rows");
  static_assert(NAP >= 16 * MT3 && KTA <= KC, "action K padding");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
  static_assert(NC == 4 || NC == 16, "columns per pass");
  static_assert(4 * MT3 * 64 * 16 >= 4 * 256, "scratch for the initial-state norms");
};

__device__ __forceinline__ bf16x8 lds_tile(const unsigned char* base, int byte_off) {
  const u32x4 raw = *reinterpret_cast<const u32x4*>(base + byte_off);
  return __builtin_bit_cast(bf16x8, raw);
}

// Keeps a weight tile in the accumulation-register half of the unified register file: an
// empty asm that "updates" the tile in place pins its register class right at the use, so
// the MFMA reads its A operand from there directly instead of through copies.
__device__ __forceinline__ void pin_agpr(bf16x8& v) { asm volatile("" : "+a"(v)); }
// ... and accumulators in the architectural half, where the epilogue's vector ALU work reads them.
__device__ __forceinline__ void pin_vgpr(f32x4& v) { asm volatile("" : "+v"(v)); }

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Four binary32 values -> four bf16 (round to nearest even), by the packed hardware convert.
__device__ __forceinline__ u32x2 pack_bf16x4(float a, float b, float c, float d) {
  u32x2 r;
  r.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
  r.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{c, d}, bf16x2));
  return r;
}

__device__ __forceinline__ f32x4 tanh4(f32x4 v) {
  return f32x4{tanh_fast(v.x), tanh_fast(v.y), tanh_fast(v.z), tanh_fast(v.w)};
}

// Column compaction for passes of 4 environment copies: the MFMA result tile has 16 columns
// of which only 0..3 are real.  Lanes of bank q (columns 4q..4q+3) fetch tile q's values of
// columns 0..3 with a row shift, so that the tanh epilogue runs once per lane, not once per tile.
template <int CTRL, int BANK>
__device__ __forceinline__ float dpp_take(float keep, float from) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, keep), __builtin_bit_cast(int, from),
                                                                CTRL, 0xF, BANK, false));
}
template <int NT>
__device__ __forceinline__ f32x4 compact4(const f32x4 (&t)[NT]) {
  f32x4 v = t[0];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    if (NT > 1) v[r] = dpp_take<0x114, 0x2>(v[r], t[NT > 1 ? 1 : 0][r]);   // row_shr:4  -> columns 4..7
    if (NT > 2) v[r] = dpp_take<0x118, 0x4>(v[r], t[NT > 2 ? 2 : 0][r]);   // row_shr:8  -> columns 8..11
    if (NT > 3) v[r] = dpp_take<0x11C, 0x8>(v[r], t[NT > 3 ? 3 : 0][r]);   // row_shr:12 -> columns 12..15
  }
  return v;
}

// Fill dst[r * pitch + c] (bf16) for r < rows_p, c < COLS with the bf16-rounded source value of
// matrix element (r, kbase + c) when r < rows and kbase + c < cols, and zero elsewhere.
// PERTURB: value = fma(scale, noise[idx], theta[idx]) with idx = off + r * cols + (kbase + c).
template <int COLS, bool PERTURB>
__device__ __forceinline__ void stage_cols(uint16_t* dst, int pitch, int rows_p, int rows, int cols, int kbase,
                                           const float* __restrict__ src, const void* __restrict__ noise_row,
                                           bool noise_bf16, float scale, uint32_t off) {
  const int total = rows_p * COLS;
  for (int q = threadIdx.x; q < total; q += 256) {
    const int r = q / COLS, k = kbase + q % COLS;
    float v = 0.0f;
    if (r < rows && k < cols) {
      const uint32_t idx = off + (uint32_t)r * (uint32_t)cols + (uint32_t)k;
      v = src[idx];
      if (PERTURB) {
        const float eps = noise_bf16 ? bf16_to_f32(static_cast<const uint16_t*>(noise_row)[idx])
                                     : static_cast<const float*>(noise_row)[idx];
        v = __fmaf_rn(scale, eps, v);
      }
    }
    dst[r * pitch + (q % COLS)] = (uint16_t)bf16_bits(v);
  }
}

template <class V>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void rollout_mfma_kernel(const MfmaArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int KT1 = V::KT1, MT3 = V::MT3, MTE = V::MTE, KTA = V::KTA, PX = V::PX, PA = V::PA;
  constexpr bool ENV_ALL = (64 * MTE == V::NOP);   // every wavefront's next-state tiles are inside the padded state
  constexpr int NC = V::NC;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront index, known uniform
  const int g = lane >> 4, n = lane & 15;
  const int col = n & (NC - 1);      // environment copy (column) this lane reads and keeps books for
  const int q = n >> 2;              // NC == 4: which tile this lane finishes after compaction
  uint16_t* stage = reinterpret_cast<uint16_t*>(lds);
  float* b1s = reinterpret_cast<float*>(lds + V::OFF_B1);
  float* b2s = reinterpret_cast<float*>(lds + V::OFF_B2);
  float* b3s = reinterpret_cast<float*>(lds + V::OFF_B3);
  uint16_t* x0s = reinterpret_cast<uint16_t*>(lds + V::OFF_X0);
  float* ss0s = reinterpret_cast<float*>(lds + V::OFF_SS0);
  const int no = (int)a.no, nh = (int)a.nh, na = (int)a.na;

  // ---------------- environment matrices -> registers / LDS (once per workgroup) ----------------
  constexpr int KTAR = V::KTAR, KTAL = V::KTAL, PAL = V::PAL;
  bf16x8 Ar[MTE][KTAR > 0 ? KTAR : 1], Br[MTE][KTA];
#pragma unroll
  for (int kr = 0; kr < (KTAR + KC - 1) / KC; ++kr) {
    stage_cols<32 * KC, false>(stage, PW, 64 * MTE, no, no, 32 * KC * kr, a.A, nullptr, false, 0.0f, 0u);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < MTE; ++t)
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
        if (kr * KC + kk < KTAR)
          Ar[t][kr * KC + kk] = lds_tile(lds, 2 * ((16 * (w * MTE + t) + n) * PW + 32 * kk + 8 * g));
    __syncthreads();
  }
  if (KTAL > 0)
    stage_cols<32 * (KTAL > 0 ? KTAL : 1), false>(reinterpret_cast<uint16_t*>(lds + V::OFF_AL), PAL, 64 * MTE, no, no,
                                                    32 * KTAR, a.A, nullptr, false, 0.0f, 0u);
  stage_cols<32 * KC, false>(stage, PW, 64 * MTE, no, na, 0, a.B, nullptr, false, 0.0f, 0u);
  __syncthreads();
#pragma unroll
  for (int t = 0; t < MTE; ++t)
#pragma unroll
    for (int kt = 0; kt < KTA; ++kt)
      Br[t][kt] = lds_tile(lds, 2 * ((16 * (w * MTE + t) + n) * PW + 32 * kt + 8 * g));
  __syncthreads();

  const uint32_t per_unit = a.antithetic ? 2u : 1u;
  const uint32_t units = a.N / per_unit;
  const uint32_t nblk = (a.E + (uint32_t)NC - 1u) / (uint32_t)NC;
  int x0_block = -1;

  for (uint32_t unit = blockIdx.x; unit < units; unit += gridDim.x) {
    for (uint32_t sub = 0; sub < per_unit; ++sub) {
      const uint32_t i = unit * per_unit + sub;
      const float scale = sub ? -a.sigma : a.sigma;
      const void* nrow = a.noise_bf16
                             ? static_cast<const void*>(static_cast<const uint16_t*>(a.noise) + (size_t)unit * a.ld)
                             : static_cast<const void*>(static_cast<const float*>(a.noise) + (size_t)unit * a.ld);

      // ---------------- perturbed policy weights -> registers ----------------
      bf16x8 W1r[MT_H][KT1], W2r[MT_H][KT_H], W3r[MT3][KS3];
      for (int u = tid; u < NHP; u += 256) {     // biases: perturbed, bf16-rounded, kept as binary32
        float v1 = 0.0f, v2 = 0.0f;
        if (u < nh) {
          const uint32_t i1 = a.ob1 + u, i2 = a.ob2 + u;
          const float e1 = a.noise_bf16 ? bf16_to_f32(static_cast<const uint16_t*>(nrow)[i1]) : static_cast<const float*>(nrow)[i1];
          const float e2 = a.noise_bf16 ? bf16_to_f32(static_cast<const uint16_t*>(nrow)[i2]) : static_cast<const float*>(nrow)[i2];
          v1 = bf16_round(__fmaf_rn(scale, e1, a.theta[i1]));
          v2 = bf16_round(__fmaf_rn(scale, e2, a.theta[i2]));
        }
        b1s[u] = v1;
        b2s[u] = v2;
      }
      for (int c = tid; c < 16 * MT3; c += 256) {
        float v3 = 0.0f;
        if (c < na) {
          const uint32_t i3 = a.ob3 + c;
          const float e3 = a.noise_bf16 ? bf16_to_f32(static_cast<const uint16_t*>(nrow)[i3]) : static_cast<const float*>(nrow)[i3];
          v3 = bf16_round(__fmaf_rn(scale, e3, a.theta[i3]));
        }
        b3s[c] = v3;
      }
#pragma unroll
      for (int kr = 0; kr < (KT1 + KC - 1) / KC; ++kr) {
        stage_cols<32 * KC, true>(stage, PW, NHP, nh, no, 32 * KC * kr, a.theta, nrow, a.noise_bf16, scale, a.oW1);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < MT_H; ++t)
#pragma unroll
          for (int kk = 0; kk < KC; ++kk)
            if (kr * KC + kk < KT1)
              W1r[t][kr * KC + kk] = lds_tile(lds, 2 * ((16 * (w * MT_H + t) + n) * PW + 32 * kk + 8 * g));
        __syncthreads();
      }
#pragma unroll
      for (int kr = 0; kr < KT_H / KC; ++kr) {
        stage_cols<32 * KC, true>(stage, PW, NHP, nh, nh, 32 * KC * kr, a.theta, nrow, a.noise_bf16, scale, a.oW2);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < MT_H; ++t)
#pragma unroll
          for (int kk = 0; kk < KC; ++kk)
            W2r[t][kr * KC + kk] = lds_tile(lds, 2 * ((16 * (w * MT_H + t) + n) * PW + 32 * kk + 8 * g));
        __syncthreads();
      }
      stage_cols<NHP, true>(stage, PH, 16 * MT3, na, nh, 0, a.theta, nrow, a.noise_bf16, scale, a.oW3);
      __syncthreads();
#pragma unroll
      for (int mt = 0; mt < MT3; ++mt)
#pragma unroll
        for (int kk = 0; kk < KS3; ++kk)
          W3r[mt][kk] = lds_tile(lds, 2 * ((16 * mt + n) * PH + 32 * (w * KS3 + kk) + 8 * g));
      __syncthreads();

      float fit_sum = 0.0f;
      for (uint32_t cb = 0; cb < nblk; ++cb) {
        // ---------------- initial states of this block of environment copies ----------------
        if (x0_block != (int)cb) {
          // thread -> (column n0, row group kq): s0[k] for k = kq, kq + 16, ...
          constexpr int KG = 256 / NC;               // row groups
          const int n0 = tid % NC, kq = tid / NC;
          const uint32_t e0 = cb * (uint32_t)NC + (uint32_t)n0;
          float part = 0.0f;
          for (int k = kq; k < V::NOP; k += KG) {
            float v = 0.0f;
            if (k < no && e0 < a.E) v = reset_value((uint32_t)k, e0, a.gen, a.k0, a.k1);
            part = __fmaf_rn(v, v, part);
            x0s[n0 * PX + k] = (uint16_t)bf16_bits(v);
          }
          float* scratch = reinterpret_cast<float*>(lds + V::OFF_P3);   // KG x NC partial norms
          scratch[kq * NC + n0] = part;
          __syncthreads();
          if (tid < NC) {
            float s = 0.0f;
            for (int r = 0; r < KG; ++r) s += scratch[r * NC + tid];
            ss0s[tid] = s;
          }
          x0_block = (int)cb;
          __syncthreads();
        }
        {
          // copy the cached initial state into the working buffer; clear the action buffer
          const uint32_t* src = reinterpret_cast<const uint32_t*>(x0s);
          uint32_t* dst = reinterpret_cast<uint32_t*>(lds + V::OFF_X);
          for (int r = tid; r < NC * PX / 2; r += 256) dst[r] = src[r];
          uint32_t* qz = reinterpret_cast<uint32_t*>(lds + V::OFF_QA);
          for (int r = tid; r < NC * PA / 2; r += 256) qz[r] = 0u;
        }
        __syncthreads();

        const uint32_t e = cb * (uint32_t)NC + (uint32_t)col;
        bool alive = e < a.E;
        float Rn = 0.0f, ssn = ss0s[col];
        int32_t Ln = 0;

        for (uint32_t t = 0; t < a.T; ++t) {
          // ---- phase 1: h1 = tanh(W1 x + b1); start s' = A x ----
          f32x4 acc[MT_H], accE[MTE];
#pragma unroll
          for (int tt = 0; tt < MT_H; ++tt) { acc[tt] = *reinterpret_cast<const f32x4*>(b1s + 16 * (w * MT_H + tt) + 4 * g); pin_vgpr(acc[tt]); }
#pragma unroll
          for (int tt = 0; tt < MTE; ++tt) { accE[tt] = f32x4{0.f, 0.f, 0.f, 0.f}; pin_vgpr(accE[tt]); }
#pragma unroll
          for (int kt = 0; kt < KT1; ++kt) {
            const bf16x8 b = lds_tile(lds, V::OFF_X + 2 * (col * PX + 32 * kt + 8 * g));
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) { pin_agpr(W1r[tt][kt]); acc[tt] = mfma16(W1r[tt][kt], b, acc[tt]); }
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt)
              if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
                if (kt < KTAR) accE[tt] = mfma16(Ar[tt][kt], b, accE[tt]);
                else accE[tt] = mfma16(lds_tile(lds, V::OFF_AL + 2 * ((16 * (w * MTE + tt) + n) * PAL + 32 * (kt - KTAR) + 8 * g)), b, accE[tt]);
              }
          }
          if (NC == 4) {
            const f32x4 h = tanh4(compact4<MT_H>(acc));
            *reinterpret_cast<u32x2*>(lds + V::OFF_H1 + 2 * (col * PH + 16 * (w * MT_H + q) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
          } else {
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) {
              const f32x4 h = tanh4(acc[tt]);
              *reinterpret_cast<u32x2*>(lds + V::OFF_H1 + 2 * (n * PH + 16 * (w * MT_H + tt) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
            }
          }
          __syncthreads();
          // ---- phase 2: h2 = tanh(W2 h1 + b2) ----
#pragma unroll
          for (int tt = 0; tt < MT_H; ++tt) { acc[tt] = *reinterpret_cast<const f32x4*>(b2s + 16 * (w * MT_H + tt) + 4 * g); pin_vgpr(acc[tt]); }
#pragma unroll
          for (int kt = 0; kt < KT_H; ++kt) {
            const bf16x8 b = lds_tile(lds, V::OFF_H1 + 2 * (col * PH + 32 * kt + 8 * g));
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) { pin_agpr(W2r[tt][kt]); acc[tt] = mfma16(W2r[tt][kt], b, acc[tt]); }
          }
          if (NC == 4) {
            const f32x4 h = tanh4(compact4<MT_H>(acc));
            *reinterpret_cast<u32x2*>(lds + V::OFF_H2 + 2 * (col * PH + 16 * (w * MT_H + q) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
          } else {
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) {
              const f32x4 h = tanh4(acc[tt]);
              *reinterpret_cast<u32x2*>(lds + V::OFF_H2 + 2 * (n * PH + 16 * (w * MT_H + tt) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
            }
          }
          __syncthreads();
          // ---- phase 3: this wavefront's K slice of W3 h2 ----
#pragma unroll
          for (int mt = 0; mt < MT3; ++mt) {
            f32x4 p = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KS3; ++kk) {
              const bf16x8 b = lds_tile(lds, V::OFF_H2 + 2 * (col * PH + 32 * (w * KS3 + kk) + 8 * g));
              p = mfma16(W3r[mt][kk], b, p);
            }
            *reinterpret_cast<f32x4*>(lds + V::OFF_P3 + 16 * ((w * MT3 + mt) * 64 + lane)) = p;
          }
          __syncthreads();
          // ---- phase 4: action (every wavefront, identically), reward, return ----
          float aa = 0.0f;
          if (NC == 4) {
            // lane (g, 4q + c) finishes action tile q of column c: its partials sit at lane 16g + c
            const int mt = q & (MT3 - 1), src = 16 * g + col;
            const bool valid = q < MT3;
            const f32x4 p0 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((0 * MT3 + mt) * 64 + src));
            const f32x4 p1 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((1 * MT3 + mt) * 64 + src));
            const f32x4 p2 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((2 * MT3 + mt) * 64 + src));
            const f32x4 p3 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((3 * MT3 + mt) * 64 + src));
            const f32x4 bb = *reinterpret_cast<const f32x4*>(b3s + 16 * mt + 4 * g);
            f32x4 v = (((p0 + p1) + p2) + p3) + bb;
            if (a.out_tanh) v = tanh4(v);
            aa = __fmaf_rn(v.x, v.x, aa); aa = __fmaf_rn(v.y, v.y, aa);
            aa = __fmaf_rn(v.z, v.z, aa); aa = __fmaf_rn(v.w, v.w, aa);
            aa = valid ? aa : 0.0f;
            if (w == 0 && valid) *reinterpret_cast<u32x2*>(lds + V::OFF_QA + 2 * (col * PA + 16 * mt + 4 * g)) = pack_bf16x4(v.x, v.y, v.z, v.w);
            aa += __shfl_xor(aa, 4, 64);
            aa += __shfl_xor(aa, 8, 64);
          } else {
#pragma unroll
            for (int mt = 0; mt < MT3; ++mt) {
              const f32x4 p0 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((0 * MT3 + mt) * 64 + lane));
              const f32x4 p1 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((1 * MT3 + mt) * 64 + lane));
              const f32x4 p2 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((2 * MT3 + mt) * 64 + lane));
              const f32x4 p3 = *reinterpret_cast<const f32x4*>(lds + V::OFF_P3 + 16 * ((3 * MT3 + mt) * 64 + lane));
              const f32x4 bb = *reinterpret_cast<const f32x4*>(b3s + 16 * mt + 4 * g);
              f32x4 v = (((p0 + p1) + p2) + p3) + bb;
              if (a.out_tanh) v = tanh4(v);
              aa = __fmaf_rn(v.x, v.x, aa); aa = __fmaf_rn(v.y, v.y, aa);
              aa = __fmaf_rn(v.z, v.z, aa); aa = __fmaf_rn(v.w, v.w, aa);
              if (w == 0) *reinterpret_cast<u32x2*>(lds + V::OFF_QA + 2 * (n * PA + 16 * mt + 4 * g)) = pack_bf16x4(v.x, v.y, v.z, v.w);
            }
          }
          aa += __shfl_xor(aa, 16, 64);
          aa += __shfl_xor(aa, 32, 64);
          if (alive) {
            Rn += (1.0f - ssn / (float)no) - a.act_cost * aa;
            Ln += 1;
          }
          __syncthreads();
          // ---- phase 5: s' = tanh(A x + B a); norms for the next reward and the termination test ----
          float ssp = 0.0f, mxp = 0.0f;
          if (NC == 4) {
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt)
#pragma unroll
              for (int kt = 0; kt < KTA; ++kt) {
                const bf16x8 b = lds_tile(lds, V::OFF_QA + 2 * (col * PA + 32 * kt + 8 * g));
                accE[tt] = mfma16(Br[tt][kt], b, accE[tt]);
              }
            const int tile = w * MTE + q;
            const bool valid = q < MTE && (ENV_ALL || 16 * tile < V::NOP);
            const f32x4 sn = tanh4(compact4<MTE>(accE));
            if (valid) {
              ssp = __fmaf_rn(sn.x, sn.x, ssp); ssp = __fmaf_rn(sn.y, sn.y, ssp);
              ssp = __fmaf_rn(sn.z, sn.z, ssp); ssp = __fmaf_rn(sn.w, sn.w, ssp);
              mxp = fmaxf(fmaxf(fabsf(sn.x), fabsf(sn.y)), fmaxf(fabsf(sn.z), fabsf(sn.w)));
              *reinterpret_cast<u32x2*>(lds + V::OFF_X + 2 * (col * PX + 16 * tile + 4 * g)) = pack_bf16x4(sn.x, sn.y, sn.z, sn.w);
            }
            ssp += __shfl_xor(ssp, 4, 64);
            ssp += __shfl_xor(ssp, 8, 64);
            mxp = fmaxf(mxp, __shfl_xor(mxp, 4, 64));
            mxp = fmaxf(mxp, __shfl_xor(mxp, 8, 64));
          } else {
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt) {
              if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
#pragma unroll
                for (int kt = 0; kt < KTA; ++kt) {
                  const bf16x8 b = lds_tile(lds, V::OFF_QA + 2 * (n * PA + 32 * kt + 8 * g));
                  accE[tt] = mfma16(Br[tt][kt], b, accE[tt]);
                }
                const f32x4 sn = tanh4(accE[tt]);
                ssp = __fmaf_rn(sn.x, sn.x, ssp); ssp = __fmaf_rn(sn.y, sn.y, ssp);
                ssp = __fmaf_rn(sn.z, sn.z, ssp); ssp = __fmaf_rn(sn.w, sn.w, ssp);
                mxp = fmaxf(fmaxf(mxp, fmaxf(fabsf(sn.x), fabsf(sn.y))), fmaxf(fabsf(sn.z), fabsf(sn.w)));
                *reinterpret_cast<u32x2*>(lds + V::OFF_X + 2 * (n * PX + 16 * (w * MTE + tt) + 4 * g)) = pack_bf16x4(sn.x, sn.y, sn.z, sn.w);
              }
            }
          }
          ssp += __shfl_xor(ssp, 16, 64);
          ssp += __shfl_xor(ssp, 32, 64);
          mxp = fmaxf(mxp, __shfl_xor(mxp, 16, 64));
          mxp = fmaxf(mxp, __shfl_xor(mxp, 32, 64));
          float* red = reinterpret_cast<float*>(lds + V::OFF_RED);
          if (g == 0 && n < NC) { red[(w * 16 + n) * 2] = ssp; red[(w * 16 + n) * 2 + 1] = mxp; }
          __syncthreads();
          // ---- phase 6: combine the four wavefronts in a fixed order; termination ----
          ssn = ((red[(0 * 16 + col) * 2] + red[(1 * 16 + col) * 2]) + red[(2 * 16 + col) * 2]) + red[(3 * 16 + col) * 2];
          const float mx = fmaxf(fmaxf(red[(0 * 16 + col) * 2 + 1], red[(1 * 16 + col) * 2 + 1]),
                                 fmaxf(red[(2 * 16 + col) * 2 + 1], red[(3 * 16 + col) * 2 + 1]));
          alive = alive && !(mx > a.done_thresh);
          if (__ballot(alive) == 0ull) break;       // identical in all four wavefronts
        }
        __syncthreads();   // all reads of the rollout buffers are done before anything is restaged

        // ---------------- outputs of this block of environment copies ----------------
        if (w == 0) {
          const uint32_t cnt = min((uint32_t)NC, a.E - cb * (uint32_t)NC);
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
}

template <int NC> using V32 = Variant<1, 1, 1, 1, NC>;     // obs <= 32,  act <= 16
template <int NC> using V64 = Variant<2, 1, 1, 2, NC>;     // obs <= 64,  act <= 16
template <int NC> using V128 = Variant<4, 2, 2, 4, NC>;    // obs <= 128, act <= 32
template <int NC> using V256 = Variant<8, 2, 4, ES_V256_KTAR, NC>;   // obs <= 256, act <= 32; part of A lives in LDS

struct VariantInfo { int max_obs, max_act; const char* name; };
static const VariantInfo kVariants[] = {
    {32, 16, "rollout_mfma_reg_bf16<obs32,hid256,act16>"},
    {64, 16, "rollout_mfma_reg_bf16<obs64,hid256,act16>"},
    {128, 32, "rollout_mfma_reg_bf16<obs128,hid256,act32>"},
    {256, 32, "rollout_mfma_reg_bf16<obs256,hid256,act32>"},
};

int mfma_variant_for(const es_config& c) {
  if (c.dtype != 1 || c.hid_dim > (uint32_t)NHP) return -1;
  // narrow policies are served better by the one-wavefront-per-episode kernel when it fits
  if (c.hid_dim < 128 && wave_rollout_lds_bytes(c) <= 160 * 1024) return -1;
  for (int v = 0; v < 4; ++v)
    if ((int)c.obs_dim <= kVariants[v].max_obs && (int)c.act_dim <= kVariants[v].max_act) return v;
  return -1;
}

const char* mfma_variant_name(int v) { return (v >= 0 && v < 4) ? kVariants[v].name : "none"; }

template <class V>
static int launch_variant(es_ctx* ctx, const MfmaArgs& a, uint32_t grid, hipStream_t st) {
  const void* fn = reinterpret_cast<const void*>(rollout_mfma_kernel<V>);
  hipError_t err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, V::LDS_BYTES);
  if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(err));
  hipLaunchKernelGGL(rollout_mfma_kernel<V>, dim3(grid), dim3(256), V::LDS_BYTES, st, a);
  return check_launch(ctx, "es_rollout (MFMA)");
}

int launch_rollout_mfma(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise, const float* A,
                        const float* B, float* returns, int32_t* ep_len, float* fitness, void* /*ws*/,
                        hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  MfmaArgs a;
  a.theta = theta; a.noise = noise; a.A = A; a.B = B; a.returns = returns; a.ep_len = ep_len; a.fitness = fitness;
  a.N = s.N; a.E = s.E; a.T = s.T; a.no = s.no; a.nh = s.nh; a.na = s.na; a.ld = s.ld;
  a.oW1 = s.oW1; a.ob1 = s.ob1; a.oW2 = s.oW2; a.ob2 = s.ob2; a.oW3 = s.oW3; a.ob3 = s.ob3;
  a.gen = gen; a.k0 = (uint32_t)c.seed; a.k1 = (uint32_t)(c.seed >> 32);
  a.antithetic = c.antithetic; a.out_tanh = c.out_tanh; a.noise_bf16 = c.noise_dtype == 1;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  if ((int)V256<16>::LDS_BYTES > ctx->lds_limit)
    return fail(ctx, ES_EUNSUPPORTED, "es_rollout: this device's LDS is too small for the register-resident kernel");
  const uint32_t units = c.antithetic ? s.N / 2 : s.N;
  const uint32_t grid = std::min<uint32_t>(units, (uint32_t)std::max(1, ctx->num_cus));
  const bool narrow = s.E <= 4;     // passes of 4 environment copies with column compaction
  switch (ctx->mfma_variant) {
    case 0: return narrow ? launch_variant<V32<4>>(ctx, a, grid, st) : launch_variant<V32<16>>(ctx, a, grid, st);
    case 1: return narrow ? launch_variant<V64<4>>(ctx, a, grid, st) : launch_variant<V64<16>>(ctx, a, grid, st);
    case 2: return narrow ? launch_variant<V128<4>>(ctx, a, grid, st) : launch_variant<V128<16>>(ctx, a, grid, st);
    case 3: return narrow ? launch_variant<V256<4>>(ctx, a, grid, st) : launch_variant<V256<16>>(ctx, a, grid, st);
    default: return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident variant for this shape");
  }
}

}  // namespace es
