// es_rollout, register-resident MFMA variant for bf16 policies with a wide hidden layer.
//
// Paper Sec. 3.2 (population x environment-copy evaluation) and Sec. 5.1/5.2 (two hidden
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
//   * The narrow 256 -> act layer is split along K: any K order is as good as another as long
//     as both MFMA operands agree, so every wavefront multiplies the 64 units of the last
//     hidden layer it has just produced - still in its registers - with its slice of the
//     action-layer weights, and only the binary32 partial sums cross the LDS (passes of four
//     copies with two hidden layers, and every pass of sixteen copies; the remaining four-copy
//     variants exchange the last hidden layer and every wavefront computes the one action tile).
//     Reward norms and the termination test are reduced through per-wavefront LDS partials;
//     every lane adds partials in the same fixed order, so reruns are bit-identical.
//   * The grid is persistent: workgroup b handles individuals b, b + grid, ...
// Bound: the dependent chain of a step (MFMA streams, activation epilogues on the vector ALU,
// three LDS hand-overs) in one in-order wavefront per SIMD; two where the register file allows.
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
  const uint32_t* noise_offs;   // shared noise table: start of every row, else null
  const float* A;
  const float* B;
  const float* obs_mean;     // frozen observation statistics (paper App. B), or null
  const float* obs_inv;
  float* returns;
  int32_t* ep_len;
  float* fitness;
  uint32_t N, E, T, no, nh, na, ld;
  uint32_t oW1, ob1, oW2, ob2, oW3, ob3;
  uint32_t gen, k0, k1;
  uint32_t antithetic, out_tanh, noise_mode;
  float sigma, done_thresh, act_cost;
  unsigned long long* prof;     // phase-timing build only (ES_PHASE_PROF): cycle totals per wavefront and phase
};

// A kernel argument read afresh from the kernel-argument segment (the one by-value argument starts at its offset 0),
// through a pointer the compiler cannot see through.  The staging code takes its arguments this way once per
// individual: read from the by-value copy they would be loaded once and then held in scalar registers across the
// step loop, which already spills scalar registers to vector lanes and reloads them every step.
template <class T>
__device__ __forceinline__ T kernarg_field(size_t byte_off) {
  const __attribute__((address_space(4))) char* p =
      (const __attribute__((address_space(4))) char*)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(p));
  return *reinterpret_cast<const __attribute__((address_space(4))) T*>(p + byte_off);
}
#define KARG(field) kernarg_field<decltype(MfmaArgs::field)>(offsetof(MfmaArgs, field))

// Phase timing for tuning (compiled in with -DES_PHASE_PROF only): shader-clock cycles between consecutive stamps,
// summed over all steps of the individuals of workgroup 0, one row of 16 slots per wavefront.
#ifdef ES_PHASE_PROF
#define PSTAMP(k) do { const unsigned long long now_ = __builtin_readcyclecounter(); prof_acc[k] += now_ - prof_last; prof_last = now_; } while (0)
#else
#define PSTAMP(k) do {} while (0)
#endif

constexpr int NHP = 256;          // padded hidden width handled by this kernel
constexpr int KT_H = NHP / 32;    // 32-deep K tiles over the hidden width
constexpr int PH = NHP + 8;       // LDS pitch (bf16 elements) of a hidden activation row

constexpr int STAGE_BATCH = 8;    // staging iterations whose loads are in flight together (4: 24 % slower staging, 16: spills)
constexpr int KC = 2;             // K tiles staged per round
constexpr int PW = 32 * KC + 8;   // LDS pitch of the staging window

template <int KT1_, int MT3_, int MTE_, int KTAR_, int NC_, int NW_, int OCC_ = 1, int ME_ = 0, bool ENVF_ = false>
struct Variant {
  static constexpr bool ENVF = ENVF_;          // the environment's products A s + B a stay binary32 (fp32 16x16x4 MFMAs, its own
                                              // binary32 copy of the state in LDS); the policy keeps its bf16 operands
  static constexpr int ME = ME_;              // hidden layers beyond the second (depth m = 2 + ME), each 256 x 256 in registers;
                                              // -1: a single hidden layer (the second layer's phase is skipped)
  static constexpr int OCC = OCC_;            // workgroups per CU the register budget is sized for (1 or 2)
  static constexpr int NW = NW_;              // wavefronts per workgroup: one per SIMD
  static constexpr int NT = 64 * NW;          // threads per workgroup
  static constexpr int MT_H = NHP / (16 * NW);   // 16-row tiles of a wide layer per wavefront
  static constexpr int ENV_ROWS = 16 * NW * MTE_;   // padded rows of the next-state vector covered by the workgroup
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
  static constexpr int OFF_SSP = OFF_QA + NW * 2 * NC * PA; // (one action buffer per wavefront) |s'|^2 partials [column][wavefront]
  static constexpr int OFF_MXP = OFF_SSP + 4 * 16 * NW;     // max|s'| partials, same layout
  static constexpr int OFF_SCR = OFF_MXP + 4 * 16 * NW;     // scratch for the initial-state norms
  static constexpr int ROLL_END = OFF_SCR + 4 * NT;
  static constexpr int WIN_BYTES = 2 * 256 * PW;
  static constexpr int REGION0 = ROLL_END > WIN_BYTES ? ROLL_END : WIN_BYTES;
  static constexpr int OFF_AL = REGION0;
  static constexpr int OFF_W3 = OFF_AL + (KTAL ? 2 * ENV_ROWS * PAL : 0);   // action-layer weights [16*MT3][PH]
  static constexpr int OFF_B1 = OFF_W3 + 2 * 16 * MT3 * PH;
  static constexpr int OFF_B2 = OFF_B1 + 4 * NHP;
  static constexpr int OFF_B3 = OFF_B2 + 4 * NHP;
  static constexpr int OFF_X0 = OFF_B3 + 4 * 16 * MT3;
  static constexpr int OFF_SS0 = OFF_X0 + 2 * NC * PX;
  // only used with observation statistics: the normalised state (the policy's operand), its cached
  // initial value, and the statistics themselves
  static constexpr int OFF_BX = OFF_SS0 + 4 * 16;              // biases of the extra hidden layers [ME][NHP]
  static constexpr int OFF_HL = (ME & 1) ? OFF_H1 : OFF_H2;   // the last hidden layer's activations (the layers ping-pong)
  static constexpr int OFF_XP = OFF_BX + 4 * NHP * (ME > 0 ? ME : 0);
  static constexpr int OFF_X0P = OFF_XP + 2 * NC * PX;
  static constexpr int OFF_MU = OFF_X0P + 2 * NC * PX;
  static constexpr int OFF_IV = OFF_MU + 4 * NOP;
  // passes of four copies with the action layer split along K (FUSE3): the second state buffer (steps alternate)
  // and the binary32 partial sums of the action layer [wavefront][copy][32 action rows]
  static constexpr bool FUSE3 = NC_ == 4 && ME_ == 0 && NW_ == 4;
  static constexpr int OFF_X1 = OFF_IV + 4 * NOP;
  static constexpr int OFF_P3 = OFF_X1 + (FUSE3 ? 2 * NC * PX : 0);
  // binary32 environment: the state as binary32 [copy][state index] (pitch PXF floats: 16-byte reads of 16 lanes hit
  // distinct banks), working buffer and cached initial value
  static constexpr int KPL = NOP / 4;          // state elements per lane group of the fp32 MFMA's K dimension
  static constexpr int PXF = NOP + 4;
  // passes of sixteen copies (KSPLIT16): the same K split of the action layer, at any depth; every lane keeps its four tiles of
  // the last hidden layer for its own column, so they feed the MFMA with no lane exchange at all.
  // Partials [wavefront][copy][PP3 rows].
  static constexpr bool KSPLIT16 = NC_ == 16 && NW_ == 4;
  static constexpr int PP3 = 16 * MT3_ + 4;    // pitch (floats) of a copy's partial rows: 16-byte accesses of 16 lanes spread over the banks
  static constexpr int OFF_XF = OFF_P3 + (FUSE3 ? 4 * NW * NC * 32 : KSPLIT16 ? 4 * NW * 16 * PP3 : 0);
  static constexpr int OFF_X0F = OFF_XF + (ENVF ? 4 * NC * PXF : 0);
  // With all of A in registers the step loop has under a hundred working registers left: B and this wavefront's slice
  // of the action-layer weights then stay in LDS and are fetched where they are used (a dozen reads per step).
  static constexpr bool SMALL_LDS = FUSE3 && KTAR_ >= KT1_ && KT1_ >= 8;
  static constexpr int OFF_BL = OFF_X0F + (ENVF ? 4 * NC * PXF : 0);      // B [ENV_ROWS][PA] bf16
  static constexpr int LDS_BYTES = OFF_BL + (SMALL_LDS ? 2 * ENV_ROWS * PA : 0);
  static_assert(!ENVF || (NC == 16 && ME == 0 && MT3 == 1 && KT1 <= 2), "binary32 environment: passes of 16 copies, two hidden layers, obs <= 64, act <= 16");
  static_assert(ENV_ROWS >= NOP, "the wavefronts must cover the padded state");
  static_assert(ENV_ROWS <= 256, "staging window rows");
  static_assert(NW == 4, "one wavefront per SIMD (two per SIMD, each with half of the rows, measured slower at every shape)");
  static_assert(MT_H >= 1 && MT_H <= 4, "wide-layer tiles per wavefront");
  static_assert(NAP >= 16 * MT3 && KTA <= KC, "action K padding");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
  static_assert(NC == 4 || NC == 16, "columns per pass");
  static_assert(ME <= 0 || (OCC == 1 && KTAL == 0), "deeper policies need the whole register file of the CU");
  static_assert(ME >= 0 || KTAL == 0, "the single-layer variant keeps all of A in registers");
  static_assert(MT3 <= 2 && MT3 <= 4, "action tiles: one wavefront each, partial layout holds two");
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

// binary32 16x16x4: lane (g, n) supplies A[row n][k = g] and B[k = g][column n]
__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
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
// hidden-layer activation: tanh, or ReLU (the paper's EA experiments, App. B) - a compile-time choice,
// so that the MFMA / vector-ALU interleaving below stays one straight-line region
template <bool RELU>
__device__ __forceinline__ f32x4 hidden4(f32x4 v) {
  if (RELU) return f32x4{fmaxf(v.x, 0.f), fmaxf(v.y, 0.f), fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)};
  return tanh4(v);
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

__device__ __forceinline__ unsigned umax(unsigned a, unsigned b) { return a > b ? a : b; }

// Sum / max over the four banks of a 16-lane row (lanes c, c+4, c+8, c+12), result in lanes 0..3.
template <int CTRL>
__device__ __forceinline__ float dpp_shl(float v) {   // lane i <- lane i + n within the row, 0 past the end
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shl_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ float row_bank_sum(float v) {
  v = v + dpp_shl<0x104>(v);
  return v + dpp_shl<0x108>(v);
}
__device__ __forceinline__ unsigned row_bank_umax(unsigned v) {   // bit patterns of non-negative values
  v = umax(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0xF, true));
  return umax(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x108, 0xF, 0xF, true));
}

// Sum / max over the four 16-lane rows of the wavefront (lanes l, l+16, l+32, l+48), result in
// every row, by the row-swap instructions of gfx950 (vector ALU speed, no LDS round trip).
__device__ __forceinline__ float rows_sum(float v) {
  const unsigned b = __builtin_bit_cast(unsigned, v);
  const auto p = __builtin_amdgcn_permlane16_swap(b, b, false, false);     // (r0,r0,r2,r2) and (r1,r1,r3,r3)
  const float t = __builtin_bit_cast(float, (unsigned)p[0]) + __builtin_bit_cast(float, (unsigned)p[1]);
  const unsigned c = __builtin_bit_cast(unsigned, t);
  const auto r = __builtin_amdgcn_permlane32_swap(c, c, false, false);     // (lo,lo) and (hi,hi)
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
// max of non-negative binary32 values = max of their bit patterns as integers (no NaN canonicalisation needed)
__device__ __forceinline__ unsigned rows_umax(unsigned b) {
  const auto p = __builtin_amdgcn_permlane16_swap(b, b, false, false);
  const unsigned c = umax((unsigned)p[0], (unsigned)p[1]);
  const auto r = __builtin_amdgcn_permlane32_swap(c, c, false, false);
  return umax((unsigned)r[0], (unsigned)r[1]);
}
__device__ __forceinline__ unsigned abs_bits(float v) { return __builtin_bit_cast(unsigned, v) & 0x7FFFFFFFu; }

// One noise row under any storage mode: a pointer to the stored row, or the counters to recompute it.
struct NoiseRow {
  const void* ptr;
  uint32_t mode, row, gen, k0, k1;
};
__device__ __forceinline__ float row_noise(const NoiseRow& nz, uint32_t idx) {
  if (nz.mode >= 2u) return noise_regen1(nz.row, idx, nz.gen, nz.k0, nz.k1, nz.mode == 3u);
  return nz.mode == 1u ? bf16_to_f32(static_cast<const uint16_t*>(nz.ptr)[idx]) : static_cast<const float*>(nz.ptr)[idx];
}

// Four stored noise values as binary32: binary32 as they are, bf16 pairs widened (an int stands for "no noise").
__device__ __forceinline__ f32x4 widen4(f32x4 e) { return e; }
__device__ __forceinline__ f32x4 widen4(u32x2 raw) {
  return f32x4{__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u),
               __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xFFFF0000u)};
}
__device__ __forceinline__ f32x4 widen4(int) { return f32x4{0.f, 0.f, 0.f, 0.f}; }

// Fill dst[r * pitch + c] (bf16) for r < rows_p, c < COLS with the bf16-rounded source value of
// matrix element (r, kbase + c) when r < rows and kbase + c < cols, and zero elsewhere.
// PERTURB: value = fma(scale, noise[idx], theta[idx]) with idx = off + r * cols + (kbase + c).
template <int COLS, bool PERTURB>
__device__ __forceinline__ void stage_cols(uint16_t* dst, int pitch, int rows_p, int rows, int cols, int kbase,
                                           const float* __restrict__ src, const NoiseRow nz, float scale, uint32_t off) {
  if (((cols | (int)off | kbase) & 3) == 0) {
    // four consecutive columns per thread: 16-byte parameter loads, 8/16-byte noise loads, 8-byte LDS stores.
    // The loads of U iterations are issued together and unconditionally (a masked-out element reads the
    // matrix's first four entries instead, which are always there), and only then consumed: a load inside the
    // bounds test would be waited for in its own iteration, and the round would cost U memory latencies, not one.
    constexpr int C4 = COLS / 4;
    const int total = rows_p * C4;
    const int step = (int)blockDim.x;
    auto batch = [&](auto fetch) {
      constexpr int U = STAGE_BATCH;
      for (int q0 = threadIdx.x; q0 < total; q0 += U * step) {
        f32x4 tv[U];
        decltype(fetch(0u)) ev[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int q = q0 + u * step;
          const int r = q / C4, k = kbase + (q % C4) * 4;
          ok[u] = q < total && r < rows && k < cols;
          const uint32_t idx = ok[u] ? off + (uint32_t)r * (uint32_t)cols + (uint32_t)k : off;
          tv[u] = *reinterpret_cast<const f32x4*>(src + idx);
          ev[u] = fetch(idx);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int q = q0 + u * step;
          if (q < total) {
            const int r = q / C4, c = (q % C4) * 4;
            f32x4 v = tv[u];
            if (PERTURB) {
              const f32x4 e = widen4(ev[u]);
              v = f32x4{__fmaf_rn(scale, e.x, v.x), __fmaf_rn(scale, e.y, v.y), __fmaf_rn(scale, e.z, v.z), __fmaf_rn(scale, e.w, v.w)};
            }
            if (!ok[u]) v = f32x4{0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<u32x2*>(dst + r * pitch + c) = pack_bf16x4(v.x, v.y, v.z, v.w);
          }
        }
      }
    };
    // one loop per storage mode, chosen outside it (the mode is uniform); the regenerating loop is not
    // unrolled: its body is two hundred instructions, and the staging code should stay in the instruction cache
    if (PERTURB && nz.mode >= 2u) {
#pragma unroll 1
      for (int q = threadIdx.x; q < total; q += step) {
        const int r = q / C4, c = (q % C4) * 4, k = kbase + c;
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
        if (r < rows && k < cols) {
          const uint32_t idx = off + (uint32_t)r * (uint32_t)cols + (uint32_t)k;
          v = *reinterpret_cast<const f32x4*>(src + idx);
          float z[4];
          noise_regen4(nz.row, idx, nz.gen, nz.k0, nz.k1, nz.mode == 3u, z);
          v = f32x4{__fmaf_rn(scale, z[0], v.x), __fmaf_rn(scale, z[1], v.y), __fmaf_rn(scale, z[2], v.z), __fmaf_rn(scale, z[3], v.w)};
        }
        *reinterpret_cast<u32x2*>(dst + r * pitch + c) = pack_bf16x4(v.x, v.y, v.z, v.w);
      }
    } else if (PERTURB && nz.mode == 1u) {
      batch([&](uint32_t idx) { return *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(nz.ptr) + idx); });
    } else if (PERTURB) {
      batch([&](uint32_t idx) { return *reinterpret_cast<const f32x4*>(static_cast<const float*>(nz.ptr) + idx); });
    } else {
      batch([&](uint32_t) { return 0; });
    }
    return;
  }
  const int total = rows_p * COLS;
  for (int q = threadIdx.x; q < total; q += (int)blockDim.x) {
    const int r = q / COLS, k = kbase + q % COLS;
    float v = 0.0f;
    if (r < rows && k < cols) {
      const uint32_t idx = off + (uint32_t)r * (uint32_t)cols + (uint32_t)k;
      v = src[idx];
      if (PERTURB) {
        v = __fmaf_rn(scale, row_noise(nz, idx), v);
      }
    }
    dst[r * pitch + (q % COLS)] = (uint16_t)bf16_bits(v);
  }
}

template <class V, bool RELU, bool NORM>
__global__ __launch_bounds__(V::NT) __attribute__((amdgpu_waves_per_eu(V::OCC * V::NW / 4, V::OCC * V::NW / 4)))
void rollout_mfma_kernel(const MfmaArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int KT1 = V::KT1, MT3 = V::MT3, MTE = V::MTE, KTA = V::KTA, PX = V::PX, PA = V::PA;
  constexpr int NW = V::NW, NT = V::NT, MT_H = V::MT_H;
  constexpr bool ENV_ALL = (V::ENV_ROWS == V::NOP);   // every wavefront's next-state tiles are inside the padded state
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
  float* bxs = reinterpret_cast<float*>(lds + V::OFF_BX);
  constexpr int ME = V::ME;
  uint16_t* x0s = reinterpret_cast<uint16_t*>(lds + V::OFF_X0);
  float* ss0s = reinterpret_cast<float*>(lds + V::OFF_SS0);
  uint16_t* x0ps = reinterpret_cast<uint16_t*>(lds + V::OFF_X0P);
  float* mus = reinterpret_cast<float*>(lds + V::OFF_MU);
  float* ivs = reinterpret_cast<float*>(lds + V::OFF_IV);
  const int no = (int)a.no, nh = (int)a.nh, na = (int)a.na;

  if (NORM) {     // padded rows get scale 0: their normalised value stays 0
    for (int k = tid; k < V::NOP; k += NT) {
      mus[k] = k < no ? a.obs_mean[k] : 0.0f;
      ivs[k] = k < no ? a.obs_inv[k] : 0.0f;
    }
  }
  // ---------------- environment matrices -> registers / LDS (once per workgroup) ----------------
  constexpr int KTAR = V::KTAR, KTAL = V::KTAL, PAL = V::PAL;
  constexpr bool ENVF = V::ENVF;
  constexpr int KPL = V::KPL, PXF = V::PXF;
  bf16x8 Ar[MTE][KTAR > 0 ? KTAR : 1], Br[MTE][KTA];
  // binary32 environment: A and B as fp32 MFMA A operands.  K slot (kk, g) of the state product stands for state
  // element KPL g + kk (so a lane's KPL operands are contiguous in the binary32 state buffer), K slot (kk, g) of the
  // action product for action row 4 g + kk (what the lane holds after the action layer): Af[tt][kk] = A[row][KPL g + kk],
  // Bf[tt][kk] = B[row][4 g + kk], row = 16 (w MTE + tt) + n.
  float Af[ENVF ? MTE : 1][ENVF ? KPL : 1], Bf[ENVF ? MTE : 1][4];
  if constexpr (ENVF) {
#pragma unroll
    for (int t = 0; t < MTE; ++t) {
      const int row = 16 * (w * MTE + t) + n;
#pragma unroll
      for (int kk = 0; kk < KPL; ++kk) { const int k = KPL * g + kk; Af[t][kk] = (row < no && k < no) ? a.A[row * no + k] : 0.0f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) { const int c = 4 * g + kk; Bf[t][kk] = (row < no && c < na) ? a.B[row * na + c] : 0.0f; }
    }
  }
#pragma unroll
  for (int kr = 0; kr < (ENVF ? 0 : (KTAR + KC - 1) / KC); ++kr) {
    stage_cols<32 * KC, false>(stage, PW, V::ENV_ROWS, no, no, 32 * KC * kr, a.A, NoiseRow{}, 0.0f, 0u);
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
    stage_cols<32 * (KTAL > 0 ? KTAL : 1), false>(reinterpret_cast<uint16_t*>(lds + V::OFF_AL), PAL, V::ENV_ROWS, no, no,
                                                    32 * KTAR, a.A, NoiseRow{}, 0.0f, 0u);
  if constexpr (V::SMALL_LDS) {
    stage_cols<V::NAP, false>(reinterpret_cast<uint16_t*>(lds + V::OFF_BL), V::PA, V::ENV_ROWS, no, na, 0, a.B, NoiseRow{}, 0.0f, 0u);
  } else if constexpr (!ENVF) {
    stage_cols<32 * KC, false>(stage, PW, V::ENV_ROWS, no, na, 0, a.B, NoiseRow{}, 0.0f, 0u);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < MTE; ++t)
#pragma unroll
      for (int kt = 0; kt < KTA; ++kt)
        Br[t][kt] = lds_tile(lds, 2 * ((16 * (w * MTE + t) + n) * PW + 32 * kt + 8 * g));
    if constexpr (V::KSPLIT16) {
      // K slot j < 4 of lane group g stands for action row 4g + j, slot j >= 4 for row 16 + 4g + (j - 4) of the second
      // action tile (padding when there is one tile) - the rows whose sums the lane holds after the action layer: the
      // action goes from those registers into the MFMA
#pragma unroll
      for (int t = 0; t < MTE; ++t) {
        const unsigned char* src = lds + 2 * ((16 * (w * MTE + t) + n) * PW + 4 * g);
        const u32x2 lo = *reinterpret_cast<const u32x2*>(src);
        u32x2 hi = u32x2{0u, 0u};                                   // second action tile: rows 16 + 4g + (j - 4) in slots 4..7
        if (MT3 > 1) hi = *reinterpret_cast<const u32x2*>(src + 2 * 16);
        Br[t][0] = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
      }
    }
    __syncthreads();
  }

  const uint32_t per_unit = a.antithetic ? 2u : 1u;
  const uint32_t nblk = (a.E + (uint32_t)NC - 1u) / (uint32_t)NC;
  int x0_block = -1;

  // the grid is persistent over individuals (not over mirrored pairs: a small population then still fills the chip;
  // the noise row is fetched once per individual either way)
  for (uint32_t i = blockIdx.x; i < a.N; i += gridDim.x) {
    {
      struct { const float* theta; const void* noise; const uint32_t* noise_offs;
               uint32_t ld, oW1, ob1, oW2, ob2, oW3, ob3, gen, k0, k1, noise_mode; float sigma; } sa;
      sa.theta = KARG(theta); sa.noise = KARG(noise); sa.noise_offs = KARG(noise_offs); sa.ld = KARG(ld);
      sa.oW1 = KARG(oW1); sa.ob1 = KARG(ob1); sa.oW2 = KARG(oW2); sa.ob2 = KARG(ob2); sa.oW3 = KARG(oW3); sa.ob3 = KARG(ob3);
      sa.gen = KARG(gen); sa.k0 = KARG(k0); sa.k1 = KARG(k1); sa.noise_mode = KARG(noise_mode); sa.sigma = KARG(sigma);
      const uint32_t unit = i / per_unit, sub = i - unit * per_unit;
      const float scale = sub ? -sa.sigma : sa.sigma;
      NoiseRow nz;
      nz.mode = sa.noise_mode; nz.row = unit; nz.gen = sa.gen; nz.k0 = sa.k0; nz.k1 = sa.k1;
      nz.ptr = nullptr;           // regenerated noise has no buffer
      if (sa.noise_offs) nz.ptr = table_row_base(sa.noise_mode, sa.noise, sa.noise_offs, unit);
      else if (sa.noise_mode == 1u) nz.ptr = static_cast<const uint16_t*>(sa.noise) + (size_t)unit * sa.ld;
      else if (sa.noise_mode == 0u) nz.ptr = static_cast<const float*>(sa.noise) + (size_t)unit * sa.ld;

      // ---------------- perturbed policy weights -> registers ----------------
      bf16x8 W1r[MT_H][KT1], W2r[MT_H][KT_H], Wxr[ME > 0 ? ME : 1][MT_H][KT_H];
      for (int u = tid; u < NHP; u += NT) {     // biases: perturbed, bf16-rounded, kept as binary32
        float v1 = 0.0f, v2 = 0.0f;
        if (u < nh) {
          const uint32_t i1 = sa.ob1 + u, i2 = sa.ob2 + u;
          v1 = bf16_round(__fmaf_rn(scale, row_noise(nz, i1), sa.theta[i1]));
          if (ME >= 0) v2 = bf16_round(__fmaf_rn(scale, row_noise(nz, i2), sa.theta[i2]));      // a single hidden layer has no second one
        }
        b1s[u] = v1;
        b2s[u] = v2;
#pragma unroll
        for (int j = 0; j < ME; ++j) {          // hidden layer 3 + j: matrix, then bias, after layer 2's
          float vx = 0.0f;
          if (u < nh) {
            const uint32_t ix = sa.ob2 + (uint32_t)(j + 1) * (uint32_t)(nh * nh + nh) + u;
            vx = bf16_round(__fmaf_rn(scale, row_noise(nz, ix), sa.theta[ix]));
          }
          bxs[j * NHP + u] = vx;
        }
      }
      for (int c = tid; c < 16 * MT3; c += NT) {
        float v3 = 0.0f;
        if (c < na) {
          const uint32_t i3 = sa.ob3 + c;
          const float e3 = row_noise(nz, i3);
          v3 = bf16_round(__fmaf_rn(scale, e3, sa.theta[i3]));
        }
        b3s[c] = v3;
      }
      // action-layer weights stay in LDS (read by one wavefront per tile each step)
      stage_cols<NHP, true>(reinterpret_cast<uint16_t*>(lds + V::OFF_W3), PH, 16 * MT3, na, nh, 0, sa.theta, nz, scale, sa.oW3);
#pragma unroll
      for (int kr = 0; kr < (KT1 + KC - 1) / KC; ++kr) {
        stage_cols<32 * KC, true>(stage, PW, NHP, nh, no, 32 * KC * kr, sa.theta, nz, scale, sa.oW1);
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
      for (int kr = 0; kr < (ME >= 0 ? KT_H / KC : 0); ++kr) {
        stage_cols<32 * KC, true>(stage, PW, NHP, nh, nh, 32 * KC * kr, sa.theta, nz, scale, sa.oW2);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < MT_H; ++t)
#pragma unroll
          for (int kk = 0; kk < KC; ++kk)
            W2r[t][kr * KC + kk] = lds_tile(lds, 2 * ((16 * (w * MT_H + t) + n) * PW + 32 * kk + 8 * g));
        __syncthreads();
      }

#pragma unroll
      for (int j = 0; j < ME; ++j) {
#pragma unroll
        for (int kr = 0; kr < KT_H / KC; ++kr) {
          stage_cols<32 * KC, true>(stage, PW, NHP, nh, nh, 32 * KC * kr, sa.theta, nz, scale,
                                    sa.oW2 + (uint32_t)(j + 1) * (uint32_t)(nh * nh + nh));
          __syncthreads();
#pragma unroll
          for (int t = 0; t < MT_H; ++t)
#pragma unroll
            for (int kk = 0; kk < KC; ++kk)
              Wxr[j][t][kr * KC + kk] = lds_tile(lds, 2 * ((16 * (w * MT_H + t) + n) * PW + 32 * kk + 8 * g));
          __syncthreads();
        }
      }

      // FUSE3: this wavefront's K slice (its own 64 hidden units) of the action-layer weights, as MFMA A operands.  The K
      // order inside a tile follows the order in which the lane holds h2 after the layer-2 epilogue: slots 0..3 = units
      // 4g..4g+3 of the even 16-unit tile, slots 4..7 = the same rows of the odd tile (any K order is as good as another
      // as long as both operands agree), so h2 goes from the epilogue's registers into the MFMA with no exchange.
      bf16x8 W3k[(V::FUSE3 || V::KSPLIT16) ? MT3 : 1][2];
      auto w3k_tile = [&](int mt, int kk) {
        const unsigned char* src = lds + V::OFF_W3 + 2 * ((16 * mt + n) * PH + 64 * w + 32 * kk + 4 * g);
        const u32x2 lo = *reinterpret_cast<const u32x2*>(src), hi = *reinterpret_cast<const u32x2*>(src + 2 * 16);
        return __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
      };
      // ... held in registers where the file has room for them; fetched from LDS at their use otherwise (all of A in
      // registers, two workgroups per CU, more than two hidden layers)
      constexpr bool W3K_REGS = (V::FUSE3 && !V::SMALL_LDS) || V::KSPLIT16;
      if constexpr (W3K_REGS) {
#pragma unroll
        for (int mt = 0; mt < MT3; ++mt)
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) W3k[mt][kk] = w3k_tile(mt, kk);
      }

      float fit_sum = 0.0f;
      for (uint32_t cb = 0; cb < nblk; ++cb) {
        // ---------------- initial states of this block of environment copies ----------------
        if (x0_block != (int)cb) {
          // thread -> (column n0, row group kq): s0[k] for k = kq, kq + 16, ...
          constexpr int KG = NT / NC;                // row groups
          const int n0 = tid % NC, kq = tid / NC;
          const uint32_t x_gen = KARG(gen), x_k0 = KARG(k0), x_k1 = KARG(k1);
          const uint32_t e0 = cb * (uint32_t)NC + (uint32_t)n0;
          float part = 0.0f;
          for (int k = kq; k < V::NOP; k += KG) {
            float v = 0.0f;
            if (k < no && e0 < a.E) v = reset_value((uint32_t)k, e0, x_gen, x_k0, x_k1);
            part = __fmaf_rn(v, v, part);
            x0s[n0 * PX + k] = (uint16_t)bf16_bits(v);
            if (ENVF) reinterpret_cast<float*>(lds + V::OFF_X0F)[n0 * PXF + k] = v;
            if (NORM) x0ps[n0 * PX + k] = (uint16_t)bf16_bits((v - mus[k]) * ivs[k]);
          }
          float* scratch = reinterpret_cast<float*>(lds + V::OFF_SCR);   // KG x NC partial norms
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
          for (int r = tid; r < NC * PX / 2; r += NT) dst[r] = src[r];
          if (ENVF) {
            const float* srcf = reinterpret_cast<const float*>(lds + V::OFF_X0F);
            float* dstf = reinterpret_cast<float*>(lds + V::OFF_XF);
            for (int r = tid; r < NC * PXF; r += NT) dstf[r] = srcf[r];
          }
          if (NORM) {
            const uint32_t* srcp = reinterpret_cast<const uint32_t*>(x0ps);
            uint32_t* dstp = reinterpret_cast<uint32_t*>(lds + V::OFF_XP);
            for (int r = tid; r < NC * PX / 2; r += NT) dstp[r] = srcp[r];
          }
          uint32_t* qz = reinterpret_cast<uint32_t*>(lds + V::OFF_QA);
          for (int r = tid; r < NW * NC * PA / 2; r += NT) qz[r] = 0u;
        }
        __syncthreads();

        const uint32_t e = cb * (uint32_t)NC + (uint32_t)col;
        bool alive = e < a.E;
        float Rn = 0.0f;
        int32_t Ln = 0;
        const float inv_no = 1.0f / (float)no;
        constexpr int KA1 = ENVF ? 0 : (ME < 0 ? KT1 : (KT1 + 1) / 2);       // K tiles of A x done beside layer 1; the rest beside layer 2
        f32x4 av = f32x4{0.f, 0.f, 0.f, 0.f};     // binary32 environment: the action (rows 4g..4g+3 of column n), kept in registers

        f32x4 acc[MT_H], accE[MTE];
#pragma unroll
        for (int tt = 0; tt < MT_H; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b1s + 16 * (w * MT_H + tt) + 4 * g);
        // the norm partials of "step -1": |s_0|^2 in slot 0, nothing above the threshold
        if (tid < 16) {
          float* sp = reinterpret_cast<float*>(lds + V::OFF_SSP) + tid * NW;
          unsigned* mp = reinterpret_cast<unsigned*>(lds + V::OFF_MXP) + tid * NW;
          for (int r = 0; r < NW; ++r) { sp[r] = 0.0f; mp[r] = 0u; }
          if (tid < NC) sp[0] = ss0s[tid];
        }
        __syncthreads();
        float aa_prev = 0.0f;     // |a_{t-1}|^2 of this lane's column
        float ss_cur = 0.0f;      // |s_{t-1}|^2 while step t starts; the reward of step t-1 is booked in step t
        bool first = true;

#ifdef ES_PHASE_PROF
        unsigned long long prof_acc[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        unsigned long long prof_last = __builtin_readcyclecounter();
#endif
        // KSPLIT16, after the last hidden layer: it stays in registers - the lane's values of tiles 0, 1 and of tiles 2, 3 are
        // the two K tiles of this wavefront's slice of the action layer - and only the binary32 partial sums cross the LDS
        auto last_hidden_ksplit = [&](const f32x4 (&accs)[MT_H]) {
          static_assert(!V::KSPLIT16 || MT_H == 4, "four hidden tiles per wavefront");
          if constexpr (!W3K_REGS) {      // requested ahead of the activation, which hides the latency
#pragma unroll
            for (int mt = 0; mt < MT3; ++mt)
#pragma unroll
              for (int kk = 0; kk < 2; ++kk) W3k[mt][kk] = w3k_tile(mt, kk);
          }
          u32x2 hp[MT_H];
#pragma unroll
          for (int tt = 0; tt < MT_H; ++tt) {
            const f32x4 h = hidden4<RELU>(accs[tt]);
            hp[tt] = pack_bf16x4(h.x, h.y, h.z, h.w);
          }
          const bf16x8 bk0 = __builtin_bit_cast(bf16x8, u32x4{hp[0].x, hp[0].y, hp[1 % MT_H].x, hp[1 % MT_H].y});
          const bf16x8 bk1 = __builtin_bit_cast(bf16x8, u32x4{hp[2 % MT_H].x, hp[2 % MT_H].y, hp[3 % MT_H].x, hp[3 % MT_H].y});
#pragma unroll
          for (int mt = 0; mt < MT3; ++mt) {
            f32x4 p3 = mfma16(W3k[mt][0], bk0, f32x4{0.f, 0.f, 0.f, 0.f});
            p3 = mfma16(W3k[mt][1], bk1, p3);
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(lds + V::OFF_P3) + (w * 16 + n) * V::PP3 + 16 * mt + 4 * g) = p3;
          }
        };
        if constexpr (V::FUSE3) {
        // Passes of four copies, two hidden layers (FUSE3): the action layer is split along K.  Every wavefront multiplies
        // the 64 units of h2 it has just produced - still in its registers - with its slice of the action-layer weights;
        // only the binary32 partial sums [wavefront][copy][action row] cross the LDS, and every wavefront adds them in the
        // same order.  h2 itself is never exchanged: three workgroup barriers per step instead of four, and no phase in
        // which two wavefronts wait for the other two.  The state has two buffers (steps alternate) so that a wavefront
        // may still read s_t while another already writes s_{t+1}; the books of the previous step ride under the layer-1 stream.
        float* p3s = reinterpret_cast<float*>(lds + V::OFF_P3);
        const int qq = q & 1;                                  // this lane adds up action rows 8g + 4qq .. + 3 of column col
        const bool arow_ok = 8 * g + 4 * qq < 16 * MT3;        // rows past the padded action width stay exactly zero
        for (uint32_t t = 0; t <= a.T; ++t) {
          const int off_x = (t & 1u) ? V::OFF_X1 : V::OFF_X, off_xn = (t & 1u) ? V::OFF_X : V::OFF_X1;
          // ---- phase A: h1 = act(W1 x + b1); books of the previous step; first half of A x under the epilogue ----
          const f32x4 sp4 = *reinterpret_cast<const f32x4*>(lds + V::OFF_SSP + 4 * NW * col);
          const u32x4 mp4 = *reinterpret_cast<const u32x4*>(lds + V::OFF_MXP + 4 * NW * col);
          bf16x8 bx[KA1 > 0 ? KA1 : 1], bxr[3];
          auto xload = [&](int kt) { return lds_tile(lds, off_x + 2 * (col * PX + 32 * kt + 8 * g)); };
          auto xfetch = [&](int kt) {
            if (NORM) {
              bxr[kt % 3] = lds_tile(lds, V::OFF_XP + 2 * (col * PX + 32 * kt + 8 * g));
              if (kt < KA1) bx[kt < KA1 ? kt : 0] = xload(kt);
            } else if (kt < KA1) {
              bx[kt < KA1 ? kt : 0] = xload(kt);
            } else {
              bxr[kt % 3] = xload(kt);
            }
          };
#pragma unroll
          for (int kt = 0; kt < 2 && kt < KT1; ++kt) xfetch(kt);
          __builtin_amdgcn_sched_barrier(0);
          constexpr int KT_BOOKS = KT1 > 2 ? 2 : KT1 - 1;      // the stage after which the books are done (their inputs have arrived by then)
#pragma unroll
          for (int kt = 0; kt < KT1; ++kt) {
            if (kt + 2 < KT1) xfetch(kt + 2);
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) {
              if (V::OCC == 1) pin_agpr(W1r[tt][kt]);
              acc[tt] = mfma16(W1r[tt][kt], (!NORM && kt < KA1) ? bx[kt < KA1 ? kt : 0] : bxr[kt % 3], acc[tt]);
            }
            if (kt == KT_BOOKS) {
              // every lane combines the four wavefronts' partials of its column in the same fixed order; branch-free, so that
              // the vector work issues between the matrix-core instructions
              const float ss_new = (sp4.x + sp4.y) + (sp4.z + sp4.w);
              const float mx = __builtin_bit_cast(float, umax(umax(mp4.x, mp4.y), umax(mp4.z, mp4.w)));
              const bool book = !first, add = book && alive;
              const float r = __fmaf_rn(-ss_cur, inv_no, 1.0f) - a.act_cost * aa_prev;
              Rn += add ? r : 0.0f;
              Ln += add ? 1 : 0;
              alive = alive && !(book && mx > a.done_thresh);
              ss_cur = ss_new;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          first = false;
          PSTAMP(0);
          if (t == a.T || __ballot(alive) == 0ull) break;       // identical in all four wavefronts
          PSTAMP(1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int tt = 0; tt < MTE; ++tt) accE[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kt = 0; kt < KA1; ++kt) {
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt)
              if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
                if (kt < KTAR) accE[tt] = mfma16(Ar[tt][kt], bx[kt], accE[tt]);
                else accE[tt] = mfma16(lds_tile(lds, V::OFF_AL + 2 * ((16 * (w * MTE + tt) + n) * PAL + 32 * (kt - KTAR) + 8 * g)), bx[kt], accE[tt]);
              }
          }
          {
            const f32x4 h = hidden4<RELU>(compact4<MT_H>(acc));
            if (q < MT_H)
              *reinterpret_cast<u32x2*>(lds + V::OFF_H1 + 2 * (col * PH + 16 * (w * MT_H + q) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
          }
#pragma unroll
          for (int r = 0; r < KA1 * MTE; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          }
          PSTAMP(2);
          // ---- phase B: h2 = act(W2 h1 + b2) with the second half of A x in the same stream; then this wavefront's K slice of W3 h2 ----
#pragma unroll
          for (int tt = 0; tt < MT_H; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b2s + 16 * (w * MT_H + tt) + 4 * g);
          __syncthreads();
          PSTAMP(3);
          {
            constexpr int NT2 = (KT1 - KA1) * MTE;      // MFMAs of the second half of A x; j = (kt - KA1) * MTE + tt
            constexpr int PS = (NT2 + KT_H - 1) / KT_H; // ... of which this many ride in each stage of the W2 stream
            bf16x8 bh[3], at[3 * (PS > 0 ? PS : 1)], bx2[KT1 - KA1 > 0 ? KT1 - KA1 : 1];
            auto fetch = [&](int kt) {
              bh[kt % 3] = lds_tile(lds, V::OFF_H1 + 2 * (col * PH + 32 * kt + 8 * g));
#pragma unroll
              for (int r = 0; r < PS; ++r) {
                const int j = kt * PS + r;
                if (j < NT2) {
                  const int ka = KA1 + j / MTE, tt = j % MTE;
                  if (ka >= KTAR) at[(kt % 3) * PS + r] = lds_tile(lds, V::OFF_AL + 2 * ((16 * (w * MTE + tt) + n) * PAL + 32 * (ka - KTAR) + 8 * g));
                  if (tt == 0 || r == 0) bx2[ka - KA1] = lds_tile(lds, off_x + 2 * (col * PX + 32 * ka + 8 * g));
                }
              }
            };
            fetch(0);
            fetch(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kt = 0; kt < KT_H; ++kt) {
              if (kt + 2 < KT_H) fetch(kt + 2);
#pragma unroll
              for (int tt = 0; tt < MT_H; ++tt) { pin_agpr(W2r[tt][kt]); acc[tt] = mfma16(W2r[tt][kt], bh[kt % 3], acc[tt]); }
#pragma unroll
              for (int r = 0; r < PS; ++r) {
                const int j = kt * PS + r;
                if (j < NT2) {
                  const int ka = KA1 + j / MTE, tt = j % MTE;
                  if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
                    if (ka < KTAR) accE[tt] = mfma16(Ar[tt][ka < KTAR ? ka : 0], bx2[ka - KA1], accE[tt]);
                    else accE[tt] = mfma16(at[(kt % 3) * PS + r], bx2[ka - KA1], accE[tt]);
                  }
                }
              }
              __builtin_amdgcn_sched_barrier(0);
            }
          }
          PSTAMP(4);
          {
            if constexpr (V::SMALL_LDS) {      // fetched here, ahead of the activation that hides the latency
#pragma unroll
              for (int mt = 0; mt < MT3; ++mt)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) W3k[mt][kk] = w3k_tile(mt, kk);
            }
            // h2 of this wavefront's 64 units stays in registers: lane (g, 4q + c) holds units 4g..4g+3 of tile q for copy c
            const f32x4 h = hidden4<RELU>(compact4<MT_H>(acc));
            const u32x2 hp = pack_bf16x4(h.x, h.y, h.z, h.w);
            // the lanes of the four real columns (n < 4) collect the other three tiles of their copy from the lanes to their right
            const uint32_t s4x = dpp_shl_u<0x104>(hp.x), s4y = dpp_shl_u<0x104>(hp.y);
            const uint32_t s8x = dpp_shl_u<0x108>(hp.x), s8y = dpp_shl_u<0x108>(hp.y);
            const uint32_t scx = dpp_shl_u<0x10C>(hp.x), scy = dpp_shl_u<0x10C>(hp.y);
            const bf16x8 bk0 = __builtin_bit_cast(bf16x8, u32x4{hp.x, hp.y, s4x, s4y});     // K tile of the wavefront's tiles 0, 1
            const bf16x8 bk1 = __builtin_bit_cast(bf16x8, u32x4{s8x, s8y, scx, scy});       // ... and of tiles 2, 3
#pragma unroll
            for (int mt = 0; mt < MT3; ++mt) {
              f32x4 p3 = mfma16(W3k[mt][0], bk0, f32x4{0.f, 0.f, 0.f, 0.f});
              p3 = mfma16(W3k[mt][1], bk1, p3);
              if (n < NC) *reinterpret_cast<f32x4*>(p3s + (w * NC + n) * 32 + 16 * mt + 4 * g) = p3;
            }
          }
#pragma unroll
          for (int tt = 0; tt < MT_H; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b1s + 16 * (w * MT_H + tt) + 4 * g);
          PSTAMP(5);
          __syncthreads();
          PSTAMP(6);
          // ---- phase D: a = tanh(sum of the partials + b3); s' = tanh(A x + B a); norms for the reward and the termination test ----
          bf16x8 ba, brt[MTE];
          if constexpr (V::SMALL_LDS) {
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt) brt[tt] = lds_tile(lds, V::OFF_BL + 2 * ((16 * (w * MTE + tt) + n) * V::PA + 8 * g));
          } else {
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt) brt[tt] = Br[tt][0];
          }
          {
            f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
            if (arow_ok) {
              const int r0 = 8 * g + 4 * qq;
              v = *reinterpret_cast<const f32x4*>(b3s + r0);
#pragma unroll
              for (int ww = 0; ww < NW; ++ww) v += *reinterpret_cast<const f32x4*>(p3s + (ww * NC + col) * 32 + r0);
              {      // branch-free: a select costs four instructions, the branch cost six register moves on the chain
                const f32x4 tv = tanh4(v);
                const bool squash = a.out_tanh != 0u;
                v = f32x4{squash ? tv.x : v.x, squash ? tv.y : v.y, squash ? tv.z : v.z, squash ? tv.w : v.w};
              }
            }
            float part = v.x * v.x;
            part = __fmaf_rn(v.y, v.y, part); part = __fmaf_rn(v.z, v.z, part); part = __fmaf_rn(v.w, v.w, part);
            part = part + dpp_shl<0x104>(part);          // rows 8g..8g+7 of the column (lanes n < 12; the books read lanes n < 4)
            aa_prev = rows_sum(part);                    // |a_t|^2 of column col
            const u32x2 ap = pack_bf16x4(v.x, v.y, v.z, v.w);
            const uint32_t a4x = dpp_shl_u<0x104>(ap.x), a4y = dpp_shl_u<0x104>(ap.y);
            ba = __builtin_bit_cast(bf16x8, u32x4{ap.x, ap.y, a4x, a4y});      // action rows 8g..8g+7 of column n (n < 4)
          }
#pragma unroll
          for (int tt = 0; tt < MTE; ++tt) accE[tt] = mfma16(brt[tt], ba, accE[tt]);
          PSTAMP(7);
          float ssp = 0.0f;
          unsigned mxp = 0u;
          {
            const int tile = w * MTE + q;
            const bool valid = q < MTE && (ENV_ALL || 16 * tile < V::NOP);
            const f32x4 sn = tanh4(compact4<MTE>(accE));
            if (valid) {
              ssp = sn.x * sn.x;
              ssp = __fmaf_rn(sn.y, sn.y, ssp); ssp = __fmaf_rn(sn.z, sn.z, ssp); ssp = __fmaf_rn(sn.w, sn.w, ssp);
              mxp = umax(umax(abs_bits(sn.x), abs_bits(sn.y)), umax(abs_bits(sn.z), abs_bits(sn.w)));
              *reinterpret_cast<u32x2*>(lds + off_xn + 2 * (col * PX + 16 * tile + 4 * g)) = pack_bf16x4(sn.x, sn.y, sn.z, sn.w);
              if (NORM) {
                const f32x4 xn = (sn - *reinterpret_cast<const f32x4*>(mus + 16 * tile + 4 * g)) * *reinterpret_cast<const f32x4*>(ivs + 16 * tile + 4 * g);
                *reinterpret_cast<u32x2*>(lds + V::OFF_XP + 2 * (col * PX + 16 * tile + 4 * g)) = pack_bf16x4(xn.x, xn.y, xn.z, xn.w);
              }
            }
            ssp = row_bank_sum(ssp);
            mxp = row_bank_umax(mxp);
          }
          ssp = rows_sum(ssp);
          mxp = rows_umax(mxp);
          if (g == 0 && n < NC) {
            reinterpret_cast<float*>(lds + V::OFF_SSP)[col * NW + w] = ssp;
            reinterpret_cast<unsigned*>(lds + V::OFF_MXP)[col * NW + w] = mxp;
          }
          PSTAMP(9);
          __syncthreads();
          PSTAMP(10);
        }
        } else {
        for (uint32_t t = 0; t <= a.T; ++t) {
          // ---- phase A: h1 = tanh(W1 x + b1); first half of A x; books of the previous step ----
          // partial norms of the previous step, one per wavefront (consumed after the MFMA stream below)
          const f32x4 sp4 = *reinterpret_cast<const f32x4*>(lds + V::OFF_SSP + 4 * NW * col);
          const u32x4 mp4 = *reinterpret_cast<const u32x4*>(lds + V::OFF_MXP + 4 * NW * col);
          float xf[ENVF ? KPL : 1];                 // binary32 environment: this lane's state operands, elements KPL g .. of column n
          if constexpr (ENVF) {
#pragma unroll
            for (int j = 0; j < KPL / 4; ++j) {
              const f32x4 v4 = *reinterpret_cast<const f32x4*>(lds + V::OFF_XF + 4 * (n * PXF + KPL * g + 4 * j));
              xf[4 * j] = v4.x; xf[4 * j + 1] = v4.y; xf[4 * j + 2] = v4.z; xf[4 * j + 3] = v4.w;
            }
          }
          // W1 stream: the B operand (state tiles) runs two stages ahead of the MFMAs
          bf16x8 bx[KA1 > 0 ? KA1 : 1], bxr[3];     // tiles < KA1 are kept for A x below; the rest pass through a ring
          auto xload = [&](int kt) { return lds_tile(lds, V::OFF_X + 2 * (col * PX + 32 * kt + 8 * g)); };
          // with observation statistics the policy reads the normalised state and A x the raw one
          auto xfetch = [&](int kt) {
            if (NORM) {
              bxr[kt % 3] = lds_tile(lds, V::OFF_XP + 2 * (col * PX + 32 * kt + 8 * g));
              if (kt < KA1) bx[kt < KA1 ? kt : 0] = xload(kt);
            } else if (kt < KA1) {
              bx[kt < KA1 ? kt : 0] = xload(kt);
            } else {
              bxr[kt % 3] = xload(kt);
            }
          };
#pragma unroll
          for (int kt = 0; kt < 2 && kt < KT1; ++kt) xfetch(kt);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int kt = 0; kt < KT1; ++kt) {
            if (kt + 2 < KT1) xfetch(kt + 2);
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) {
              if (V::OCC == 1 && ME == 0) pin_agpr(W1r[tt][kt]);    // with two workgroups per CU, or deeper policies, the accumulation half belongs to the 256x256 layers
              acc[tt] = mfma16(W1r[tt][kt], (!NORM && kt < KA1) ? bx[kt < KA1 ? kt : 0] : bxr[kt % 3], acc[tt]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          PSTAMP(0);
          // every lane combines the four wavefronts' partials of its column in the same fixed order
          float ss_new = (sp4.x + sp4.y) + (sp4.z + sp4.w);
          unsigned mxb = umax(umax(mp4.x, mp4.y), umax(mp4.z, mp4.w));
          const float mx = __builtin_bit_cast(float, mxb);
          const float aa = aa_prev;
          if (!first) {
            if (alive) {
              Rn += __fmaf_rn(-ss_cur, inv_no, 1.0f) - a.act_cost * aa;
              Ln += 1;
            }
            alive = alive && !(mx > a.done_thresh);
          }
          first = false;
          ss_cur = ss_new;
          if (t == a.T || __ballot(alive) == 0ull) break;       // identical in all four wavefronts
          PSTAMP(1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int tt = 0; tt < MTE; ++tt) accE[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
          // first half of A x (register tiles first) interleaved with the layer-1 epilogue
#pragma unroll
          for (int kt = 0; kt < KA1; ++kt) {
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt)
              if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
                if (kt < KTAR) accE[tt] = mfma16(Ar[tt][kt], bx[kt], accE[tt]);
                else accE[tt] = mfma16(lds_tile(lds, V::OFF_AL + 2 * ((16 * (w * MTE + tt) + n) * PAL + 32 * (kt - KTAR) + 8 * g)), bx[kt], accE[tt]);
              }
          }
          if constexpr (ENVF) {          // A s in binary32, under the layer-1 epilogue like the bf16 tiles above
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk)
#pragma unroll
              for (int tt = 0; tt < MTE; ++tt)
                if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) accE[tt] = mfma4(Af[tt][kk], xf[kk], accE[tt]);
          }
          if (NC == 4) {
            const f32x4 h = hidden4<RELU>(compact4<MT_H>(acc));
            if (q < MT_H)
              *reinterpret_cast<u32x2*>(lds + V::OFF_H1 + 2 * (col * PH + 16 * (w * MT_H + q) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
          } else if constexpr (V::KSPLIT16 && ME < 0) {
            last_hidden_ksplit(acc);
          } else {
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) {
              const f32x4 h = hidden4<RELU>(acc[tt]);
              *reinterpret_cast<u32x2*>(lds + V::OFF_H1 + 2 * (n * PH + 16 * (w * MT_H + tt) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
            }
          }
#pragma unroll
          for (int r = 0; r < (ENVF ? KPL * MTE : KA1 * MTE); ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, NC == 4 ? 4 : 8, 0);
          }
          // ---- phase B: h2 = tanh(W2 h1 + b2); second half of A x ----
          PSTAMP(2);
          if constexpr (ME >= 0) {
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b2s + 16 * (w * MT_H + tt) + 4 * g);
            __syncthreads();
            PSTAMP(3);
            constexpr int NT2 = ENVF ? 0 : (KT1 - KA1) * MTE;      // MFMAs of the second half of A x; j = (kt - KA1) * MTE + tt
            constexpr int PS = (NT2 + KT_H - 1) / KT_H; // ... of which this many ride in each stage of the W2 stream
            bf16x8 bh[3], at[3 * (PS > 0 ? PS : 1)], bx2[KT1 - KA1 > 0 ? KT1 - KA1 : 1];
            // operands of stage kt are fetched two stages ahead: h1 tile, LDS-resident A tiles, state tiles
            auto fetch = [&](int kt) {
              bh[kt % 3] = lds_tile(lds, V::OFF_H1 + 2 * (col * PH + 32 * kt + 8 * g));
#pragma unroll
              for (int r = 0; r < PS; ++r) {
                const int j = kt * PS + r;
                if (j < NT2) {
                  const int ka = KA1 + j / MTE, tt = j % MTE;
                  if (ka >= KTAR) at[(kt % 3) * PS + r] = lds_tile(lds, V::OFF_AL + 2 * ((16 * (w * MTE + tt) + n) * PAL + 32 * (ka - KTAR) + 8 * g));
                  if (tt == 0 || r == 0) bx2[ka - KA1] = lds_tile(lds, V::OFF_X + 2 * (col * PX + 32 * ka + 8 * g));
                }
              }
            };
            fetch(0);
            fetch(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kt = 0; kt < KT_H; ++kt) {
              if (kt + 2 < KT_H) fetch(kt + 2);
#pragma unroll
              for (int tt = 0; tt < MT_H; ++tt) { pin_agpr(W2r[tt][kt]); acc[tt] = mfma16(W2r[tt][kt], bh[kt % 3], acc[tt]); }
#pragma unroll
              for (int r = 0; r < PS; ++r) {
                const int j = kt * PS + r;
                if (j < NT2) {
                  const int ka = KA1 + j / MTE, tt = j % MTE;
                  if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
                    if (ka < KTAR) accE[tt] = mfma16(Ar[tt][ka < KTAR ? ka : 0], bx2[ka - KA1], accE[tt]);
                    else accE[tt] = mfma16(at[(kt % 3) * PS + r], bx2[ka - KA1], accE[tt]);
                  }
                }
              }
              __builtin_amdgcn_sched_barrier(0);
            }
            PSTAMP(4);
            if (NC == 4) {
              const f32x4 h = hidden4<RELU>(compact4<MT_H>(acc));
              if (q < MT_H)
                *reinterpret_cast<u32x2*>(lds + V::OFF_H2 + 2 * (col * PH + 16 * (w * MT_H + q) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
            } else if constexpr (V::KSPLIT16 && ME == 0) {
              last_hidden_ksplit(acc);
            } else {
#pragma unroll
              for (int tt = 0; tt < MT_H; ++tt) {
                const f32x4 h = hidden4<RELU>(acc[tt]);
                *reinterpret_cast<u32x2*>(lds + V::OFF_H2 + 2 * (n * PH + 16 * (w * MT_H + tt) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
              }
            }
          }
          // ---- further hidden layers (depth m > 2): the same stream, ping-ponging between the two buffers ----
#pragma unroll
          for (int j = 0; j < ME; ++j) {
            const int off_in = (j & 1) ? V::OFF_H1 : V::OFF_H2, off_out = (j & 1) ? V::OFF_H2 : V::OFF_H1;
#pragma unroll
            for (int tt = 0; tt < MT_H; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(bxs + j * NHP + 16 * (w * MT_H + tt) + 4 * g);
            __syncthreads();
            bf16x8 bh[3];
            bh[0] = lds_tile(lds, off_in + 2 * (col * PH + 8 * g));
            bh[1] = lds_tile(lds, off_in + 2 * (col * PH + 32 + 8 * g));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kt = 0; kt < KT_H; ++kt) {
              if (kt + 2 < KT_H) bh[(kt + 2) % 3] = lds_tile(lds, off_in + 2 * (col * PH + 32 * (kt + 2) + 8 * g));
#pragma unroll
              for (int tt = 0; tt < MT_H; ++tt) {
                if (j == 0) pin_agpr(Wxr[j][tt][kt]);      // the first extra layer shares the accumulation half with layer 2
                acc[tt] = mfma16(Wxr[j][tt][kt], bh[kt % 3], acc[tt]);
              }
              __builtin_amdgcn_sched_barrier(0);
            }
            if (NC == 4) {
              const f32x4 h = hidden4<RELU>(compact4<MT_H>(acc));
              if (q < MT_H)
                *reinterpret_cast<u32x2*>(lds + off_out + 2 * (col * PH + 16 * (w * MT_H + q) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
            } else if (V::KSPLIT16 && j == ME - 1) {
              last_hidden_ksplit(acc);
            } else {
#pragma unroll
              for (int tt = 0; tt < MT_H; ++tt) {
                const f32x4 h = hidden4<RELU>(acc[tt]);
                *reinterpret_cast<u32x2*>(lds + off_out + 2 * (n * PH + 16 * (w * MT_H + tt) + 4 * g)) = pack_bf16x4(h.x, h.y, h.z, h.w);
              }
            }
          }
          PSTAMP(5);
          __syncthreads();
          PSTAMP(6);
          // ---- phase C: a = tanh(W3 h2 + b3), weights from LDS ----
          unsigned char* qaw = lds + V::OFF_QA + w * (2 * NC * PA);   // this wavefront's action buffer (four-copy passes of the other depths)
          bf16x8 ba16 = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});   // KSPLIT16: the action as a B operand, from registers
          if constexpr (V::KSPLIT16) {
            // every lane adds the four wavefronts' partials of rows 4g..4g+3 (of every action tile) of its column, in the same order everywhere
            const float* p3s = reinterpret_cast<const float*>(lds + V::OFF_P3);
            f32x4 v[MT3];
            float part = 0.0f;
#pragma unroll
            for (int mt = 0; mt < MT3; ++mt) {
              v[mt] = *reinterpret_cast<const f32x4*>(b3s + 16 * mt + 4 * g);
#pragma unroll
              for (int ww = 0; ww < NW; ++ww) v[mt] += *reinterpret_cast<const f32x4*>(p3s + (ww * 16 + n) * V::PP3 + 16 * mt + 4 * g);
              {
                const f32x4 tv = tanh4(v[mt]);
                const bool squash = a.out_tanh != 0u;
                v[mt] = f32x4{squash ? tv.x : v[mt].x, squash ? tv.y : v[mt].y, squash ? tv.z : v[mt].z, squash ? tv.w : v[mt].w};
              }
              part = __fmaf_rn(v[mt].x, v[mt].x, part); part = __fmaf_rn(v[mt].y, v[mt].y, part);
              part = __fmaf_rn(v[mt].z, v[mt].z, part); part = __fmaf_rn(v[mt].w, v[mt].w, part);
            }
            aa_prev = rows_sum(part);
            if (ENVF) av = v[0];
            else {
              const u32x2 lo = pack_bf16x4(v[0].x, v[0].y, v[0].z, v[0].w);
              u32x2 hi = u32x2{0u, 0u};
              if (MT3 > 1) hi = pack_bf16x4(v[MT3 - 1].x, v[MT3 - 1].y, v[MT3 - 1].z, v[MT3 - 1].w);
              ba16 = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
            }
          } else {
            // every wavefront computes the single action tile itself: no exchange before the environment step
            f32x4 p[MT3][2];
#pragma unroll
            for (int mt = 0; mt < MT3; ++mt) {
              p[mt][0] = *reinterpret_cast<const f32x4*>(b3s + 16 * mt + 4 * g);
              p[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int kt = 0; kt < KT_H; ++kt) {
              const bf16x8 b = lds_tile(lds, V::OFF_HL + 2 * (col * PH + 32 * kt + 8 * g));
#pragma unroll
              for (int mt = 0; mt < MT3; ++mt) {
                const bf16x8 wt = lds_tile(lds, V::OFF_W3 + 2 * ((16 * mt + n) * PH + 32 * kt + 8 * g));
                p[mt][kt & 1] = mfma16(wt, b, p[mt][kt & 1]);
              }
            }
            float part = 0.0f;
#pragma unroll
            for (int mt = 0; mt < MT3; ++mt) {
              f32x4 v = p[mt][0] + p[mt][1];
              if (a.out_tanh) v = tanh4(v);
              part = __fmaf_rn(v.x, v.x, part); part = __fmaf_rn(v.y, v.y, part);
              part = __fmaf_rn(v.z, v.z, part); part = __fmaf_rn(v.w, v.w, part);
              if (ENVF) av = v;                // one action tile (asserted): the environment reads it from these registers
              else if (n < NC)     // with 4-column passes the lanes of columns 4..15 hold copies
                *reinterpret_cast<u32x2*>(qaw + 2 * (col * PA + 16 * mt + 4 * g)) = pack_bf16x4(v.x, v.y, v.z, v.w);
            }
            aa_prev = rows_sum(part);      // |a_t|^2 of column `col` (lanes of columns >= NC hold copies)
          }
          // ---- phase D: s' = tanh(A x + B a); partial norms for the reward and the termination test ----
          float ssp = 0.0f;
          unsigned mxp = 0u;
          if (NC == 4) {
#pragma unroll
            for (int kt = 0; kt < KTA; ++kt) {
              const bf16x8 b = lds_tile(qaw, 2 * (col * PA + 32 * kt + 8 * g));
#pragma unroll
              for (int tt = 0; tt < MTE; ++tt) accE[tt] = mfma16(Br[tt][kt], b, accE[tt]);
            }
            const int tile = w * MTE + q;
            const bool valid = q < MTE && (ENV_ALL || 16 * tile < V::NOP);
            const f32x4 sn = tanh4(compact4<MTE>(accE));
            if (valid) {
              ssp = sn.x * sn.x;
              ssp = __fmaf_rn(sn.y, sn.y, ssp); ssp = __fmaf_rn(sn.z, sn.z, ssp); ssp = __fmaf_rn(sn.w, sn.w, ssp);
              mxp = umax(umax(abs_bits(sn.x), abs_bits(sn.y)), umax(abs_bits(sn.z), abs_bits(sn.w)));
              *reinterpret_cast<u32x2*>(lds + V::OFF_X + 2 * (col * PX + 16 * tile + 4 * g)) = pack_bf16x4(sn.x, sn.y, sn.z, sn.w);
              if (NORM) {
                const f32x4 xn = (sn - *reinterpret_cast<const f32x4*>(mus + 16 * tile + 4 * g)) * *reinterpret_cast<const f32x4*>(ivs + 16 * tile + 4 * g);
                *reinterpret_cast<u32x2*>(lds + V::OFF_XP + 2 * (col * PX + 16 * tile + 4 * g)) = pack_bf16x4(xn.x, xn.y, xn.z, xn.w);
              }
            }
            ssp = row_bank_sum(ssp);
            mxp = row_bank_umax(mxp);
          } else {
            if constexpr (ENVF) {
#pragma unroll
              for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int tt = 0; tt < MTE; ++tt)
                  if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) accE[tt] = mfma4(Bf[tt][kk], av[kk], accE[tt]);
            } else {
#pragma unroll
              for (int kt = 0; kt < KTA; ++kt) {
                const bf16x8 b = V::KSPLIT16 ? ba16 : lds_tile(qaw, 2 * (n * PA + 32 * kt + 8 * g));
#pragma unroll
                for (int tt = 0; tt < MTE; ++tt)
                  if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) accE[tt] = mfma16(Br[tt][kt], b, accE[tt]);
              }
            }
#pragma unroll
            for (int tt = 0; tt < MTE; ++tt) {
              if (ENV_ALL || 16 * (w * MTE + tt) < V::NOP) {
                const f32x4 sn = tanh4(accE[tt]);
                ssp = __fmaf_rn(sn.x, sn.x, ssp); ssp = __fmaf_rn(sn.y, sn.y, ssp);
                ssp = __fmaf_rn(sn.z, sn.z, ssp); ssp = __fmaf_rn(sn.w, sn.w, ssp);
                mxp = umax(mxp, umax(umax(abs_bits(sn.x), abs_bits(sn.y)), umax(abs_bits(sn.z), abs_bits(sn.w))));
                *reinterpret_cast<u32x2*>(lds + V::OFF_X + 2 * (n * PX + 16 * (w * MTE + tt) + 4 * g)) = pack_bf16x4(sn.x, sn.y, sn.z, sn.w);
                if (ENVF) *reinterpret_cast<f32x4*>(lds + V::OFF_XF + 4 * (n * PXF + 16 * (w * MTE + tt) + 4 * g)) = sn;
                if (NORM) {
                  const int r0 = 16 * (w * MTE + tt) + 4 * g;
                  const f32x4 xn = (sn - *reinterpret_cast<const f32x4*>(mus + r0)) * *reinterpret_cast<const f32x4*>(ivs + r0);
                  *reinterpret_cast<u32x2*>(lds + V::OFF_XP + 2 * (n * PX + r0)) = pack_bf16x4(xn.x, xn.y, xn.z, xn.w);
                }
              }
            }
          }
          ssp = rows_sum(ssp);
          mxp = rows_umax(mxp);
          if (g == 0 && n < NC) {
            reinterpret_cast<float*>(lds + V::OFF_SSP)[col * NW + w] = ssp;
            reinterpret_cast<unsigned*>(lds + V::OFF_MXP)[col * NW + w] = mxp;
          }
#pragma unroll
          for (int tt = 0; tt < MT_H; ++tt) acc[tt] = *reinterpret_cast<const f32x4*>(b1s + 16 * (w * MT_H + tt) + 4 * g);
          PSTAMP(9);
          __syncthreads();
          PSTAMP(10);
        }
        }
#ifdef ES_PHASE_PROF
        if (blockIdx.x == 0 && lane == 0 && a.prof)
          for (int k = 0; k < 12; ++k) a.prof[w * 16 + k] += prof_acc[k];
#endif
        __syncthreads();   // all reads of the rollout buffers are done before anything is restaged

        // ---------------- outputs of this block of environment copies ----------------
        if (w == 0) {
          const uint32_t cnt = min((uint32_t)NC, a.E - cb * (uint32_t)NC);
          if (g == 0 && (uint32_t)n < cnt) {
            KARG(returns)[(size_t)i * a.E + e] = Rn;
            KARG(ep_len)[(size_t)i * a.E + e] = Ln;
          }
          for (uint32_t r = 0; r < cnt; ++r) fit_sum += __shfl(Rn, (int)r, 64);
        }
      }
      if (tid == 0) KARG(fitness)[i] = fit_sum / (float)a.E;
    }
  }
}

constexpr int env_tiles(int nop, int nw) { return (nop / 16 + nw - 1) / nw > 0 ? (nop / 16 + nw - 1) / nw : 1; }
// The smallest-observation variant leaves half of the register file free: two workgroups (two
// individuals) share a CU and hide each other's LDS round trips and barriers (1.5x at obs 27).
// (Passes of sixteen copies: A stays in LDS - with two workgroups per CU the register file has no four registers to spare
// for its tile, and a spilled tile would be reloaded from scratch memory every step.)
template <int NC, int NW> using V32 = Variant<1, 1, env_tiles(32, NW), NC == 16 ? 0 : 1, NC, NW, 2>;   // obs <= 32,  act <= 16
template <int NC, int NW> using V64 = Variant<2, 1, env_tiles(64, NW), 2, NC, NW>;      // obs <= 64,  act <= 16
// the same two shapes with the environment's products in binary32 (es_config.env_dtype = 1)
template <int NC, int NW> using V32F = Variant<1, 1, env_tiles(32, NW), 1, NC, NW, 2, 0, true>;
template <int NC, int NW> using V64F = Variant<2, 1, env_tiles(64, NW), 2, NC, NW, 1, 0, true>;
template <int NC, int NW> using V128 = Variant<4, 2, env_tiles(128, NW), 4, NC, NW>;    // obs <= 128, act <= 32
// Deeper policies (m = 3, 4 hidden layers) of the two narrow-observation shapes: one workgroup per CU, the
// extra 256 x 256 layers take the registers the second workgroup would have used.
template <int NC, int NW, int ME> using V32D = Variant<1, 1, env_tiles(32, NW), 1, NC, NW, 1, ME>;
template <int NC, int NW, int ME> using V64D = Variant<2, 1, env_tiles(64, NW), 2, NC, NW, 1, ME>;
// A single hidden layer (m = 1) of the same two shapes: the second layer's phase and weights drop out.
template <int NC, int NW> using V32S = Variant<1, 1, env_tiles(32, NW), 1, NC, NW, 2, -1>;
template <int NC, int NW> using V64S = Variant<2, 1, env_tiles(64, NW), 2, NC, NW, 1, -1>;
// obs <= 256, act <= 32.  KTAR of the eight K tiles of the environment matrix A sit in registers, the rest in LDS.  Measured at
// configs[4] (ms per rollout): passes of four copies with tanh 27.5 (all eight in registers) against 28.6 (four); with ReLU the
// register allocation of the epilogue differs and four is better (27.6 against 29.5); passes of sixteen copies have the larger
// working set and four is as fast (37.9 with four episodes per copy either way).
template <int NC, int NW, int KTAR> using V256K = Variant<8, 2, env_tiles(256, NW), KTAR, NC, NW>;
template <int NC, int NW> using V256 = V256K<NC, NW, 4>;

struct VariantInfo { int max_obs, max_act; const char* name; };
static const VariantInfo kVariants[] = {
    {32, 16, "rollout_mfma_reg_bf16<obs32,hid256,act16>"},
    {64, 16, "rollout_mfma_reg_bf16<obs64,hid256,act16>"},
    {128, 32, "rollout_mfma_reg_bf16<obs128,hid256,act32>"},
    {256, 32, "rollout_mfma_reg_bf16<obs256,hid256,act32>"},
};

int mfma_variant_for(const es_config& c) {
  const uint32_t m = c.num_hidden ? c.num_hidden : 2;
  if (c.dtype != 1 || c.hid_dim > (uint32_t)NHP || m < 1 || m > 4) return -1;
  // a binary32 environment is built for the two narrow-observation shapes with two hidden layers
  if (c.env_dtype == 1 && (m != 2 || c.obs_dim > 64 || c.act_dim > 16)) return -1;
  // narrow policies are served better by the one-wavefront-per-episode kernel when it fits
  if (c.hid_dim < 128 && wave_rollout_lds_bytes(c) <= 160 * 1024) return -1;
  for (int v = 0; v < 4; ++v)
    if ((int)c.obs_dim <= kVariants[v].max_obs && (int)c.act_dim <= kVariants[v].max_act)
      return (m != 2 && v > 1) ? -1 : v;      // one, three and four hidden layers: the two narrow-observation shapes only
  return -1;
}

const char* mfma_variant_name(int v) { return (v >= 0 && v < 4) ? kVariants[v].name : "none"; }

template <class V, bool RELU, bool NORM>
static int launch_variant_act(es_ctx* ctx, const MfmaArgs& a, uint32_t units, hipStream_t st) {
  const void* fn = reinterpret_cast<const void*>(rollout_mfma_kernel<V, RELU, NORM>);
  hipError_t err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, V::LDS_BYTES);
  if (err != hipSuccess) return fail(ctx, ES_EHIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(err));
  // persistent grid: as many workgroups as the chip holds at once (register- and LDS-limited)
  const int per_cu = std::min(V::OCC, std::max(1, ctx->lds_limit / V::LDS_BYTES));
  const uint32_t grid = std::min<uint32_t>(units, (uint32_t)(std::max(1, ctx->num_cus) * per_cu));
  hipLaunchKernelGGL((rollout_mfma_kernel<V, RELU, NORM>), dim3(grid), dim3(V::NT), V::LDS_BYTES, st, a);
  return check_launch(ctx, "es_rollout (MFMA)");
}
template <class V>
static int launch_variant(es_ctx* ctx, const MfmaArgs& a, uint32_t units, hipStream_t st) {
  const bool relu = ctx->cfg.hidden_act == 1, norm = ctx->obs_mean != nullptr;
  if (relu) return norm ? launch_variant_act<V, true, true>(ctx, a, units, st) : launch_variant_act<V, true, false>(ctx, a, units, st);
  return norm ? launch_variant_act<V, false, true>(ctx, a, units, st) : launch_variant_act<V, false, false>(ctx, a, units, st);
}

int launch_rollout_mfma(es_ctx* ctx, uint32_t gen, const float* theta, const void* noise, const float* A,
                        const float* B, float* returns, int32_t* ep_len, float* fitness, void* ws,
                        hipStream_t st) {
  const Shape& s = ctx->shp;
  const es_config& c = ctx->cfg;
  MfmaArgs a;
  const NoiseView nv = noise_view(ctx, noise);
  a.theta = theta; a.noise = nv.base; a.noise_offs = nv.offs; a.A = A; a.B = B; a.obs_mean = ctx->obs_mean; a.obs_inv = ctx->obs_inv_std; a.returns = returns; a.ep_len = ep_len; a.fitness = fitness;
  a.N = s.N; a.E = s.E; a.T = s.T; a.no = s.no; a.nh = s.nh; a.na = s.na; a.ld = s.ld;
  a.oW1 = s.oW1; a.ob1 = s.ob1; a.oW2 = s.oW2; a.ob2 = s.ob2; a.oW3 = s.oW3; a.ob3 = s.ob3;
  a.gen = gen; a.k0 = (uint32_t)c.seed; a.k1 = (uint32_t)(c.seed >> 32);
  a.antithetic = c.antithetic; a.out_tanh = c.out_tanh; a.noise_mode = nv.mode;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  a.prof = static_cast<unsigned long long*>(ws);
  if ((int)V256<16, 4>::LDS_BYTES > ctx->lds_limit)
    return fail(ctx, ES_EUNSUPPORTED, "es_rollout: this device's LDS is too small for the register-resident kernel");
  const uint32_t units = s.N;      // one work item per individual
  const bool narrow = s.E <= 4;     // passes of 4 environment copies with column compaction
#ifdef ES_DEV_FAST   // tuning builds only: one variant, seconds to compile
  if (c.env_dtype == 1 && ctx->mfma_variant == 0 && ctx->cfg.hidden_act == 0 && !ctx->obs_mean)
    return launch_variant_act<V32F<16, 4>, false, false>(ctx, a, units, st);
  if (ctx->mfma_variant == 3 && narrow && s.m == 2 && ctx->cfg.hidden_act == 0 && !ctx->obs_mean)
    return launch_variant_act<V256K<4, 4, 8>, false, false>(ctx, a, units, st);
  if (ctx->mfma_variant == 0 && !narrow && s.m == 2 && ctx->cfg.hidden_act == 0 && !ctx->obs_mean)
    return launch_variant_act<V32<16, 4>, false, false>(ctx, a, units, st);
  return fail(ctx, ES_EUNSUPPORTED, "tuning build: variant not compiled");
#else
  if (c.env_dtype == 1) {          // binary32 environment: passes of 16 copies whatever E is
    if (ctx->mfma_variant == 0) return launch_variant<V32F<16, 4>>(ctx, a, units, st);
    if (ctx->mfma_variant == 1) return launch_variant<V64F<16, 4>>(ctx, a, units, st);
    return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident variant with a binary32 environment for this shape");
  }
  if (s.m == 1) {
    if (ctx->mfma_variant == 0) return narrow ? launch_variant<V32S<4, 4>>(ctx, a, units, st) : launch_variant<V32S<16, 4>>(ctx, a, units, st);
    if (ctx->mfma_variant == 1) return narrow ? launch_variant<V64S<4, 4>>(ctx, a, units, st) : launch_variant<V64S<16, 4>>(ctx, a, units, st);
  } else if (s.m == 3) {
    if (ctx->mfma_variant == 0) return narrow ? launch_variant<V32D<4, 4, 1>>(ctx, a, units, st) : launch_variant<V32D<16, 4, 1>>(ctx, a, units, st);
    if (ctx->mfma_variant == 1) return narrow ? launch_variant<V64D<4, 4, 1>>(ctx, a, units, st) : launch_variant<V64D<16, 4, 1>>(ctx, a, units, st);
  } else if (s.m == 4) {
    if (ctx->mfma_variant == 0) return narrow ? launch_variant<V32D<4, 4, 2>>(ctx, a, units, st) : launch_variant<V32D<16, 4, 2>>(ctx, a, units, st);
    if (ctx->mfma_variant == 1) return narrow ? launch_variant<V64D<4, 4, 2>>(ctx, a, units, st) : launch_variant<V64D<16, 4, 2>>(ctx, a, units, st);
  }
  if (s.m != 2) return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident variant for this depth");
  switch (ctx->mfma_variant) {
    case 0: return narrow ? launch_variant<V32<4, 4>>(ctx, a, units, st) : launch_variant<V32<16, 4>>(ctx, a, units, st);
    case 1: return narrow ? launch_variant<V64<4, 4>>(ctx, a, units, st) : launch_variant<V64<16, 4>>(ctx, a, units, st);
    case 2: return narrow ? launch_variant<V128<4, 4>>(ctx, a, units, st) : launch_variant<V128<16, 4>>(ctx, a, units, st);
    case 3: {
      if (!narrow) return launch_variant<V256<16, 4>>(ctx, a, units, st);
      const bool norm = ctx->obs_mean != nullptr;
      if (ctx->cfg.hidden_act == 1) return norm ? launch_variant_act<V256K<4, 4, 4>, true, true>(ctx, a, units, st) : launch_variant_act<V256K<4, 4, 4>, true, false>(ctx, a, units, st);
      return norm ? launch_variant_act<V256K<4, 4, 8>, false, true>(ctx, a, units, st) : launch_variant_act<V256K<4, 4, 8>, false, false>(ctx, a, units, st);
    }
    default: return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident variant for this shape");
  }
#endif
}

}  // namespace es
