// es_rollout, register-resident binary32 variant for narrow policies (hidden width <= 64).
//
// Paper Sec. 3.2 / 5.2: population x environment-copy evaluation of a deterministic
// two-hidden-layer MLP policy, fitness = mean undiscounted return.  One wavefront runs one
// (individual, environment copy) episode; lane u owns hidden unit u, and the state vector is spread
// over the four 16-lane rows of the wavefront (element k in row k % 4, column k / 4).  The individual's
// perturbed weights (theta + sign*sigma*eps, fused into the load) and the environment matrices live in
// registers for all T steps.
// Every matrix-vector product broadcasts its inputs within the 16-lane rows by DPP, fused into the
// multiply-add (v_fmac_f32_dpp ... row_newbcast:j, one instruction per multiply-add, no scalar hop):
// the lane in row r, column c adds up the inputs that live in ITS row into partial sums for the outputs
// that belong to ITS column (hidden units c, c + 16, ...; state elements 4 c .. 4 c + 3), and two
// row-swap stages (v_permlane32_swap, v_permlane16_swap + add) add the four rows' partial sums and
// leave each output's total in the lane that owns it.  The reward norms are reduced the same way and end
// in lane 15.  No LDS, no barriers, one scalar read per step (the termination test).
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
  uint32_t antithetic, noise_mode;
  float sigma, done_thresh, act_cost;
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_zero(float v) {      // lanes without a source (or masked off) read 0
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, ROW_MASK == 0xF));
}
// The matrix-vector products.  "v_fmac_f32_dpp acc, h, w row_newbcast:j" adds w * (lane j of h's 16-lane row) to acc: the
// input element is broadcast within each row by the DPP modifier, fused into the multiply-add - one instruction per
// multiply-add, no scalar hop.  The compiler folds a DPP move into v_mul / v_add but not into v_fmac, so the runs below
// are inline assembly.  Its hazard checks do not look inside inline assembly: a vector ALU write of `h` must be two
// wait states away from the first DPP read, hence the s_nop that leads every run.  A run starts with multiplies (no
// zeroed accumulators) and interleaves its accumulators, so that consecutive instructions never depend on each other.
#define ES_DPP_TAIL(J) " row_newbcast:" #J " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
#define ES_MUL(ACC, H, OP, J) "v_mul_f32_dpp %" #ACC ", %" #H ", %" #OP ES_DPP_TAIL(J)
#define ES_MAC(ACC, H, OP, J) "v_fmac_f32_dpp %" #ACC ", %" #H ", %" #OP ES_DPP_TAIL(J)

// o_q = sum_{j < N} w[N q + j] * (lane j of h's row), q = 0..3
template <int N>
__device__ __forceinline__ void row_bcast_dot_x4(float& o0, float& o1, float& o2, float& o3, float h, const float (&w)[4 * N]) {
  static_assert(N == 3 || N == 5 || N == 16, "run lengths the register-resident shapes need");
  if constexpr (N == 3)
    asm volatile("s_nop 1\n\t"
      ES_MUL(0, 4, 5, 0) ES_MUL(1, 4, 8, 0) ES_MUL(2, 4, 11, 0) ES_MUL(3, 4, 14, 0)
      ES_MAC(0, 4, 6, 1) ES_MAC(1, 4, 9, 1) ES_MAC(2, 4, 12, 1) ES_MAC(3, 4, 15, 1)
      ES_MAC(0, 4, 7, 2) ES_MAC(1, 4, 10, 2) ES_MAC(2, 4, 13, 2) ES_MAC(3, 4, 16, 2)
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(h),
        "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]), "v"(w[8]), "v"(w[9]), "v"(w[10]),
        "v"(w[11]));
  else if constexpr (N == 5)
    asm volatile("s_nop 1\n\t"
      ES_MUL(0, 4, 5, 0) ES_MUL(1, 4, 10, 0) ES_MUL(2, 4, 15, 0) ES_MUL(3, 4, 20, 0)
      ES_MAC(0, 4, 6, 1) ES_MAC(1, 4, 11, 1) ES_MAC(2, 4, 16, 1) ES_MAC(3, 4, 21, 1)
      ES_MAC(0, 4, 7, 2) ES_MAC(1, 4, 12, 2) ES_MAC(2, 4, 17, 2) ES_MAC(3, 4, 22, 2)
      ES_MAC(0, 4, 8, 3) ES_MAC(1, 4, 13, 3) ES_MAC(2, 4, 18, 3) ES_MAC(3, 4, 23, 3)
      ES_MAC(0, 4, 9, 4) ES_MAC(1, 4, 14, 4) ES_MAC(2, 4, 19, 4) ES_MAC(3, 4, 24, 4)
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(h),
        "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]), "v"(w[8]), "v"(w[9]), "v"(w[10]),
        "v"(w[11]), "v"(w[12]), "v"(w[13]), "v"(w[14]), "v"(w[15]), "v"(w[16]), "v"(w[17]), "v"(w[18]), "v"(w[19]));
  else
    asm volatile("s_nop 1\n\t"
      ES_MUL(0, 4, 5, 0) ES_MUL(1, 4, 21, 0) ES_MUL(2, 4, 37, 0) ES_MUL(3, 4, 53, 0)
      ES_MAC(0, 4, 6, 1) ES_MAC(1, 4, 22, 1) ES_MAC(2, 4, 38, 1) ES_MAC(3, 4, 54, 1)
      ES_MAC(0, 4, 7, 2) ES_MAC(1, 4, 23, 2) ES_MAC(2, 4, 39, 2) ES_MAC(3, 4, 55, 2)
      ES_MAC(0, 4, 8, 3) ES_MAC(1, 4, 24, 3) ES_MAC(2, 4, 40, 3) ES_MAC(3, 4, 56, 3)
      ES_MAC(0, 4, 9, 4) ES_MAC(1, 4, 25, 4) ES_MAC(2, 4, 41, 4) ES_MAC(3, 4, 57, 4)
      ES_MAC(0, 4, 10, 5) ES_MAC(1, 4, 26, 5) ES_MAC(2, 4, 42, 5) ES_MAC(3, 4, 58, 5)
      ES_MAC(0, 4, 11, 6) ES_MAC(1, 4, 27, 6) ES_MAC(2, 4, 43, 6) ES_MAC(3, 4, 59, 6)
      ES_MAC(0, 4, 12, 7) ES_MAC(1, 4, 28, 7) ES_MAC(2, 4, 44, 7) ES_MAC(3, 4, 60, 7)
      ES_MAC(0, 4, 13, 8) ES_MAC(1, 4, 29, 8) ES_MAC(2, 4, 45, 8) ES_MAC(3, 4, 61, 8)
      ES_MAC(0, 4, 14, 9) ES_MAC(1, 4, 30, 9) ES_MAC(2, 4, 46, 9) ES_MAC(3, 4, 62, 9)
      ES_MAC(0, 4, 15, 10) ES_MAC(1, 4, 31, 10) ES_MAC(2, 4, 47, 10) ES_MAC(3, 4, 63, 10)
      ES_MAC(0, 4, 16, 11) ES_MAC(1, 4, 32, 11) ES_MAC(2, 4, 48, 11) ES_MAC(3, 4, 64, 11)
      ES_MAC(0, 4, 17, 12) ES_MAC(1, 4, 33, 12) ES_MAC(2, 4, 49, 12) ES_MAC(3, 4, 65, 12)
      ES_MAC(0, 4, 18, 13) ES_MAC(1, 4, 34, 13) ES_MAC(2, 4, 50, 13) ES_MAC(3, 4, 66, 13)
      ES_MAC(0, 4, 19, 14) ES_MAC(1, 4, 35, 14) ES_MAC(2, 4, 51, 14) ES_MAC(3, 4, 67, 14)
      ES_MAC(0, 4, 20, 15) ES_MAC(1, 4, 36, 15) ES_MAC(2, 4, 52, 15) ES_MAC(3, 4, 68, 15)
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(h),
        "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]), "v"(w[8]), "v"(w[9]), "v"(w[10]),
        "v"(w[11]), "v"(w[12]), "v"(w[13]), "v"(w[14]), "v"(w[15]), "v"(w[16]), "v"(w[17]), "v"(w[18]), "v"(w[19]), "v"(w[20]), "v"(w[21]),
        "v"(w[22]), "v"(w[23]), "v"(w[24]), "v"(w[25]), "v"(w[26]), "v"(w[27]), "v"(w[28]), "v"(w[29]), "v"(w[30]), "v"(w[31]), "v"(w[32]),
        "v"(w[33]), "v"(w[34]), "v"(w[35]), "v"(w[36]), "v"(w[37]), "v"(w[38]), "v"(w[39]), "v"(w[40]), "v"(w[41]), "v"(w[42]), "v"(w[43]),
        "v"(w[44]), "v"(w[45]), "v"(w[46]), "v"(w[47]), "v"(w[48]), "v"(w[49]), "v"(w[50]), "v"(w[51]), "v"(w[52]), "v"(w[53]), "v"(w[54]),
        "v"(w[55]), "v"(w[56]), "v"(w[57]), "v"(w[58]), "v"(w[59]), "v"(w[60]), "v"(w[61]), "v"(w[62]), "v"(w[63]));
}
// the same for two accumulators (hidden width 32)
template <int N>
__device__ __forceinline__ void row_bcast_dot_x2(float& o0, float& o1, float h, const float (&w)[2 * N]) {
  static_assert(N == 3 || N == 16, "run lengths the register-resident shapes need");
  if constexpr (N == 3)
    asm volatile("s_nop 1\n\t"
      ES_MUL(0, 2, 3, 0) ES_MUL(1, 2, 6, 0)
      ES_MAC(0, 2, 4, 1) ES_MAC(1, 2, 7, 1)
      ES_MAC(0, 2, 5, 2) ES_MAC(1, 2, 8, 2)
      : "=&v"(o0), "=&v"(o1)
      : "v"(h),
        "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]));
  else
    asm volatile("s_nop 1\n\t"
      ES_MUL(0, 2, 3, 0) ES_MUL(1, 2, 19, 0)
      ES_MAC(0, 2, 4, 1) ES_MAC(1, 2, 20, 1)
      ES_MAC(0, 2, 5, 2) ES_MAC(1, 2, 21, 2)
      ES_MAC(0, 2, 6, 3) ES_MAC(1, 2, 22, 3)
      ES_MAC(0, 2, 7, 4) ES_MAC(1, 2, 23, 4)
      ES_MAC(0, 2, 8, 5) ES_MAC(1, 2, 24, 5)
      ES_MAC(0, 2, 9, 6) ES_MAC(1, 2, 25, 6)
      ES_MAC(0, 2, 10, 7) ES_MAC(1, 2, 26, 7)
      ES_MAC(0, 2, 11, 8) ES_MAC(1, 2, 27, 8)
      ES_MAC(0, 2, 12, 9) ES_MAC(1, 2, 28, 9)
      ES_MAC(0, 2, 13, 10) ES_MAC(1, 2, 29, 10)
      ES_MAC(0, 2, 14, 11) ES_MAC(1, 2, 30, 11)
      ES_MAC(0, 2, 15, 12) ES_MAC(1, 2, 31, 12)
      ES_MAC(0, 2, 16, 13) ES_MAC(1, 2, 32, 13)
      ES_MAC(0, 2, 17, 14) ES_MAC(1, 2, 33, 14)
      ES_MAC(0, 2, 18, 15) ES_MAC(1, 2, 34, 15)
      : "=&v"(o0), "=&v"(o1)
      : "v"(h),
        "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]), "v"(w[8]), "v"(w[9]), "v"(w[10]),
        "v"(w[11]), "v"(w[12]), "v"(w[13]), "v"(w[14]), "v"(w[15]), "v"(w[16]), "v"(w[17]), "v"(w[18]), "v"(w[19]), "v"(w[20]), "v"(w[21]),
        "v"(w[22]), "v"(w[23]), "v"(w[24]), "v"(w[25]), "v"(w[26]), "v"(w[27]), "v"(w[28]), "v"(w[29]), "v"(w[30]), "v"(w[31]));
}
// sum_{j < 16} w[j] * (lane j of h's row), in four interleaved partial sums
__device__ __forceinline__ float row_bcast_dot16(float h, const float (&w)[16]) {
  float o0, o1, o2, o3;
  asm volatile("s_nop 1\n\t"
      ES_MUL(0, 4, 5, 0) ES_MUL(1, 4, 6, 1) ES_MUL(2, 4, 7, 2) ES_MUL(3, 4, 8, 3)
      ES_MAC(0, 4, 9, 4) ES_MAC(1, 4, 10, 5) ES_MAC(2, 4, 11, 6) ES_MAC(3, 4, 12, 7)
      ES_MAC(0, 4, 13, 8) ES_MAC(1, 4, 14, 9) ES_MAC(2, 4, 15, 10) ES_MAC(3, 4, 16, 11)
      ES_MAC(0, 4, 17, 12) ES_MAC(1, 4, 18, 13) ES_MAC(2, 4, 19, 14) ES_MAC(3, 4, 20, 15)
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(h),
        "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]), "v"(w[8]), "v"(w[9]), "v"(w[10]),
        "v"(w[11]), "v"(w[12]), "v"(w[13]), "v"(w[14]), "v"(w[15]));
  return (o0 + o1) + (o2 + o3);
}
// acc + sum_{j < N} w[j] * (lane j of h's row): the short action term of the environment step
template <int N>
__device__ __forceinline__ float row_bcast_mac(float acc, float h, const float (&w)[N]) {
  static_assert(N == 3 || N == 6, "action widths of the register-resident shapes");
  if constexpr (N == 3)
    asm volatile("s_nop 1\n\t" ES_MAC(0, 1, 2, 0) ES_MAC(0, 1, 3, 1) ES_MAC(0, 1, 4, 2)
                 : "+v"(acc) : "v"(h), "v"(w[0]), "v"(w[1]), "v"(w[2]));
  else
    asm volatile("s_nop 1\n\t" ES_MAC(0, 1, 2, 0) ES_MAC(0, 1, 3, 1) ES_MAC(0, 1, 4, 2) ES_MAC(0, 1, 5, 3) ES_MAC(0, 1, 6, 4) ES_MAC(0, 1, 7, 5)
                 : "+v"(acc) : "v"(h), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]));
  return acc;
}
#undef ES_MAC
#undef ES_MUL
#undef ES_DPP_TAIL
// x + (the same register of the other 16-lane row of the pair / of the other half), via the row-swap instructions
__device__ __forceinline__ float swap16_add(float x, float y) {   // rows (0,1,2,3) <- x0+y... see the caller
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
// sum over the lanes of each 16-lane row, result in lane 15 of the row (lanes without a source read 0)
__device__ __forceinline__ float row_total(float v) {
  v += dpp_zero<0x111, 0xF>(v);
  v += dpp_zero<0x112, 0xF>(v);
  v += dpp_zero<0x114, 0xF>(v);
  return v + dpp_zero<0x118, 0xF>(v);
}

// RELU / OUT_TANH: the activations are compile-time choices, and lanes that own no unit need no masking (their weights
// and biases are zero, and both activations map 0 to 0), so a step is one straight-line block: a taken branch costs
// this single in-order wavefront more than the few instructions it would skip.
template <int NO, int NH, int NA, bool RELU, bool OUT_TANH, bool NORM>
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
  const bool hid = u < NH;
  // Lane (row lr, column lc).  Hidden unit u lives in lane u.  The state is spread over the four rows so that every row
  // holds a quarter of it: element k sits in row k % 4, column k / 4 - then a row-broadcast run of CJ = ceil(obs / 4)
  // multiply-adds per output covers a whole observation-wide product, all four rows working.
  const int lr = u >> 4, lc = u & 15;
  constexpr int CJ = (NO + 3) / 4;
  const int ks = 4 * lc + lr;                    // the state element of this lane
  const bool sval = lc < CJ && ks < NO;

  const void* nbase = a.noise;      // shared table: this individual's row, addressed as row 0
  uint32_t nrow = row;
  if (a.noise_offs) { nbase = table_row_base(a.noise_mode, a.noise, a.noise_offs, row); nrow = 0u; }
  auto param = [&](uint32_t d) -> float {     // perturbed parameter d of individual i (binary32, one rounding)
    return __fmaf_rn(scale, noise_value(a.noise_mode, nbase, a.ld, nrow, d, a.gen, a.k0, a.k1), a.theta[d]);
  };

  // ---- this lane's weights ----
  // first layer: partial sums of the units lc, lc + 16, ... over the inputs of row lr: w1[CJ q + j] = W1[lc + 16 q][4 j + lr]
  // second layer and action layer: the same over the 16 hidden units of row lr: w2[16 q + j] = W2[lc + 16 q][16 lr + j],
  //   w3[j] = W3[lc][16 lr + j]
  // environment: partial sums of the four state elements of column lc: ar[CJ r + j] = A[4 lc + r][4 j + lr];
  //   action term of this lane's own element: br[c] = B[ks][c]
  float w1[NQ * CJ], w2[NH], w3[16], ar[4 * CJ], br[NA];
  float b1 = 0.f, b2 = 0.f, b3 = 0.f;
#pragma unroll
  for (int qq = 0; qq < NQ; ++qq)
#pragma unroll
    for (int j = 0; j < CJ; ++j) w1[CJ * qq + j] = (4 * j + lr < NO) ? param(oW1 + (uint32_t)(lc + 16 * qq) * NO + 4 * j + lr) : 0.f;
#pragma unroll
  for (int qq = 0; qq < NQ; ++qq) {
    const uint32_t d0 = oW2 + (uint32_t)(lc + 16 * qq) * NH + 16u * (uint32_t)lr;     // sixteen consecutive parameters
#pragma unroll
    for (int j = 0; j < 16; ++j) w2[16 * qq + j] = hid ? param(d0 + j) : 0.f;
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) w3[j] = (hid && lc < NA) ? param(oW3 + (uint32_t)lc * NH + 16u * (uint32_t)lr + j) : 0.f;
  if (hid) { b1 = param(ob1 + u); b2 = param(ob2 + u); }
  if (lc < NA) b3 = param(ob3 + lc);            // in every row: the action vector is kept once per row
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int j = 0; j < CJ; ++j)
      ar[CJ * r + j] = (lc < CJ && 4 * lc + r < NO && 4 * j + lr < NO) ? a.A[(4 * lc + r) * NO + 4 * j + lr] : 0.f;
#pragma unroll
  for (int c = 0; c < NA; ++c) br[c] = sval ? a.B[ks * NA + c] : 0.f;

  // frozen observation statistics of this lane's state element (NORM: a context with statistics set)
  const float mu = (NORM && sval) ? a.obs_mean[ks] : 0.f;
  const float iv = (NORM && sval) ? a.obs_inv[ks] : 1.f;
  float s = sval ? reset_value((uint32_t)ks, e, a.gen, a.k0, a.k1) : 0.f;
  float R = 0.f;                      // per-lane share of the return
  int32_t len = 0;
  const float inv_no = 1.0f / (float)NO, quarter_cost = 0.25f * a.act_cost;

  for (uint32_t t = 0; t < a.T; ++t) {
    // h1 = tanh(W1 s + b1)
    const float xp = NORM ? (s - mu) * iv : s;      // the policy's input (paper App. B: fixed normalisation statistics)
    float l1;
    if constexpr (NQ == 4) {
      float p0, p1, p2, p3;
      row_bcast_dot_x4<CJ>(p0, p1, p2, p3, xp, w1);
      l1 = rows_transpose_add(p0, p1, p2, p3);
    } else {
      float p0, p1;
      row_bcast_dot_x2<CJ>(p0, p1, xp, w1);
      l1 = rows_transpose_add(p0, p1);
    }
    l1 += b1;
    const float h1 = RELU ? fmaxf(l1, 0.f) : tanh_fast(l1);
    // h2 = tanh(W2 h1 + b2): every lane accumulates over its own row's inputs (row-broadcast DPP multiply-adds),
    // then the rows' partial sums are added and moved to the lane of their unit by two row-swap stages
    float l2;
    if constexpr (NQ == 4) {
      float p0, p1, p2, p3;
      row_bcast_dot_x4<16>(p0, p1, p2, p3, h1, w2);
      l2 = rows_transpose_add(p0, p1, p2, p3);
    } else {
      float p0, p1;
      row_bcast_dot_x2<16>(p0, p1, h1, w2);
      l2 = swap16_add(p0, p1);          // the units' own rows 0 and 1 hold all of their inputs; rows 2 and 3 have zero weights
    }
    l2 += b2;
    const float h2 = RELU ? fmaxf(l2, 0.f) : tanh_fast(l2);
    // a = tanh(W3 h2 + b3): row-broadcast multiply-adds as above, the four rows' partial sums added by two row swaps;
    // column c of every row then holds unit c's total, and one tanh serves all units
    float pv = row_bcast_dot16(h2, w3);
    pv = swap16_add(pv, pv);
    pv = swap32_add(pv, pv);
    pv = pv + b3;
    const float tv = OUT_TANH ? tanh_fast(pv) : pv;      // columns >= act: weights and bias are zero
    // reward from the pre-step state, 1 - |s|^2 / obs - cost |a|^2: a sum over all 64 lanes (the action vector is held
    // once per row, hence the quarter)
    R += __fmaf_rn(-inv_no * s, s, -quarter_cost * (tv * tv));      // this lane's share; the lanes are added after the last step
    len += 1;
    // s' = tanh(A s + B a): partial sums of the four elements of this column over the inputs of this row, rows added
    // and moved to their element's lane; the action term straight from the row's action vector
    float pre;
    {
      float e0, e1, e2, e3;
      row_bcast_dot_x4<CJ>(e0, e1, e2, e3, s, ar);
      pre = rows_transpose_add(e0, e1, e2, e3);
    }
    pre = row_bcast_mac<NA>(pre, tv, br);
    s = tanh_fast(pre);                                  // lanes without a state element: zero weights, tanh(0) = 0
    if (__ballot(fabsf(s) > a.done_thresh) != 0ull) break;       // max |s| > threshold: some lane exceeds it
  }
  const float r2 = swap16_add(R, R);
  R = (float)len + row_total(swap32_add(r2, r2));      // ends in lane 15
  if (u == 15) {
    a.returns[(size_t)i * a.E + e] = R;
    a.ep_len[(size_t)i * a.E + e] = len;
  }
}

template <int O, int H, int A> struct RegWidths { static constexpr int no = O, nh = H, na = A; };
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
  a.antithetic = c.antithetic; a.noise_mode = nv.mode;
  a.sigma = c.sigma; a.done_thresh = c.done_thresh; a.act_cost = c.act_cost;
  const dim3 grid(s.N * s.E), block(64);
  const bool relu = c.hidden_act == 1, otanh = c.out_tanh != 0, norm = ctx->obs_mean != nullptr;
  auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, st, a); };
  auto pick = [&](auto shape) {       // shape carries the three widths; the activations and the statistics select the variant
    constexpr int O = decltype(shape)::no, H = decltype(shape)::nh, A = decltype(shape)::na;
    const int v = (relu ? 4 : 0) | (otanh ? 2 : 0) | (norm ? 1 : 0);
    switch (v) {
      case 0: go(rollout_reg_kernel<O, H, A, false, false, false>); break;
      case 1: go(rollout_reg_kernel<O, H, A, false, false, true>); break;
      case 2: go(rollout_reg_kernel<O, H, A, false, true, false>); break;
      case 3: go(rollout_reg_kernel<O, H, A, false, true, true>); break;
      case 4: go(rollout_reg_kernel<O, H, A, true, false, false>); break;
      case 5: go(rollout_reg_kernel<O, H, A, true, false, true>); break;
      case 6: go(rollout_reg_kernel<O, H, A, true, true, false>); break;
      default: go(rollout_reg_kernel<O, H, A, true, true, true>); break;
    }
  };
  switch (ctx->reg_variant) {
    case 0: pick(RegWidths<11, 32, 3>{}); break;
    case 1: pick(RegWidths<17, 64, 6>{}); break;
    default: return fail(ctx, ES_EUNSUPPORTED, "es_rollout: no register-resident binary32 variant for this shape");
  }
  int rc = check_launch(ctx, "es_rollout (register-resident f32)");
  if (rc != ES_OK) return rc;
  return launch_fitness(ctx, returns, fitness, st);
}

}  // namespace es
