/*
 * CPU checker ("oracle") for one OpenES generation: TEST INFRASTRUCTURE ONLY.
 *
 * This file is the definition of "right" that the HIP library is compared
 * against.  It is plain, slow, sequential C: nested loops over individuals,
 * environments and steps, no blocking, no fusion, no reordering.  It shares no
 * code, header, table or constant generator with the HIP path and is never on
 * the product path: only the tests, the smoke check and the benchmark's
 * CPU-baseline leg may load it.
 *
 * What it follows (paper = arXiv 2501.15129):
 *   - Sec. 3.2 "Computation model": every individual of the population is
 *     evaluated at once, each on several parallel environment copies
 *     (two-level vectorisation: agents x environments).
 *   - Sec. 5.2: deterministic two-hidden-layer MLP policy; fitness = mean
 *     undiscounted episodic return over the episodes, no action noise.
 *   - Sec. 5.1 / App. B Table 5(b): OpenES with Adam, learning rate 0.01,
 *     weight decay 0.005, noise std 0.02; noise generated on the fly each
 *     generation rather than read from a pre-built table.
 * The paper leaves the numerics of OpenES to its citation (Salimans et al.
 * 2017); every finer choice made here (counter layout, Gaussian transform,
 * mirrored sampling, centred ranks, gradient scale, bf16 placement, reward /
 * termination indexing) is a stated reading, listed in the design notes.
 *
 * Precision: integer work (Philox words, ranks, episode lengths) is exact.
 * The Gaussian transform and the perturbation are *defined* as a fixed
 * sequence of IEEE-754 binary32 operations (so they are bit-reproducible);
 * they are evaluated exactly as written, with contraction disabled
 * (-ffp-contract=off) and explicit fmaf.  Everything tolerance-checked
 * (rollout arithmetic, gradient estimate, Adam) is computed in binary64.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors of the published
 * generator; Gaussian vs. a libm binary64 Box-Muller of the same integers and
 * sample moments; rollout special cases with closed forms, a library
 * (torch.nn.functional) one-step evaluation and a pure-Python enumeration;
 * ranks vs. a stable library sort; gradient estimate vs. its closed form on a
 * quadratic; Adam vs. torch.optim.Adam.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_config {
  uint32_t pop;          /* N */
  uint32_t envs;         /* E */
  uint32_t horizon;      /* T */
  uint32_t obs, hid, act;
  uint32_t dtype;        /* 0 fp32 ; 1 bf16 contraction operands */
  uint32_t noise_dtype;  /* 0 fp32 ; 1 noise rounded to bf16 */
  uint32_t antithetic;
  uint32_t out_tanh;
  float sigma, lr, beta1, beta2, adam_eps, weight_decay;
  float done_thresh, act_cost;
  uint64_t seed;
  uint32_t hidden_act;   /* hidden-layer activation: 0 tanh ; 1 ReLU (paper App. B: the EA experiments use ReLU MLPs) */
  uint32_t num_hidden;   /* m hidden layers of width hid (paper Sec. 5.1 varies m; the base case is 2); 0 means 2 */
  uint32_t episodes;     /* episodes run one after the other in every environment copy, the environment resetting
                            itself in between (paper Sec. 3.1: the auto-reset wrapper); 0 means 1 */
  uint32_t env_dtype;    /* only with dtype = 1.  0: the environment's products use bf16 operands too (A, B, the state and
                            the action as operands of A s + B a are rounded to bf16); 1: the environment stays in
                            binary32 - only the POLICY has "bf16 weights and activations", the simulator it acts on
                            is not part of the policy's precision */
} orc_config;

enum { STREAM_NOISE = 1, STREAM_RESET = 2, STREAM_TABLE = 3, STREAM_OFFSET = 4 };

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: */
/* as easy as 1, 2, 3", SC'11).  128-bit counter, 64-bit key.           */
/* ------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void stream_block(const orc_config *cfg, uint32_t block, uint32_t row, uint64_t gen,
                         uint32_t stream, uint32_t out[4]) {
  uint32_t ctr[4] = {block, row, (uint32_t)gen, stream};
  uint32_t key[2] = {(uint32_t)cfg->seed, (uint32_t)(cfg->seed >> 32)};
  orc_philox4x32_10(ctr, key, out);
}

static float f32_from_bits(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t bits_from_f32(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

/* bf16 round-to-nearest-even of a finite binary32 value, returned as binary32. */
float orc_bf16_round(float x) {
  uint32_t b = bits_from_f32(x);
  b += 0x7FFFu + ((b >> 16) & 1u);
  b &= 0xFFFF0000u;
  return f32_from_bits(b);
}

/* ------------------------------------------------------------------ */
/* Gaussian transform: two 32-bit words -> two N(0,1) variates.         */
/* Box-Muller on u1 = k1 / 2^24 (k1 in [1, 2^24]) and angle             */
/* 2 pi k2 / 2^24, written as a fixed binary32 operation sequence:      */
/*   -ln u1 = n ln2 - ln m,  u1 = m 2^-n,  m in (sqrt(1/2), sqrt 2],    */
/*   ln m = 2 atanh((m-1)/(m+1)) by its odd series through s^11;        */
/*   sin / cos on [0, pi/4] by Taylor polynomials, octant symmetry.     */
/* ------------------------------------------------------------------ */
void orc_gauss_pair(uint32_t xa, uint32_t xb, float z[2]) {
  uint32_t k1 = (xa >> 8) + 1u;
  uint32_t k2 = xb >> 8;

  uint32_t fb = bits_from_f32((float)k1);               /* exact: k1 <= 2^24 */
  int e = (int)(fb >> 23) - 127;
  float m = f32_from_bits((fb & 0x007FFFFFu) | 0x3F800000u);
  if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
  int n = 24 - e;
  float s = (m - 1.0f) / (m + 1.0f);
  float t = s * s;
  float p = (float)(1.0 / 11.0);
  p = fmaf(t, p, (float)(1.0 / 9.0));
  p = fmaf(t, p, (float)(1.0 / 7.0));
  p = fmaf(t, p, (float)(1.0 / 5.0));
  p = fmaf(t, p, (float)(1.0 / 3.0));
  p = fmaf(t, p, 1.0f);
  float lnm = s * p;
  lnm = lnm + lnm;
  float neg_ln_u = fmaf((float)n, 0.693147182f, -lnm);
  float rad = sqrtf(neg_ln_u + neg_ln_u);

  uint32_t oct = k2 >> 21;
  uint32_t f = k2 & 0x1FFFFFu;
  if (oct & 1u) f = 0x200000u - f;
  float x = ((float)f * 0.785398185f) * 4.76837158203125e-07f;   /* * 2^-21 */
  float y = x * x;
  float sp = (float)(1.0 / 362880.0);
  sp = fmaf(y, sp, (float)(-1.0 / 5040.0));
  sp = fmaf(y, sp, (float)(1.0 / 120.0));
  sp = fmaf(y, sp, (float)(-1.0 / 6.0));
  sp = fmaf(y, sp, 1.0f);
  sp = x * sp;
  float cp = (float)(-1.0 / 3628800.0);
  cp = fmaf(y, cp, (float)(1.0 / 40320.0));
  cp = fmaf(y, cp, (float)(-1.0 / 720.0));
  cp = fmaf(y, cp, (float)(1.0 / 24.0));
  cp = fmaf(y, cp, -0.5f);
  cp = fmaf(y, cp, 1.0f);

  float c, sn;
  switch (oct) {
    case 0: c = cp;  sn = sp;  break;
    case 1: c = sp;  sn = cp;  break;
    case 2: c = -sp; sn = cp;  break;
    case 3: c = -cp; sn = sp;  break;
    case 4: c = -cp; sn = -sp; break;
    case 5: c = -sp; sn = -cp; break;
    case 6: c = sp;  sn = -cp; break;
    default: c = cp; sn = -sp; break;
  }
  z[0] = rad * c;
  z[1] = rad * sn;
}

static uint32_t noise_rows(const orc_config *cfg) { return cfg->antithetic ? cfg->pop / 2 : cfg->pop; }

static uint32_t hidden_layers(const orc_config *cfg) { return cfg->num_hidden ? cfg->num_hidden : 2u; }

/* obs -> hid, (m - 1) x (hid -> hid), hid -> act, every layer with a bias. */
size_t orc_param_count(const orc_config *cfg) {
  size_t o = cfg->obs, h = cfg->hid, a = cfg->act, m = hidden_layers(cfg);
  return (o + 1) * h + (m - 1) * (h + 1) * h + (h + 1) * a;
}

/* Noise matrix eps[j, d], j < rows, d < D, dense row-major binary32.
 * Element d of row j is variate (d mod 4) of the Philox block with counter
 * (d / 4, j, generation, STREAM_NOISE); variates (0,1) come from words (0,1),
 * variates (2,3) from words (2,3).  With noise_dtype = 1 each value is then
 * rounded to bf16 and THAT value is the noise everywhere downstream.
 * orc_sample_rows writes rows j0 <= j < j1 only (output indexed from j0). */
void orc_sample_rows(const orc_config *cfg, uint64_t gen, uint32_t j0, uint32_t j1, float *noise) {
  size_t D = orc_param_count(cfg);
#pragma omp parallel for schedule(static)
  for (uint32_t j = j0; j < j1; ++j) {
    for (size_t d = 0; d < D; ++d) {
      uint32_t w[4];
      float z[2];
      stream_block(cfg, (uint32_t)(d / 4), j, gen, STREAM_NOISE, w);
      uint32_t q = (uint32_t)(d % 4);
      orc_gauss_pair(w[q & 2u], w[(q & 2u) + 1], z);
      float v = z[q & 1u];
      if (cfg->noise_dtype == 1) v = orc_bf16_round(v);
      noise[(size_t)(j - j0) * D + d] = v;
    }
  }
}

/* Pre-built shared noise table (paper Sec. 5.1: the variant with a noise table built once at
 * the start of training, after Salimans et al. 2017; the RLlib baseline works this way).
 * table[t], t < len: variate (t mod 4) of the Philox block with counter (t / 4, 0, 0, STREAM_TABLE),
 * same Gaussian transform as the noise matrix; rounded to bf16 when round_bf16 is set.
 * orc_table_slice writes entries t0 <= t < t1 (output indexed from t0). */
void orc_table_slice(const orc_config *cfg, uint64_t t0, uint64_t t1, int round_bf16, float *table) {
#pragma omp parallel for schedule(static)
  for (uint64_t t = t0; t < t1; ++t) {
    uint32_t w[4];
    float z[2];
    stream_block(cfg, (uint32_t)(t / 4), 0, 0, STREAM_TABLE, w);
    uint32_t q = (uint32_t)(t % 4);
    orc_gauss_pair(w[q & 2u], w[(q & 2u) + 1], z);
    float v = z[q & 1u];
    table[t - t0] = round_bf16 ? orc_bf16_round(v) : v;
  }
}

/* Where noise row j of generation gen starts in a table of `len` entries when rows are read with
 * stride-free length `span` (the padded row length): 8 * (x mod M), M = (len - span) / 8 + 1,
 * x = word 0 of the Philox block with counter (j, gen, 0, STREAM_OFFSET).  Offsets are multiples
 * of 8 entries so that rows stay 16-byte aligned; integer work, bit-exact. */
void orc_table_offsets(const orc_config *cfg, uint64_t gen, uint64_t len, uint64_t span, uint32_t rows,
                       uint32_t *offsets) {
  uint64_t M = (len - span) / 8 + 1;
  for (uint32_t j = 0; j < rows; ++j) {
    uint32_t w[4];
    stream_block(cfg, j, (uint32_t)gen, 0, STREAM_OFFSET, w);
    offsets[j] = (uint32_t)(8u * (uint64_t)(w[0] % M));
  }
}

void orc_sample_population(const orc_config *cfg, uint64_t gen, float *noise) {
  orc_sample_rows(cfg, gen, 0, noise_rows(cfg), noise);
}

/* Parameters of individual i: theta_i[d] = fma(sign * sigma, eps_row[d], theta[d]) in
 * binary32 (one rounding), sign = +1 / -1 for even / odd i under mirrored sampling;
 * rounded to bf16 afterwards when dtype = 1.  eps_row is the noise row of this individual
 * (row i/2 when mirrored, else row i). */
void orc_perturb(const orc_config *cfg, const float *theta, const float *eps_row, uint32_t i, float *theta_i) {
  size_t D = orc_param_count(cfg);
  float scale = (cfg->antithetic && (i & 1u)) ? -cfg->sigma : cfg->sigma;
  for (size_t d = 0; d < D; ++d) {
    float v = fmaf(scale, eps_row[d], theta[d]);
    if (cfg->dtype == 1) v = orc_bf16_round(v);
    theta_i[d] = v;
  }
}

/* Initial state of environment copy e in generation gen: uniform on [-0.1, 0.1),
 * the same for every individual. */
static uint32_t episodes_per_env(const orc_config *cfg) { return cfg->episodes ? cfg->episodes : 1u; }

void orc_reset(const orc_config *cfg, uint64_t gen, uint32_t e, float *s0) {
  for (uint32_t k = 0; k < cfg->obs; ++k) {
    uint32_t w[4];
    stream_block(cfg, k / 4, e, gen, STREAM_RESET, w);
    float u = (float)(w[k % 4] >> 8) * 5.9604644775390625e-08f;   /* * 2^-24, exact */
    s0[k] = fmaf(u, 0.2f, -0.1f);
  }
}

/* ------------------------------------------------------------------ */
/* Rollout of one (individual, environment) pair.                      */
/* ------------------------------------------------------------------ */
/* bf16 mode: a contraction operand is the value rounded to binary32, then to bf16. */
static double q_operand(const orc_config *cfg, double x) {
  return cfg->dtype == 1 ? (double)orc_bf16_round((float)x) : x;
}
/* ... an operand of the ENVIRONMENT's products A s + B a: rounded like the policy's unless env_dtype keeps it binary32 */
static int env_rounds(const orc_config *cfg) { return cfg->dtype == 1 && cfg->env_dtype == 0; }
static double q_env_operand(const orc_config *cfg, double x) {
  return env_rounds(cfg) ? (double)orc_bf16_round((float)x) : x;
}

#define REAL double
#define REAL_TANH tanh
#define REAL_FABS fabs
#define ROLLOUT_FN rollout_pair_f64
#include "rollout_body.inc"
#undef REAL
#undef REAL_TANH
#undef REAL_FABS
#undef ROLLOUT_FN

/* Same loops in binary32: used only to MEASURE how far a binary32 evaluation may
 * drift from the binary64 one (tolerance derivation), never as the reference. */
#define REAL float
#define REAL_TANH tanhf
#define REAL_FABS fabsf
#define ROLLOUT_FN rollout_pair_f32
#include "rollout_body.inc"
#undef REAL
#undef REAL_TANH
#undef REAL_FABS
#undef ROLLOUT_FN

/* Evaluate individuals i0 <= i < i1 (outputs indexed from i0):
 *   returns[((i-i0)*E + e)*K + p], ep_len[same], fitness[i-i0] = mean over the E*K episodes
 *   (K = episodes per environment copy, 1 unless configured),
 *   margin[same index] = min over executed steps of | max_k|s_{t+1,k}| - done_thresh |
 *   (how close the termination test came to flipping; +inf when the rule is off).
 * noise holds the rows from noise_row0 on (dense, D per row): row r of the matrix is at
 * noise + (r - noise_row0) * D.
 * arith = 0: binary64 (the reference); 1: binary32 (sensitivity probe).
 * obs_mean, obs_inv_std [obs] (both or neither): frozen observation statistics; the policy's input is
 * (s - mean) * inv_std (paper App. B), reward, termination and environment use the raw state. */
void orc_rollout_norm(const orc_config *cfg, uint64_t gen, const float *theta, const float *noise,
                      uint32_t noise_row0, const float *A, const float *B, const float *obs_mean,
                      const float *obs_inv_std, uint32_t i0, uint32_t i1, int arith,
                      float *returns, int32_t *ep_len, float *fitness, float *margin) {
  size_t D = orc_param_count(cfg);
  uint32_t E = cfg->envs, no = cfg->obs, na = cfg->act, K = episodes_per_env(cfg);
  /* environment matrices as the rollout sees them */
  float *Ae = (float *)malloc(sizeof(float) * no * no);
  float *Be = (float *)malloc(sizeof(float) * no * na);
  for (uint32_t k = 0; k < no * no; ++k) Ae[k] = env_rounds(cfg) ? orc_bf16_round(A[k]) : A[k];
  for (uint32_t k = 0; k < no * na; ++k) Be[k] = env_rounds(cfg) ? orc_bf16_round(B[k]) : B[k];
#pragma omp parallel for schedule(dynamic, 1)
  for (uint32_t i = i0; i < i1; ++i) {
    float *theta_i = (float *)malloc(sizeof(float) * D);
    float *s0 = (float *)malloc(sizeof(float) * no);
    uint32_t row = cfg->antithetic ? i / 2 : i;
    orc_perturb(cfg, theta, noise + (size_t)(row - noise_row0) * D, i, theta_i);
    double fit = 0.0;
    for (uint32_t e = 0; e < E; ++e) {
      /* K episodes one after the other in this environment copy; episode p starts from reset number e * K + p */
      for (uint32_t p = 0; p < K; ++p) {
        double ret, mar;
        int32_t len;
        orc_reset(cfg, gen, e * K + p, s0);
        if (arith == 0) rollout_pair_f64(cfg, theta_i, Ae, Be, obs_mean, obs_inv_std, s0, &ret, &len, &mar);
        else rollout_pair_f32(cfg, theta_i, Ae, Be, obs_mean, obs_inv_std, s0, &ret, &len, &mar);
        size_t o = ((size_t)(i - i0) * E + e) * K + p;
        returns[o] = (float)ret;
        ep_len[o] = len;
        if (margin) margin[o] = (float)mar;
        fit += ret;
      }
    }
    fitness[i - i0] = (float)(fit / ((double)E * (double)K));
    free(theta_i);
    free(s0);
  }
  free(Ae);
  free(Be);
}

/* Without observation statistics (obs_mean = obs_inv_std = NULL in orc_rollout_norm: the policy sees the raw state). */
void orc_rollout(const orc_config *cfg, uint64_t gen, const float *theta, const float *noise,
                 uint32_t noise_row0, const float *A, const float *B, uint32_t i0, uint32_t i1, int arith,
                 float *returns, int32_t *ep_len, float *fitness, float *margin) {
  orc_rollout_norm(cfg, gen, theta, noise, noise_row0, A, B, NULL, NULL, i0, i1, arith, returns, ep_len, fitness, margin);
}

/* ------------------------------------------------------------------ */
/* Centred-rank fitness shaping.                                       */
/* rank_i = number of individuals strictly below i in the total order   */
/* "fitness ascending, ties by index"; shaped_i = rank_i/(N-1) - 1/2.   */
/* The order on floats is the integer order of a sign-folded bit        */
/* pattern (-0 treated as +0), so NaNs sort by bit pattern, no error.   */
/* ------------------------------------------------------------------ */
static uint32_t order_key(float f) {
  f = f + 0.0f;
  uint32_t b = bits_from_f32(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

void orc_rank(uint32_t n, const float *fitness, int32_t *rank, float *shaped) {
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t ki = order_key(fitness[i]);
    int32_t r = 0;
    for (uint32_t j = 0; j < n; ++j) {
      uint32_t kj = order_key(fitness[j]);
      if (kj < ki || (kj == ki && j < i)) ++r;
    }
    rank[i] = r;
    shaped[i] = n > 1 ? (float)r / (float)(n - 1) - 0.5f : 0.0f;
  }
}

/* ------------------------------------------------------------------ */
/* Search-gradient estimate and Adam step (binary64 arithmetic).       */
/*   g[d]   = 1/(N sigma) * sum_i shaped_i * sign_i * eps[row(i), d]     */
/*   grad   = -g + weight_decay * theta      (ascent on fitness, L2)    */
/*   m <- b1 m + (1-b1) grad ; v <- b2 v + (1-b2) grad^2                */
/*   theta <- theta - lr * (m/(1-b1^k)) / (sqrt(v/(1-b2^k)) + eps)      */
/* theta, m, v are stored in binary32 between generations.             */
/* ------------------------------------------------------------------ */
void orc_update(const orc_config *cfg, uint64_t adam_step, const float *noise, const float *shaped,
                float *theta, float *m, float *v, float *grad_out) {
  size_t D = orc_param_count(cfg);
  uint32_t N = cfg->pop;
  double b1 = (double)cfg->beta1, b2 = (double)cfg->beta2;
  double c1 = 1.0 - pow(b1, (double)adam_step);
  double c2 = 1.0 - pow(b2, (double)adam_step);
  /* g[d] accumulated individual by individual, i ascending, for every d. */
  double *g = (double *)calloc(D, sizeof(double));
  for (uint32_t i = 0; i < N; ++i) {
    uint32_t row = cfg->antithetic ? i / 2 : i;
    double sign = (cfg->antithetic && (i & 1u)) ? -1.0 : 1.0;
    const float *eps = noise + (size_t)row * D;
    for (size_t d = 0; d < D; ++d) g[d] += (double)shaped[i] * sign * (double)eps[d];
  }
  for (size_t d = 0; d < D; ++d) {
    g[d] /= (double)N * (double)cfg->sigma;
    double grad = -g[d] + (double)cfg->weight_decay * (double)theta[d];
    double mn = b1 * (double)m[d] + (1.0 - b1) * grad;
    double vn = b2 * (double)v[d] + (1.0 - b2) * grad * grad;
    double mhat = mn / c1, vhat = vn / c2;
    double th = (double)theta[d] - (double)cfg->lr * mhat / (sqrt(vhat) + (double)cfg->adam_eps);
    if (grad_out) grad_out[d] = (float)g[d];
    m[d] = (float)mn;
    v[d] = (float)vn;
    theta[d] = (float)th;
  }
  free(g);
}

/* ------------------------------------------------------------------ */
/* Sibling evolution strategies on the same sampling and evaluation     */
/* (paper Sec. 4 lists ARS and VanillaES beside OpenES; App. B        */
/* Table 5(a): ARS, 16 elites, SGD, learning rate 0.02, noise std 0.03; */
/* Table 5(c): VanillaES, 16 elites, noise std 0.02).  The paper        */
/* delegates both algorithms to their publications; what is written     */
/* here is the published update of each, on mirrored pairs for ARS and  */
/* on independent offspring for VanillaES.                              */
/* ------------------------------------------------------------------ */

/* ARS (Mania et al. 2018): direction j = the mirrored pair (2j, 2j+1).  Directions are     */
/* ordered by max(F+, F-) descending (ties: lower j first; the comparison is the integer     */
/* order of the sign-folded bit patterns, as in orc_rank) and the best b are kept.           */
/* sigma_R = population standard deviation of the 2b returns of the kept directions.         */
/* rank[2j] = rank[2j+1] = position of direction j (0 = best);                               */
/* shaped_i = F_i / sigma_R for members of kept directions, else 0 (all 0 if sigma_R = 0).   */
void orc_rank_ars(uint32_t n, uint32_t b, const float *fitness, int32_t *rank, float *shaped) {
  uint32_t R = n / 2;
  for (uint32_t j = 0; j < R; ++j) {
    uint32_t a0 = order_key(fitness[2 * j]), a1 = order_key(fitness[2 * j + 1]);
    uint32_t kj = a0 > a1 ? a0 : a1;
    int32_t pos = 0;
    for (uint32_t l = 0; l < R; ++l) {
      uint32_t b0 = order_key(fitness[2 * l]), b1 = order_key(fitness[2 * l + 1]);
      uint32_t kl = b0 > b1 ? b0 : b1;
      if (kl > kj || (kl == kj && l < j)) ++pos;
    }
    rank[2 * j] = rank[2 * j + 1] = pos;
  }
  double sum = 0.0, cnt = 0.0;
  for (uint32_t i = 0; i < 2 * R; ++i)
    if ((uint32_t)rank[i] < b) { sum += (double)fitness[i]; cnt += 1.0; }
  double mean = cnt > 0.0 ? sum / cnt : 0.0, var = 0.0;
  for (uint32_t i = 0; i < 2 * R; ++i)
    if ((uint32_t)rank[i] < b) { double dlt = (double)fitness[i] - mean; var += dlt * dlt; }
  double sigma_r = cnt > 0.0 ? sqrt(var / cnt) : 0.0;
  for (uint32_t i = 0; i < 2 * R; ++i)
    shaped[i] = ((uint32_t)rank[i] < b && sigma_r > 0.0) ? (float)((double)fitness[i] / sigma_r) : 0.0f;
}

/* theta <- theta + lr/b * sum_j (shaped_{2j} - shaped_{2j+1}) eps[j, :]   (plain SGD ascent). */
void orc_update_ars(const orc_config *cfg, uint32_t b, const float *noise, const float *shaped,
                    float *theta, float *grad_out) {
  size_t D = orc_param_count(cfg);
  uint32_t R = cfg->pop / 2;
  double *g = (double *)calloc(D, sizeof(double));
  for (uint32_t j = 0; j < R; ++j) {
    double c = (double)shaped[2 * j] - (double)shaped[2 * j + 1];
    const float *eps = noise + (size_t)j * D;
    for (size_t d = 0; d < D; ++d) g[d] += c * (double)eps[d];
  }
  for (size_t d = 0; d < D; ++d) {
    g[d] /= (double)b;
    if (grad_out) grad_out[d] = (float)g[d];
    theta[d] = (float)((double)theta[d] + (double)cfg->lr * g[d]);
  }
  free(g);
}

/* VanillaES, the canonical (mu, lambda) strategy of Chrabaszcz et al. 2018: offspring i =   */
/* theta + sigma eps[i, :] (no mirroring); ordered by fitness descending (ties: lower i      */
/* first); the best mu are recombined with weights w_k = (ln(mu + 1/2) - ln k) / sum_j (...) */
/* for k = 1..mu.  rank_i = position (0 = best); shaped_i = w_{rank_i + 1} or 0.             */
void orc_rank_vanilla(uint32_t n, uint32_t mu, const float *fitness, int32_t *rank, float *shaped) {
  double wsum = 0.0;
  for (uint32_t k = 1; k <= mu; ++k) wsum += log((double)mu + 0.5) - log((double)k);
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t ki = order_key(fitness[i]);
    int32_t pos = 0;
    for (uint32_t l = 0; l < n; ++l) {
      uint32_t kl = order_key(fitness[l]);
      if (kl > ki || (kl == ki && l < i)) ++pos;
    }
    rank[i] = pos;
    shaped[i] = (uint32_t)pos < mu ? (float)((log((double)mu + 0.5) - log((double)pos + 1.0)) / wsum) : 0.0f;
  }
}

/* theta <- sum_k w_k (theta + sigma eps_(k)) = theta + sigma * sum_i shaped_i eps[i, :]. */
void orc_update_vanilla(const orc_config *cfg, const float *noise, const float *shaped, float *theta,
                        float *grad_out) {
  size_t D = orc_param_count(cfg);
  double *g = (double *)calloc(D, sizeof(double));
  for (uint32_t i = 0; i < cfg->pop; ++i) {
    const float *eps = noise + (size_t)i * D;
    for (size_t d = 0; d < D; ++d) g[d] += (double)shaped[i] * (double)eps[d];
  }
  for (size_t d = 0; d < D; ++d) {
    g[d] *= (double)cfg->sigma;
    if (grad_out) grad_out[d] = (float)g[d];
    theta[d] = (float)((double)theta[d] + g[d]);
  }
  free(g);
}

void orc_set_threads(int n) {
#ifdef _OPENMP
  extern void omp_set_num_threads(int);
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int orc_max_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
