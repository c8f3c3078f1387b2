/*
 * es.h - C boundary of the MI355X (gfx950) OpenES hot path.
 *
 * One generation of the evolutionary policy search of arXiv 2501.15129 is four
 * enqueues on one HIP stream, with no host synchronisation in between (the paper's
 * Workflow.step() runs as one device program: Sec. 3.1, Sec. 3.2):
 *
 *     es_sample_population -> es_rollout -> es_rank -> es_update
 *
 * Conventions
 *   - Every pointer whose name ends in _d is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees or retains device memory (the one exception is the built-in
 *     scratch of es_update_static); the buffers must stay valid until the work enqueued on
 *     `stream` has completed.
 *   - Alignment: theta_d, noise_d, A_d, B_d and workspace_d must be 16-byte aligned (the kernels
 *     read them with 16-byte vector loads); every other array needs the alignment of its element
 *     type.  A misaligned pointer is ES_EINVAL.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every hot
 *     call only enqueues kernels; none of them synchronises or reads back.
 *   - Return value: ES_OK (0) or a negative es_status.  Nothing throws or aborts;
 *     es_strerror() names the code and es_last_error() gives the detail of the last
 *     failure on that context.  Arguments are validated on the host BEFORE any launch,
 *     so a failing call enqueues nothing.
 *   - Determinism: no floating-point atomics; the same inputs give bit-identical
 *     outputs on every run.
 *   - N = pop, E = envs_per_ind * episodes_per_env (episodes per fitness evaluation), T = horizon,
 *     D = es_param_count().
 *
 * Flat parameter vector theta[D] (binary32): W1[hid,obs], b1[hid], W2[hid,hid], b2[hid],
 * W3[act,hid], b3[act], in this order, each matrix row-major [out,in].
 *
 * Noise matrix: es_noise_rows() rows (N/2 with mirrored sampling, else N), row stride
 * es_noise_ld() ELEMENTS (D rounded up so that every row starts 1 KiB-aligned), element
 * type binary32 (noise_dtype 0) or bf16 bit patterns (noise_dtype 1).  Columns
 * D <= d < ld are written as zero by es_sample_population and must be zero if the caller
 * fills the matrix itself.
 *
 * Regenerated noise (noise_dtype 2 and 3; paper Sec. 5.1, generation on the fly taken to its
 * end): no matrix exists.  es_noise_bytes() is 0, every noise_d argument is ignored and may
 * be NULL, es_sample_population only records the generation (host side, no device work), and
 * es_rollout / es_update recompute each value from the counter stream where they need it.
 * Mode 2 uses the binary32 values (the results of noise_dtype 0), mode 3 rounds them to bf16
 * (the results of noise_dtype 1), bit for bit.
 *
 * Shared noise table (noise_dtype 4: binary32 entries, 5: bf16 entries; the paper's Sec. 5.1
 * variant with a table built once at the start of training, after Salimans et al. 2017): the
 * noise buffer is [table: noise_table_len entries | row offsets: es_noise_rows() uint32].
 * es_build_noise_table fills the table once; es_sample_population only draws, for every noise
 * row of the generation, where in the table the row starts (a multiple of 8 entries, so rows
 * stay 16-byte aligned), and es_rollout / es_update read row j at table + offset[j].
 */
#ifndef ES_H_
#define ES_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum es_status {
  ES_OK = 0,
  ES_EINVAL = -1,       /* null pointer, zero dimension, odd pop with mirrored sampling, ... */
  ES_EUNSUPPORTED = -2, /* a shape or mode no kernel of this build can place on chip        */
  ES_EHIP = -3          /* the HIP runtime reported an error (text in es_last_error)        */
} es_status;

typedef struct es_config {
  uint32_t pop;          /* N; must be even when antithetic = 1                              */
  uint32_t envs_per_ind; /* environment copies per individual (see episodes_per_env)          */
  uint32_t horizon;      /* T: maximum episode length                                        */
  uint32_t obs_dim, hid_dim, act_dim; /* policy MLP obs -> hid -> hid -> act                 */
  uint32_t dtype;        /* 0: binary32 everywhere.  1: every operand of a matrix product
                            (perturbed weights and biases, env matrices A and B, the state,
                            hidden activations and action as inputs of the next product) is
                            rounded to bf16; accumulation, tanh, reward, return are binary32 */
  uint32_t noise_dtype;  /* 0: binary32 noise matrix ; 1: bf16 noise matrix ;
                            2 / 3: no matrix, values regenerated (binary32 / bf16-rounded) ;
                            4 / 5: rows read from a shared table (binary32 / bf16 entries)   */
  uint32_t antithetic;   /* 1: individuals 2j and 2j+1 use +eps_j and -eps_j                 */
  uint32_t out_tanh;     /* 1: tanh on the action layer as well                              */
  float sigma;           /* noise std (paper App. B Table 5b: 0.02)                          */
  float lr, beta1, beta2, adam_eps; /* Adam (Table 5b: lr 0.01)                              */
  float weight_decay;    /* L2 coefficient added to the gradient (Table 5b: 0.005)           */
  float done_thresh;     /* episode ends after the step whose new state has max|s| > this;
                            +inf = fixed-length episodes (the paper's timing protocol, Sec. 5.1) */
  float act_cost;        /* reward = 1 - |s|^2/obs_dim - act_cost |a|^2                      */
  uint64_t seed;         /* key of the counter-based noise / reset streams                   */
  uint32_t algorithm;    /* which strategy es_rank / es_update implement (es_algorithm)      */
  uint32_t num_elites;   /* ARS: directions kept (b); VanillaES: parents (mu); else ignored  */
  uint32_t hidden_act;   /* activation of the two hidden layers: 0 tanh ; 1 ReLU (the paper's
                            EA experiments use ReLU MLPs, App. B); the action layer follows out_tanh */
  uint32_t num_hidden;   /* m hidden layers of width hid_dim (the paper's Sec. 5.1 varies m; its base
                            case and the default are 2; 0 means 2).  Flat parameters: W1[hid,obs], b1,
                            then (m - 1) x (W[hid,hid], b[hid]), then W3[act,hid], b3.  The one-
                            wavefront register kernel serves m = 2 with obs, hid <= 64, act <= 16; the
                            bf16 matrix-core kernel m = 2 for hid <= 256, obs <= 256, act <= 32 and
                            m = 1, 3, 4 for obs_dim <= 64, act_dim <= 16; everything else runs on the LDS
                            kernel if the individual fits the LDS (else ES_EUNSUPPORTED from es_rollout) */
  uint64_t noise_table_len; /* entries of the shared noise table (noise_dtype 4, 5 only): a multiple
                            of 8, at least es_noise_ld(), below 2^32                                    */
  uint32_t episodes_per_env; /* k episodes run back to back in every environment copy, the copy resetting
                            itself in between (the auto-reset environment wrapper of the paper's Sec. 3.1);
                            0 means 1.  Episode p of copy e starts from reset number e * k + p and its return
                            sits at column e * k + p, so E = envs_per_ind * k episodes make up the fitness.
                            The episodes of one copy do not depend on each other, so the kernels run all E
                            side by side (with few copies this also fills matrix-core columns that would
                            otherwise idle) and the results equal the sequential schedule's exactly         */
  uint32_t env_dtype;    /* only with dtype = 1.  0: the environment's products A s + B a use bf16 operands too
                            (A, B, the state and the action rounded; configs[4] needs that to hold A on chip).
                            1: the environment stays binary32 - "bf16 weights and activations" is a property of the
                            policy, not of the simulator it acts on; built for two hidden layers with obs_dim <= 64
                            (any width on the LDS kernel if the individual fits), else ES_EUNSUPPORTED from es_rollout */
} es_config;

/*
 * The strategies of the paper's Sec. 4 that share this sampling and evaluation.
 * Sampling and es_rollout are the same for all; es_rank and es_update differ:
 *   ES_OPENES   centred ranks, Adam                                  (App. B Table 5b)
 *   ES_ARS      the best b mirrored directions by max(F+, F-), returns divided by the standard
 *               deviation of the 2b kept returns, plain SGD ascent   (Table 5a; Mania et al. 2018)
 *               requires antithetic = 1, 1 <= num_elites <= pop / 2
 *   ES_VANILLA  (mu, lambda) truncation selection with log-rank weights, recombination
 *               theta <- sum_k w_k (theta + sigma eps_(k))           (Table 5c; Chrabaszcz et al. 2018)
 *               requires antithetic = 0, 1 <= num_elites <= pop
 * ES_ARS and ES_VANILLA support pop <= 8192.
 */
typedef enum es_algorithm { ES_OPENES = 0, ES_ARS = 1, ES_VANILLA = 2 } es_algorithm;

typedef struct es_ctx es_ctx; /* opaque, host-side: validated config + kernel choice */

/* Validate `cfg` and build a context.  Allocates host memory only.  Must be called with the
 * target GPU current; the kernel choice depends on that device's LDS size. */
int es_create(const es_config* cfg, es_ctx** out);
int es_destroy(es_ctx* ctx);

size_t es_param_count(const es_ctx* ctx);      /* D                                           */
size_t es_noise_rows(const es_ctx* ctx);       /* N/2 (mirrored) or N                         */
size_t es_noise_ld(const es_ctx* ctx);         /* row stride of the noise matrix, in elements */
size_t es_noise_bytes(const es_ctx* ctx);      /* rows * ld * sizeof(element)                 */
size_t es_workspace_bytes(const es_ctx* ctx);  /* scratch for es_rollout / es_update (>= 256) */
const char* es_rollout_kernel(const es_ctx* ctx); /* name of the rollout variant chosen       */
const char* es_update_kernel(const es_ctx* ctx);  /* name of the es_update kernel(s) chosen        */
const char* es_strerror(int status);
const char* es_last_error(const es_ctx* ctx);

/*
 * Frozen observation normalisation (paper App. B: virtual batch normalisation - mean and
 * standard deviation of the observations computed once from random timesteps and kept fixed
 * for the whole run).  With statistics set, the policy of every later es_rollout sees
 * (s - mean) * inv_std, computed in binary32 (and rounded to bf16 as a matrix operand when
 * dtype = 1); reward, termination test and the environment keep the raw state.
 * mean_d, inv_std_d: [obs_dim] f32 device arrays owned by the caller; they are read by
 * es_rollout, not copied, and must stay valid until replaced.  Both NULL (the default)
 * switches normalisation off; exactly one NULL is ES_EINVAL.  Host-side only: no device work.
 */
int es_set_obs_norm(es_ctx* ctx, const float* mean_d, const float* inv_std_d);

/*
 * Fills the shared noise table (noise_dtype 4, 5; ES_EINVAL otherwise): entry t < noise_table_len is
 * variate (t mod 4) of the Philox4x32-10 block with counter (t / 4, 0, 0, 3) and key (seed low,
 * seed high), through the same binary32 Box-Muller sequence as the noise matrix, rounded to bf16
 * in mode 5.  Called once; the table does not depend on the generation.
 */
int es_build_noise_table(es_ctx* ctx, void* noise_d, void* stream);

/*
 * Noise of generation `generation` (paper Sec. 5.1: perturbations are generated on the fly
 * each generation, not read from a pre-built table).  noise[j, d] for j < rows, d < D is
 * variate (d mod 4) of the Philox4x32-10 block with counter (d / 4, j, generation, 1) and
 * key (seed low, seed high), mapped to N(0,1) by a fixed binary32 Box-Muller sequence, then
 * rounded to bf16 (nearest-even) when noise_dtype = 1.  generation < 2^32.
 * Writes rows * ld elements to noise_d.  With regenerated noise (noise_dtype 2, 3) nothing is
 * written: the call records `generation` in the context for the next es_update.
 * With a shared table (noise_dtype 4, 5) it writes the row offsets of this generation behind the
 * table: offset[j] = 8 * (x mod M), M = (noise_table_len - ld) / 8 + 1, x = word 0 of the Philox
 * block with counter (j, generation, 0, 4).
 */
int es_sample_population(es_ctx* ctx, uint64_t generation, void* noise_d, void* stream);

/*
 * Population x environment evaluation (paper Sec. 3.2: all individuals at once, each on E
 * parallel environment copies; Sec. 5.2: deterministic MLP policy, fitness = mean
 * undiscounted episodic return).  For individual i (noise row j = i/2, sign +/- when
 * mirrored, else j = i, +):
 *     theta_i = fma(sign * sigma, noise[j, :], theta)        (binary32; bf16-rounded if dtype 1)
 *     s_0[e]  = uniform[-0.1, 0.1) from Philox counter (k / 4, e, generation, 2), the same for all i
 *     per step: h1 = act(W1 s + b1), h2 = act(W2 h1 + b2), a = tanh(W3 h2 + b3),   (act = tanh or ReLU)
 *               r = 1 - |s|^2/obs_dim - act_cost |a|^2,  R += r,  L += 1,
 *               s <- tanh(A s + B a),  stop after this step if max|s| > done_thresh.
 * In:  theta_d [D] f32, noise_d (layout above), A_d [obs,obs] f32, B_d [obs,act] f32 (row-major).
 * Out: returns_d [N,E] f32, ep_len_d [N,E] i32, fitness_d [N] f32 (mean over E).
 * workspace_d: es_workspace_bytes() bytes, contents irrelevant on entry.
 */
int es_rollout(es_ctx* ctx, uint64_t generation, const float* theta_d, const void* noise_d,
               const float* A_d, const float* B_d, float* returns_d, int32_t* ep_len_d,
               float* fitness_d, void* workspace_d, void* stream);

/*
 * Centred-rank fitness shaping (the OpenES of the paper's Sec. 4, after Salimans et al.):
 * rank_i = position of individual i in ascending fitness order, ties broken by index
 * (-0 equals +0; NaNs sort by bit pattern, no error); shaped_i = rank_i / (N-1) - 1/2.
 * In: fitness_d [N] f32.  Out: rank_d [N] i32, shaped_d [N] f32.
 * ES_ARS: rank_d[2j] = rank_d[2j+1] = position of direction j when directions are ordered by
 *   max(F_2j, F_2j+1) descending (ties: lower j first); shaped_i = F_i / sigma_R for the members
 *   of the best num_elites directions, 0 elsewhere (all 0 when sigma_R = 0).
 * ES_VANILLA: rank_d[i] = position of individual i in descending fitness order (ties: lower i
 *   first); shaped_i = (ln(mu + 1/2) - ln(rank_i + 1)) / sum_{k<=mu} (ln(mu + 1/2) - ln k) for
 *   rank_i < mu = num_elites, 0 elsewhere.
 */
int es_rank(es_ctx* ctx, const float* fitness_d, int32_t* rank_d, float* shaped_d, void* stream);

/*
 * Search-gradient estimate and Adam step (paper App. B Table 5b: Adam, lr 0.01, weight decay 0.005):
 *     g[d]  = 1/(N sigma) * sum_i shaped_i * sign_i * noise[row(i), d]
 *     grad  = -g + weight_decay * theta ;  m, v = Adam moments ;  k = adam_step >= 1
 *     theta <- theta - lr * (m / (1 - beta1^k)) / (sqrt(v / (1 - beta2^k)) + adam_eps)
 * The noise matrix is streamed exactly once; sums are taken in binary64 in a fixed order.
 * In: noise_d, shaped_d [N] f32.  In/out: theta_d, m_d, v_d [D] f32.
 * Out (optional, may be NULL): grad_d [D] f32 receives g.
 * workspace_d: es_workspace_bytes() bytes.  sigma must be > 0.
 * With regenerated noise the values are those of the generation passed to the most recent
 * es_sample_population call on this context (ES_EINVAL if there was none).
 * ES_ARS:     g = 1/b * sum_j (shaped_2j - shaped_2j+1) noise[j, :] ;  theta <- theta + lr g.
 * ES_VANILLA: g = sigma * sum_i shaped_i noise[i, :] ;                 theta <- theta + g.
 * For both, adam_step is ignored and m_d, v_d are neither read nor written (may be NULL).
 */
int es_update(es_ctx* ctx, uint64_t adam_step, const void* noise_d, const float* shaped_d,
              float* theta_d, float* m_d, float* v_d, float* grad_d, void* workspace_d,
              void* stream);

/*
 * es_update for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as es_update, bit for bit, minus workspace_d: the binary64 partial sums live
 * in a built-in device array of es_static_scratch_bytes() = 32 MiB that every GPU the library runs
 * on holds until the process ends (all five benchmark shapes fit, stored or regenerated noise).
 * The call allocates and frees nothing and clears nothing (the reduction writes every partial it
 * later reads).  A context whose es_workspace_bytes() exceeds the array is refused with
 * ES_EUNSUPPORTED before any launch.  All calls on one GPU share that GPU's array, whatever their
 * context: calls that may overlap in time on one GPU (different streams or threads) race and must
 * be serialised by the caller; calls on one stream are safe.  The array's address is looked up
 * once per device (in es_create when a GPU is current, else on the first call).
 */
size_t es_static_scratch_bytes(void);
int es_update_static(es_ctx* ctx, uint64_t adam_step, const void* noise_d, const float* shaped_d,
                     float* theta_d, float* m_d, float* v_d, float* grad_d, void* stream);

/*
 * One whole generation - the four calls above in their order, es_sample_population(generation),
 * es_rollout(generation), es_rank, es_update(adam_step), enqueued on `stream` by one call: the
 * counterpart of the paper's Workflow.step() running as one device program (Sec. 3.1, 3.2).
 * Arguments mean what they mean in the stage calls (noise_d NULL with regenerated noise; m_d, v_d
 * NULL allowed for ES_ARS / ES_VANILLA; grad_d optional); results are bit-identical to the four
 * separate calls.  All arguments of all stages are checked before the first launch, so a failing
 * call enqueues nothing.  The call neither allocates nor synchronises nor clears memory with
 * memset nodes, so a caller may record it into a HIP graph (stream capture) and replay it; a
 * replay repeats the recorded generation and adam_step numbers.
 */
int es_generation(es_ctx* ctx, uint64_t generation, uint64_t adam_step, void* noise_d,
                  const float* A_d, const float* B_d, float* theta_d, float* m_d, float* v_d,
                  float* returns_d, int32_t* ep_len_d, float* fitness_d, int32_t* rank_d,
                  float* shaped_d, float* grad_d, void* workspace_d, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ES_H_ */
