/*
 * pop.h -- C boundary of the population update engine (gfx950 / MI355X).
 *
 * The library carries out what Sec. 4.1 of "Fast Population-Based Reinforcement
 * Learning on a Single Machine" speeds up: ONE gradient-update step applied at
 * once to a population of P independent off-policy agents (TD3).  Every agent
 * owns its MLP actor, twin critics, the three target copies, Adam moments,
 * hyperparameters, seed and replay buffer; agents never exchange anything.
 *
 * Conventions for every call
 *   - Return value: POP_OK (0) or a negative POP_E* code.  Nothing throws or
 *     aborts across this boundary.  pop_last_error() gives a readable message
 *     for the last failing call on that context (or for a failing pop_create
 *     when passed NULL).
 *   - Argument checks run on the host before anything is launched; a failing
 *     call launches nothing and writes nothing.
 *   - "device pointer" = HIP device memory of the GPU that was current at
 *     pop_create; "host pointer" = ordinary host memory.  The caller owns every
 *     pointer it passes, including the workspace and the stream; the library
 *     allocates no device memory (a context holds 8 bytes of pinned host memory)
 *     and frees nothing of the caller's.
 *   - All work is enqueued on the stream given to pop_create.  pop_update and
 *     calls with device pointers are asynchronous; calls that take or fill host
 *     pointers synchronise that stream before returning.
 *   - Shapes are row-major, the population index first (App. A of the paper:
 *     the agents' batches are stacked on a new leading axis; App. C: weights
 *     are [P, in, out], biases [P, 1, out]).
 */
#ifndef POP_H
#define POP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pop_ctx pop_ctx; /* opaque; host memory owned by the library */

enum {
  POP_OK = 0,
  POP_EINVAL = -1,       /* bad argument (NULL, out of range, wrong length) */
  POP_ENOMEM = -2,       /* workspace smaller than pop_workspace_bytes() */
  POP_EEMPTY = -3,       /* pop_update while some agent's buffer is empty */
  POP_EHIP = -4,         /* a HIP runtime call failed; see pop_last_error() */
  POP_EUNSUPPORTED = -5  /* shape or algorithm the kernels do not cover */
};

enum { POP_ALGO_TD3 = 0, POP_ALGO_SAC = 1, POP_ALGO_TD3_SHARED = 2 };

/* Per-agent hyperparameters (Sec. 4.1: replicas differ in initial weights and
 * hyperparameters; App. B.1 lists the ones a population tunes).  Read at
 * pop_create and copied. */
typedef struct {
  uint64_t seed;        /* key of every random draw of this agent (initial
                           weights, replay sampling, smoothing noise).  0 means
                           "derive from the population seed and the index". */
  float lr_actor, lr_critic;
  float gamma;          /* discount */
  float tau;            /* Polyak rate of the target networks */
  float policy_noise;   /* std of the target-policy smoothing noise */
  float noise_clip;     /* clip of that noise */
  int32_t policy_delay; /* actor and targets are updated when step % delay == 0 */
  float adam_b1, adam_b2, adam_eps;
  float lr_alpha, target_entropy, init_log_alpha; /* SAC only (learning rate of log alpha, the entropy the
                           temperature steers to, log alpha at step 0); ignored for TD3.  SAC in turn ignores
                           policy_noise, noise_clip and policy_delay: it updates everything every step */
  int32_t reserved_;    /* keeps sizeof == 64 */
} pop_hparams;

/* POP_ALGO_TD3_SHARED (Sec. 4.2 of the paper, "Training Agents Sharing Parameters"): TD3 with ONE pair of critics
 * (and target critics) for the whole population; every agent keeps its own policy, target policy, buffer, seed,
 * discount and smoothing noise.  A step runs every agent's batch through that agent's policy networks, takes one
 * Adam step on the critics for the critic loss averaged over the population, then (on delayed steps) the ordinary
 * TD3 policy step of every agent through the updated critic.  The critics take their initial weights (seed),
 * learning rate, Adam constants and tau from agent 0's hyperparameters; policy_delay must be the same for all
 * agents (POP_EINVAL otherwise).  The tensor codes of the critics name the shared tensors whatever `agent` is;
 * pop_copy_agent copies the policy side only.  Shapes as for TD3.
 *
 * Population-wide shapes.  Supported now: algo TD3, TD3_SHARED or SAC, n_hidden == 2 with
 * hidden = {256, 256}, batch == 256 (the batch of every workload of Sec. 4.1),
 * 1 <= capacity < 2^32; obs_dim + act_dim <= 448, act_dim <= 24 (HalfCheetah-v2 of Sec. 4.1 is 17 / 6,
 * Humanoid-v2 376 / 17).  Anything else gives POP_EUNSUPPORTED. */

/* How the kernels of an update step are launched and tiled.  All zeros (the default of a cleared pop_config) lets
 * the library choose by population size; the fields exist for measurements and for tests that compare the choices
 * with one another.  They change no result beyond the order of fp32 sums: with the same rows and tile widths, and actor_ahead
 * off, every launch structure gives bit-identical results.  Nothing is read from the process environment. */
enum {
  POP_LAUNCH_AUTO = 0,
  POP_LAUNCH_PER_PART = 1,       /* one launch per part of the step: POP_K_TARGET .. POP_K_WGRAD_ACTOR */
  POP_LAUNCH_TARGET_CRITIC = 2,  /* target and critic chains in one launch (POP_K_TARGET_CRITIC), the rest per part */
  POP_LAUNCH_SINGLE = 3,         /* the whole step in one launch (POP_K_STEP) */
  POP_LAUNCH_TAIL = 4            /* as TARGET_CRITIC, and on steps with an actor update the rest in one launch
                                    (POP_K_STEP_TAIL) */
};
typedef struct {
  int32_t launch;        /* POP_LAUNCH_*.  SINGLE and TAIL exist for TD3 whose chains all take 32 or 64 batch rows per
                            workgroup, or (16, 64, 16); pop_create refuses them with POP_EINVAL otherwise.  SAC and
                            shared critics take PER_PART or TARGET_CRITIC. */
  int32_t rows_target, rows_critic, rows_actor;   /* batch rows per workgroup of the three layer chains: 0 = choose;
                            32 or 64, and 16 for the target and actor chains.  A launch structure that has no kernel
                            for the rows asked for fails at pop_update with POP_EHIP and runs nothing. */
  int32_t rows_critic1;  /* 0 = choose; 16: the 16-row target workgroups go on into critic 1 for their own rows and only
                            critic 2 has workgroups of its own (TD3 with TARGET_CRITIC and rows_target == 16 only);
                            otherwise equal to rows_critic */
  int32_t half_tiles;    /* weight-gradient tiles of half the width in the stand-alone tile launches: 0 = choose (on
                            while all of them are resident at once, up to 10 agents), 1 = off, 2 = on.  The sums over
                            the batch then come in two halves: compare launch structures with this set to 1. */
  int32_t actor_ahead;   /* the actor's own forward pass of a step with a policy update runs inside the target / critic
                            launch, in the 32-row workgroups of critic 2 while they wait for their Bellman targets, and
                            the actor launch starts at the critic: 0 = choose (on with rows_critic1 == 16 while every
                            workgroup of the launch has a CU of its own), 1 = off, 2 = on.  Exists for TD3 and shared critics with TARGET_CRITIC and
                            rows (16, 32, 16); POP_EINVAL for 2 elsewhere.  That pass then runs on 32-row instead of
                            16-row tiles, another order of the fp32 sums: compare launch structures with this set to 1. */
} pop_tuning;

typedef struct {
  int32_t algo;
  int32_t P;
  int32_t obs_dim, act_dim;
  int32_t n_hidden;
  int32_t hidden[4];
  int32_t batch;
  int64_t capacity;     /* replay rows per agent */
  pop_tuning tuning;    /* all zeros: the library chooses */
} pop_config;

/* Which tensor pop_get_params returns.  Networks come in the canonical flat
 * order: layer by layer, W[in, out] row-major then b[out] (App. C layout of
 * one population member).  Critic input is concat(obs, act). */
enum {
  POP_ACTOR = 0, POP_CRITIC1 = 1, POP_CRITIC2 = 2,
  POP_T_ACTOR = 3, POP_T_CRITIC1 = 4, POP_T_CRITIC2 = 5,
  POP_ADAM_M_ACTOR = 6, POP_ADAM_M_CRITIC1 = 7, POP_ADAM_M_CRITIC2 = 8,
  POP_ADAM_V_ACTOR = 9, POP_ADAM_V_CRITIC1 = 10, POP_ADAM_V_CRITIC2 = 11,
  /* gradients of the last step that updated that network; only recorded
   * while pop_set_debug(ctx, 1) is on */
  POP_GRAD_ACTOR = 12, POP_GRAD_CRITIC1 = 13, POP_GRAD_CRITIC2 = 14,
  /* SAC only, one float each: the log of the temperature alpha and its Adam
   * moments.  (For SAC the POP_T_ACTOR slot exists but is unused: there is no
   * target actor; the actor network has 2 * act_dim outputs, the means of the
   * actions followed by their log standard deviations.) */
  POP_LOG_ALPHA = 15, POP_ADAM_M_LOG_ALPHA = 16, POP_ADAM_V_LOG_ALPHA = 17
};

/* What pop_debug_get returns (state of the most recent update step). */
enum {
  POP_DBG_INDICES = 0,       /* uint32 [P, batch]: replay rows sampled */
  POP_DBG_BATCH = 1,         /* float  [P, batch, 2*obs+act+2]: rows as stored:
                                obs, act, reward, done, next_obs */
  POP_DBG_TARGET_ACTION = 2, /* float  [P, batch, act]: smoothed target action */
  POP_DBG_TARGET_Y = 3,      /* float  [P, batch]: Bellman target */
  POP_DBG_LOSSES = 4         /* float  [P, 2]: critic loss, actor loss (the
                                actor loss of the last step that had one) */
};

/* Bytes of device workspace a population of this shape needs, or a negative POP_E* code.  Everything the
 * population owns lives in that one allocation -- the stacked parameter tensors of all agents (App. C: one [P, in,
 * out] array per layer instead of P small ones; Sec. 4.1 names the single allocation as what keeps memory from
 * fragmenting), targets, Adam moments, the per-agent replay buffers (App. A) and the step's scratch. */
int64_t pop_workspace_bytes(const pop_config* cfg);

/* Number of floats of one network of one agent in canonical order (App. C: per layer W[in, out] then b[out]):
 * which = POP_ACTOR or any critic code.  Negative POP_E* code on bad arguments. */
int64_t pop_net_size(const pop_config* cfg, int32_t which);

/* Create a population (Sec. 4.1: N replicas with different initial weights
 * and hyperparameters).  Weights are Glorot-uniform from each agent's seed,
 * biases 0, targets exact copies, Adam moments 0, step counter 0, buffers
 * empty.  `hp` is a host array of P entries.  `workspace` is a device
 * pointer, 256-byte aligned, of at least pop_workspace_bytes(cfg) bytes that
 * must stay valid until pop_destroy.  `hip_stream` is a hipStream_t (NULL =
 * the default stream).  Initialisation is enqueued on that stream. */
int pop_create(pop_ctx** out, const pop_config* cfg, const pop_hparams* hp,
               uint64_t seed, void* workspace, int64_t workspace_bytes,
               void* hip_stream);

/* Append n transitions to the replay buffer(s) in arrival order; once a
 * buffer is full the oldest rows are overwritten (Sec. 1 / App. A: bounded
 * first-in-first-out buffer, one per agent).  agent >= 0: arrays are
 * obs[n, obs_dim], act[n, act_dim], rew[n], done[n] (0 or 1), next_obs[n,
 * obs_dim] for that agent.  agent == -1: every array has a leading P axis
 * ([P, n, ...]) and agent i receives slice i.  ptrs_on_device tells whether
 * the five arrays are device or host pointers (all the same kind). */
int pop_insert(pop_ctx* ctx, int32_t agent, int64_t n, const float* obs,
               const float* act, const float* rew, const float* done,
               const float* next_obs, int32_t ptrs_on_device);

/* Run n_steps update steps for every agent, back to back on the device with
 * no host synchronisation in between (Sec. 4.1: many update steps chained
 * without returning parameters to the host).  A step also draws and gathers the
 * replay rows of the step after it, so that a later call starts at once; rows
 * gathered ahead are dropped when an insert, a buffer copy or new hyperparameters
 * come in between.  One step of one agent: sample a
 * batch from its own buffer, TD3 critic update, and -- when step %
 * policy_delay == 0 -- actor update and Polyak update of all three targets.
 * POP_EEMPTY if some agent has no transitions. */
int pop_update(pop_ctx* ctx, int32_t n_steps);

/* Kernels of an update step (indices into the arrays of pop_update_timed).  The parts of a step -- target chains,
 * critic chains, critic weight-gradient tiles, actor chains, actor weight-gradient tiles, the gather of the next
 * step's rows -- run as one launch each, or several of them as parts of one grid that hand their results on per
 * agent / per network inside the launch (Sec. 4.1: the cost of a small population's step is dispatch, not
 * arithmetic); pop_tuning.launch says which. */
enum {
  POP_K_GATHER = 0,        /* replay index draw + row gather (first step of a call only) */
  POP_K_TARGET = 1,        /* target actor, smoothing, twin target critics, y */
  POP_K_CRITIC = 2,        /* twin critics forward + backward to pre-activations */
  POP_K_WGRAD_CRITIC = 3,  /* critic weight gradients + Adam (+ Polyak) */
  POP_K_ACTOR = 4,         /* actor forward, critic-1 forward/input-gradient, actor backward */
  POP_K_WGRAD_ACTOR = 5,   /* actor weight gradients + Adam + Polyak */
  POP_K_TARGET_CRITIC = 6, /* POP_K_TARGET and POP_K_CRITIC in one launch */
  POP_K_STEP = 7,          /* the whole step in one launch */
  POP_K_STEP_TAIL = 8,     /* critic weight gradients, actor chain, actor weight gradients in one launch */
  POP_K_COUNT = 9
};

/* Measurement variant of pop_update (same work, same results): every kernel
 * launch is bracketed by HIP events on the context's stream; ms[k] receives
 * the summed elapsed milliseconds of kernel k and launches[k] its number of
 * launches (host arrays of POP_K_COUNT entries, overwritten).  Synchronises
 * the stream before returning. */
int pop_update_timed(pop_ctx* ctx, int32_t n_steps, double* ms, int64_t* launches);

/* Deterministic actions of every agent's current actor (for SAC: the tanh of
 * the mean): obs[P, n, obs_dim] -> act_out[P, n, act_dim] (agent i acts on
 * slice i).  This is the inference the paper's actor processes run on their copy of the parameters (App. A), here
 * for the whole population at once on the device that holds them. */
int pop_act(pop_ctx* ctx, const float* obs, int32_t n, float* act_out,
            int32_t ptrs_on_device);

/* The same with Gaussian exploration noise, as the data-collecting actors of
 * a TD3 agent use it: a = clip(pi(obs) + sigma[i] * eps, -1, 1) for agent i,
 * sigma = host array of P non-negative values (0: no noise for that agent).
 * eps is unit normal number r * act_dim + j (r = row of the agent's slice, j =
 * action component) of the agent's exploration stream at counter `step`, so a
 * call is reproducible and independent of how it is split into pieces; callers
 * pass a fresh `step` per call (e.g. their environment-step counter).
 * For SAC the policy itself is sampled instead: a = tanh(mu + sigma[i] *
 * std * eps) with the policy's own std (sigma[i] = 1 is the policy).
 * Synchronises the stream (sigma is staged on the device). */
int pop_act_explore(pop_ctx* ctx, const float* obs, int32_t n, float* act_out,
                    int32_t ptrs_on_device, const float* sigma, uint32_t step);

/* pop_act_explore for callers that cannot allocate device memory or wait for the device: code under HIP graph
 * capture, tight acting loops, harnesses that forbid hipMalloc.  Same result as pop_act_explore with device
 * pointers (obs and act_out are device pointers, sigma a host array of P values read before the call returns).
 * It allocates nothing, copies nothing and synchronises nothing: the noise scales reach the device as a kernel
 * argument and are staged in a static device array of 256 floats (1 KiB per GPU, held until the process ends), so
 * populations of more than 256 agents are refused with POP_EUNSUPPORTED.  Every call on a GPU shares that GPU's
 * array, whatever the context: calls that can overlap on one GPU (different streams, different threads) race on
 * it; calls on one stream are ordered.  Nothing in the array has to be cleared between calls: a call writes the P
 * entries it reads. */
int pop_act_explore_noalloc(pop_ctx* ctx, const float* obs, int32_t n, float* act_out,
                            const float* sigma, uint32_t step);

/* Copy one tensor of one agent (see the POP_* codes) into out[out_len];
 * out_len must be at least the tensor's length, else POP_EINVAL and nothing
 * is written.  Returns the number of floats written (>= 0) or an error. */
int64_t pop_get_params(pop_ctx* ctx, int32_t agent, int32_t which, float* out,
                       int64_t out_len, int32_t on_device);

/* Overwrite one tensor of one agent (POP_ACTOR .. POP_ADAM_V_CRITIC2; the
 * gradient codes are read-only) with in[in_len] floats in canonical order;
 * in_len must equal the tensor's length.  This is the primitive a population
 * method needs to copy a good agent over a bad one (App. B.1 of the paper:
 * the worst agents are replaced by copies of the best) and what tests use to
 * start a step from a prescribed state.  Enqueued on the context's stream;
 * synchronises when `in` is a host pointer. */
int pop_set_params(pop_ctx* ctx, int32_t agent, int32_t which, const float* in,
                   int64_t in_len, int32_t on_device);

/* Agent dst becomes a copy of agent src: online and target networks, Adam
 * moments and the actor's Adam step count (device-to-device copies on the
 * context's stream); with_buffer != 0: also the replay buffer with its fill
 * level and write position.  dst keeps its own seed and hyperparameters.
 * This is the "exploit" half of the population step of App. B.1 of the paper
 * (the worst agents are replaced by copies of randomly chosen good ones);
 * which agents are good is the caller's business.  Synchronises the stream.
 * POP_EINVAL for an agent index out of range; dst == src is a no-op. */
int pop_copy_agent(pop_ctx* ctx, int32_t dst, int32_t src, int32_t with_buffer);

/* New hyperparameters (and seed) for one agent, in force from its next update
 * step on: the "explore" half of the same population step (App. B.1: the
 * copies have their hyperparameters re-sampled -- learning rates, update
 * frequency of the policy, noise parameters, discount).  Checked like the
 * hyperparameters given to pop_create; seed 0 is rejected here.  Adam's step
 * counts stay continuous: the critics count every step, the actor the actor
 * updates actually taken, whatever policy_delay was at the time.
 * Synchronises the stream. */
int pop_set_hparams(pop_ctx* ctx, int32_t agent, const pop_hparams* hp);

/* Record per-parameter gradients for POP_GRAD_* (costs one extra store per
 * parameter per step).  Off by default. */
int pop_set_debug(pop_ctx* ctx, int32_t on);

/* Copy a diagnostic array of the last step (POP_DBG_*) into out; out_bytes
 * must be at least its size.  Returns bytes written or an error. */
int64_t pop_debug_get(pop_ctx* ctx, int32_t what, void* out, int64_t out_bytes,
                      int32_t on_device);

/* Replay indices of the last step widened to int64 [P, batch] (host pointer). */
int pop_debug_indices(pop_ctx* ctx, int64_t* out);

/* Number of update steps taken so far, and rows held by one agent's buffer. */
int64_t pop_step_count(const pop_ctx* ctx);
int64_t pop_buffer_count(const pop_ctx* ctx, int32_t agent);

/* The launch structure and tiling in force for this context, with every "choose" of pop_config.tuning resolved
 * (Sec. 4.1 leaves the mapping of the population onto the device to the implementation; this is the mapping taken):
 * launch = POP_LAUNCH_*, rows_* = batch rows per workgroup, half_tiles and actor_ahead = 1 (off) or 2 (on).  For
 * reports and measurements; host only, no device work. */
int pop_get_tuning(const pop_ctx* ctx, pop_tuning* out);

/* Runtime options of a context. */
enum {
  POP_OPT_WAIT_LIMIT_TICKS = 0   /* longest wait of one workgroup for another of the same launch, in 10 ns ticks
                                    (1 .. 10^9; default 5,000,000 = 50 ms).  In force from the next launch on. */
};
int pop_set_option(pop_ctx* ctx, int32_t key, int64_t value);

/* Block until everything enqueued by this context has finished (Sec. 4.1: the host takes part only between
 * device calls of many update steps each); reports asynchronous kernel errors as POP_EHIP.
 * A wait between workgroups of a fused launch that ran into its time limit (the launch still completes, its
 * results are invalid) is reported once, as POP_EHIP, by the first call that synchronises after it -- pop_sync,
 * pop_update_timed, and pop_get_params / pop_debug_get / pop_act with host pointers -- and then cleared: the
 * population's state is invalid from that step on until the caller restores it (pop_set_params). */
int pop_sync(pop_ctx* ctx);

/* Free the host-side context (never the workspace: Sec. 4.1's single allocation stays the caller's). */
int pop_destroy(pop_ctx* ctx);

/* Message of the last failing call on this context (of the last failing pop_create, pop_workspace_bytes or
 * pop_net_size of this thread when ctx is NULL).  Valid until the next call on the context. */
const char* pop_last_error(const pop_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* POP_H */
