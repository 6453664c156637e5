/*
 * mpe.h -- C ABI of libmpe: batched MPE simple-spread rollouts on one MI355X (gfx950).
 *
 * The calls follow the environment interface of JaxMARL (arXiv 2311.10090, App. C, API
 * listing): reset(key) -> (obs, state) and step(key, state, actions) -> (obs, state,
 * reward, done), with the state an explicit value and the random key explicit.  Here the
 * state lives in device memory owned by the handle (readable and writable through
 * mpe_get_state / mpe_set_state), the key is (seed, run) plus the absolute step counter,
 * and thousands of independent environments advance in lockstep (the paper's vmap over
 * environments, Sec. 2 "Hardware-accelerated environments").  mpe_rollout is the fused
 * T-step loop of policy forward, sampling and environment step that the paper obtains by
 * jit-compiling the scan of its training loop (Sec. 3.2; App. G: 128 rollout steps, two
 * tanh layers of width 64 with parameters shared by all agents).
 *
 * Conventions for every function:
 *   - returns MPE_OK (0) or a negative MPE_E* code; mpe_last_error() then describes it;
 *   - no C++ exception crosses this boundary;
 *   - every data pointer is a DEVICE pointer owned by the caller and at least 16-byte
 *     aligned unless stated otherwise; the library neither frees nor keeps them after the
 *     enqueued work has run (mpe_set_policy copies the weights into its own buffers);
 *   - `stream` is a hipStream_t (NULL = the default stream); work is enqueued on it and the
 *     call returns without waiting; calls on one handle must be stream-ordered by the caller;
 *   - arguments are validated on the host before any device work is enqueued;
 *   - a handle belongs to the device that is current when mpe_create is called: make every later
 *     call on it with that device current (the library never changes the current device), with
 *     pointers and a stream of that device.
 *
 * Sizes: E = num_envs (per run), R = num_runs, TE = R*E, N = num_agents, L = num_landmarks
 * (= N), D = 4 + 2L + 4(N-1) = 6N floats per observation, A = 5 actions.
 * Global env index g = run*E + env.  All trajectory arrays are row-major, env-major
 * inside a time slice: obs[t][g][agent][D], act[t][g][agent], rew[t][g] (rew[t][g][agent] with
 * MPE_REWARD_MIXED and with MPE_SCENARIO_TAG), done[t][g].
 *
 * Second scenario, MPE_SCENARIO_TAG (predator-prey; the paper implements the whole MPE family,
 * App. B.7): agents 0..num_adversaries-1 are adversaries, the other G = N - num_adversaries are
 * good agents; L >= 0 landmarks are fixed obstacles.  Differences from simple spread:
 *   - every agent pair AND every (agent, landmark) pair collides, with contact distance = sum of
 *     the two radii (adv_radius for adversaries, agent_radius for good agents, landmark_radius);
 *   - control force = adv_accel or accel (good agents) times the action's direction; after the
 *     velocity update a velocity longer than adv_max_speed / good_max_speed is scaled to that length;
 *   - rewards are per agent ([TE][N], [T][TE][N]), on the positions after the step; two entities
 *     touch when their centre distance is strictly below the sum of their radii; every adversary
 *     gets 10 * (number of touching (good, adversary) pairs); a good agent gets -10 per adversary
 *     touching it, minus bound(|x|) + bound(|y|), bound(u) = 0 below 0.9, 10 (u - 0.9) below 1,
 *     min(exp(2u - 2), 10) above;
 *   - reset draws landmark coordinates in [-0.9, 0.9): the fp32 product of the grid value and 0.9f;
 *   - observation of agent i, D = 4 + 2L + 2(N-1) + 2G floats: own velocity, own position,
 *     landmarks relative, other agents relative (ascending), velocities of the other good agents
 *     (ascending); a good agent's row ends with two zeros so that all rows have the same length.
 */
#ifndef MPE_H_
#define MPE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MPE_OK       0
#define MPE_EINVAL  (-1)  /* bad config, NULL or misaligned pointer, size out of range */
#define MPE_ESTATE  (-2)  /* call out of order: step/rollout before reset or set_state  */
#define MPE_EHIP    (-3)  /* a HIP runtime call failed; text in mpe_last_error()        */

#define MPE_NUM_ACTIONS 5
#define MPE_MAX_AGENTS  10
#define MPE_MAX_ROLLOUT_STEPS (1 << 24)  /* largest T of one mpe_rollout / mpe_rollout_ac call */

#define MPE_WEIGHTS_FP32 0  /* fp32 weights and layer inputs, fp32 accumulate; the products run on the 16-bit matrix cores on
                             * operands held as sums of fp16 terms: every operand to within one fp32 unit in the last place
                             * (2^-23 relative), the network's outputs as close to a float64 evaluation (1.4e-7 in the mean,
                             * set by the hardware tanh) as with exact operands */
#define MPE_WEIGHTS_BF16 1  /* weights and layer inputs rounded to bf16 (RNE), fp32 accumulate */

/* Reward modes.  SHARED: one value per env, the coverage term  c = -sum_l min_a |p_a - p_l|
 * on the positions after the step.  MIXED: one value per agent; agent i also pays 1 for every
 * other agent whose centre is closer than 2 * agent_radius after the step (strictly), and
 *   r_i = (1 - local_ratio) * c - local_ratio * overlaps_i
 * -- the reward of the CPU implementation that the paper's MPE port corresponds to (App. C:
 * the environments match existing CPU-based implementations, version by version).  Reward
 * arrays then carry N values per env: reward [TE][N], rew_traj [T][TE][N]. */
#define MPE_REWARD_SHARED 0
#define MPE_REWARD_MIXED  1

#define MPE_SCENARIO_SPREAD 0  /* cooperative coverage of N landmarks by N agents           */
#define MPE_SCENARIO_TAG    1  /* predator-prey with obstacle landmarks (see the top comment) */

typedef struct mpe_env mpe_env; /* opaque; host memory owned by the library */

typedef struct {
  int32_t num_envs;          /* E >= 1, environments per run                               */
  int32_t num_agents;        /* N in [1, MPE_MAX_AGENTS]                                   */
  int32_t num_landmarks;     /* L, must equal N (simple-spread); 0..4 with MPE_SCENARIO_TAG */
  int32_t num_runs;          /* R >= 1 independent runs (own RNG key, own policy weights)  */
  int32_t max_episode_steps; /* done fires on this many steps after a reset (25)           */
  float   dt;                /* 0.1                                                        */
  float   damping;           /* 0.25 : v <- v * (1 - damping) + (F / mass) * dt            */
  float   mass;              /* 1                                                          */
  float   accel;             /* 5   : control force = accel * unit direction of the action
                                (tag: of the good agents, 4)                               */
  float   agent_radius;      /* 0.15: agents touch at distance 2 * agent_radius
                                (tag: radius of the good agents, 0.05)                     */
  float   landmark_radius;   /* 0.05: unused by simple spread, whose landmarks never collide
                                (tag: radius of the obstacles, 0.2)                        */
  float   contact_force;     /* 100                                                        */
  float   contact_margin;    /* 1e-3: softness of the softplus penetration                 */
  int32_t hidden;            /* policy width H: 64 or 128 (0 if no policy will be set)     */
  int32_t weight_dtype;      /* MPE_WEIGHTS_FP32 or MPE_WEIGHTS_BF16                       */
  int32_t reward_mode;       /* MPE_REWARD_SHARED or MPE_REWARD_MIXED                      */
  float   local_ratio;       /* in [0, 1]; used by MPE_REWARD_MIXED only (0.5)             */
  int32_t scenario;          /* MPE_SCENARIO_SPREAD or MPE_SCENARIO_TAG                    */
  /* MPE_SCENARIO_TAG only (ignored otherwise; reward_mode and local_ratio are then unused): */
  int32_t num_adversaries;   /* in [1, N-1]: agents 0..num_adversaries-1                   */
  float   adv_radius;        /* 0.075                                                      */
  float   adv_accel;         /* 3                                                          */
  float   adv_max_speed;     /* 1.0 : > 0                                                  */
  float   good_max_speed;    /* 1.3 : > 0                                                  */
} mpe_config;

/* The paper's make(name) (App. C, API listing: an environment object from the registry), with the
 * scenario and its constants given as a struct instead of a name.
 * Validate `cfg` (host only), then allocate the device state of TE environments:
 * pos_a, vel_a [2][N][TE] fp32, pos_l [2][L][TE] fp32, ep_step [TE] int32.
 * MPE_SCENARIO_TAG is built for (N, L, good agents) in (4, 2, 1), (2, 1, 1), (3, 0, 1), (6, 2, 2),
 * (5, 2, 1), (8, 2, 2), (10, 3, 2); MPE_EINVAL for other shapes.
 * `*out` receives the handle.  MPE_EINVAL for a bad config, MPE_EHIP if allocation fails. */
int mpe_create(const mpe_config* cfg, mpe_env** out);

/* Free the handle and its device buffers (synchronises the device first). NULL is allowed.  (The paper's
 * environments are garbage-collected Python objects, App. C; a C handle needs the explicit call.) */
int mpe_destroy(mpe_env* env);

/* Observation length D of this handle (6N; tag: 4 + 2L + 2(N-1) + 2G), or MPE_EINVAL for NULL. */
int mpe_obs_dim(const mpe_env* env);

/* reset(key): start every environment from the seeded initial distribution -- agent and
 * landmark positions uniform on the 24-bit grid of [-1,1)^2, velocities 0, episode counter
 * 0 -- drawn from Philox4x32-10 with key (seed, run) and counter (env, 0, entity, 0).
 * Sets the absolute step counter to 0 and remembers `seed` for later calls.
 * obs: [TE][N][D] fp32 out, may be NULL. */
int mpe_reset(mpe_env* env, uint32_t seed, float* obs, void* stream);

/* step(key, state, actions): one transition of every environment under given actions.
 * actions: [TE][N] uint8 in, values 0..4 (0 none, 1 -x, 2 +x, 3 -y, 4 +y); a value above 4 is
 *          treated as 0 (device data is not read back for validation).
 * obs:     [TE][N][D] fp32 out, observation after the step (of the new episode where done),
 *          may be NULL.
 * reward:  [TE] fp32 out, shared by the env's agents: -sum_l min_a |p_a - p_l| after the step
 *          ([TE][N] per-agent rewards with MPE_REWARD_MIXED and with MPE_SCENARIO_TAG).
 * done:    [TE] uint8 out, 1 when the episode reached max_episode_steps; that env has then
 *          already been reset with counter (env, abs_step + 1, entity, 0).
 * reward and done may be NULL.  Advances the absolute step counter by 1.
 * MPE_ESTATE if neither mpe_reset nor mpe_set_state has been called; MPE_EINVAL if the absolute
 * step counter (a 32-bit word of the Philox counter) would pass 2^32 - 1. */
int mpe_step(mpe_env* env, const uint8_t* actions, float* obs, float* reward, uint8_t* done,
             void* stream);

/* Install (or with all six NULL, remove) the policy used by mpe_rollout:
 *   logits = W3^T tanh(W2^T tanh(W1^T obs + b1) + b2) + b3
 * W1 [R][D][H], b1 [R][H], W2 [R][H][H], b2 [R][H], W3 [R][H][5], b3 [R][5], all fp32,
 * row-major [fan_in][fan_out], device pointers.  The library copies them into its own
 * operand layout on `stream` (rounding W to bf16, ties to even, when weight_dtype is
 * MPE_WEIGHTS_BF16); the caller's arrays are not referenced after that work has run.
 * Policies are built for (num_agents, hidden, weight_dtype) in (1..3, 64, fp32 or bf16), (4..10, 64, fp32)
 * and (4..10, 64 | 128, bf16); with MPE_SCENARIO_TAG for hidden 64, fp32 or bf16, every shape of mpe_create
 * (D <= 32).  MPE_EINVAL for other shapes, if only some pointers are NULL, or if the config has no
 * usable `hidden`. */
int mpe_set_policy(mpe_env* env, const float* W1, const float* b1, const float* W2,
                   const float* b2, const float* W3, const float* b3, void* stream);

/* T fused steps.  For t = 0..T-1: record the current observation, choose every agent's
 * action (policy -- feed-forward or recurrent -- + Gumbel-max with Philox counter (env, abs_step + t,
 * agent, 2|3); or, with no policy, uniform with counter (env, abs_step + t, agent, 1)), record it, apply the
 * transition, record reward and done.
 * obs_traj [T][TE][N][D] fp32, act_traj [T][TE][N] uint8, rew_traj [T][TE] fp32
 * ([T][TE][N] with MPE_REWARD_MIXED and MPE_SCENARIO_TAG), done_traj [T][TE] uint8, last_obs [TE][N][D] fp32
 * (observation after the last step).
 * Any of the five may be NULL (that output is then not written).
 * 1 <= T <= MPE_MAX_ROLLOUT_STEPS.  Advances the absolute step counter by T.  MPE_ESTATE and the counter's
 * limit as for mpe_step.  MPE_EHIP, on this and every later stepping call of the handle, if a kernel of an
 * earlier call gave up one of its bounded waits (it then ran to its end with invalid results; that takes a
 * defect in the library, and the handle is to be destroyed).  With a policy and several runs (one set of weights per run) num_envs must be a multiple
 * of 16 (the policies for 4 and more agents: of 64; of 32 with 8 agents), MPE_EINVAL otherwise;
 * multiples of 64 run fastest. */
int mpe_rollout(mpe_env* env, int32_t T, float* obs_traj, uint8_t* act_traj, float* rew_traj,
                uint8_t* done_traj, float* last_obs, void* stream);

/* Install (or with all ten NULL, remove) a RECURRENT policy for mpe_rollout -- the agent network of
 * the paper's headline speed comparison (Fig. 3: an RNN agent on MPE; App. G "Recurrent network":
 * hidden width 128, two fully-connected layers of width 128).  Per agent, with one carried vector h
 * of 128 floats per agent (zero at every episode start):
 *   e = tanh(We^T obs + be)
 *   r = sigmoid(Wi_r^T e + bi_r + Wh_r^T h + bh_r),  z likewise,
 *   n = tanh(Wi_n^T e + bi_n + r * (Wh_n^T h + bh_n)),  h <- (1 - z) * n + z * h
 *   y = tanh(Wf^T h + bf),  logits = Wo^T y + bo
 * We [R][D][128], be [R][128], Wi, Wh [R][128][384] (columns r | z | n), bi, bh [R][384],
 * Wf [R][128][128], bf [R][128], Wo [R][128][5], bo [R][5] (one set per run): fp32 device pointers,
 * row-major [fan_in][fan_out], copied on `stream`.  The
 * matrices and every vector that enters a matrix product (obs, e, h, y) are rounded to bf16 (ties
 * to even); sums, biases, gate arithmetic and the carried h are fp32.  While installed it takes
 * precedence over the policy of mpe_set_policy.  h is owned by the handle, cleared by mpe_reset and
 * wherever an episode ends inside mpe_rollout, carried across mpe_rollout calls, untouched by
 * mpe_set_state and by mpe_step (which takes its actions from the caller and neither advances nor
 * clears h: a caller that mixes the two sets h itself with mpe_set_hidden).
 * Built for hidden 128 and MPE_WEIGHTS_BF16: MPE_SCENARIO_SPREAD with 1..10 agents and every
 * MPE_SCENARIO_TAG shape mpe_create accepts (D = the scenario's observation length, at most 64);
 * MPE_EINVAL otherwise or if only some pointers are NULL.  With several runs mpe_rollout needs num_envs to be a multiple of 16. */
int mpe_set_gru_policy(mpe_env* env, const float* We, const float* be, const float* Wi, const float* bi,
                       const float* Wh, const float* bh, const float* Wf, const float* bf, const float* Wo,
                       const float* bo, void* stream);

/* Install (or with all four NULL, remove) the critic head of the RECURRENT actor-critic used by
 * mpe_rollout_ac while a recurrent policy is installed (the paper's IPPO with an RNN agent, Sec. 3.2 and
 * App. G: actor and critic share the embedding and the recurrent layer; each has its own fully-connected
 * layer of width 128).  With h' the carried state AFTER this step's update (the vector the actor's second
 * layer reads):
 *   yc = tanh(Wc^T h' + bc),  value = wv^T yc + bv
 * Wc [R][128][128] (row-major [fan_in][fan_out]), bc [R][128], wv [R][128], bv [R]: fp32 device pointers,
 * copied on `stream`.  Wc, wv and the vectors entering the two products (h', yc) are rounded to bf16 (ties
 * to even); sums and biases are fp32.  Needs the configuration of mpe_set_gru_policy (hidden 128,
 * MPE_WEIGHTS_BF16); MPE_EINVAL otherwise or if only some pointers are NULL. */
int mpe_set_gru_critic(mpe_env* env, const float* Wc, const float* bc, const float* wv, const float* bv,
                       void* stream);

/* Copy the carried state of the recurrent policy out / in: hidden [TE][N][128] fp32 device pointer
 * (device to device, on `stream`); mpe_set_hidden(NULL) clears it.  MPE_ESTATE if no recurrent
 * policy has been installed on this handle. */
int mpe_get_hidden(mpe_env* env, float* hidden, void* stream);
int mpe_set_hidden(mpe_env* env, const float* hidden, void* stream);

/* Failure-handling hook.  The rollout kernels whose wavefronts meet at counters in LDS (the large block
 * shapes of mpe_rollout / mpe_rollout_ac) bound every such wait: after `polls` polls a wavefront gives up,
 * the kernel still runs to its end with invalid results, and every later stepping call on the handle
 * returns MPE_EHIP (see mpe_rollout).  The default, 2^24 polls (about a second; a wait normally ends within
 * microseconds), is restored by polls = 0.  A test lowers the limit to a few polls to drive that path from
 * the host; there is no other use for it.  MPE_EINVAL for a NULL handle. */
int mpe_set_barrier_poll_limit(mpe_env* env, uint32_t polls);

/* Install (or with all six NULL, remove) the critic used by mpe_rollout_ac: a second network of
 * the policy's shape with ONE output, fed the agent's own observation (the actor-critic pair of
 * the paper's IPPO, Sec. 3.2; App. G: two tanh layers of width 64):
 *   value = V3^T tanh(V2^T tanh(V1^T obs + c1) + c2) + c3
 * V1 [R][D][H], c1 [R][H], V2 [R][H][H], c2 [R][H], V3 [R][H], c3 [R], fp32 device pointers;
 * copied (and rounded, with MPE_WEIGHTS_BF16) as in mpe_set_policy.  Built for the shapes of
 * mpe_set_policy with MPE_SCENARIO_SPREAD (1..3 agents, hidden 64, fp32 or bf16 weights; 4..10 agents,
 * hidden 64, fp32 weights; 4..10 agents, hidden 64 or 128, bf16 weights), and for MPE_SCENARIO_TAG with hidden 64, fp32 or bf16 weights;
 * MPE_EINVAL otherwise. */
int mpe_set_critic(mpe_env* env, const float* V1, const float* c1, const float* V2,
                   const float* c2, const float* V3, const float* c3, void* stream);

/* mpe_rollout plus what an actor-critic learner takes from a rollout: for every step and agent
 * the log-probability of the sampled action, log pi(a|obs) = z_a - ln sum_k exp(z_k), and the
 * critic's value of the observation acted on; and the value of the observation after the last
 * step (the bootstrap value).
 * logp_traj, value_traj [T][TE][N] fp32, last_value [TE][N] fp32; the other arrays as in
 * mpe_rollout (rewards [T][TE][N] where mpe_rollout's are).  Any of the eight may be NULL.
 * With a recurrent policy installed (mpe_set_gru_policy) the critic is the head of mpe_set_gru_critic:
 * value_traj holds the value of the carried state each step produced, last_value one more evaluation of the
 * network on the observation after the last step, which does not advance the carried state; the carried
 * state moves exactly as under mpe_rollout, and every other output equals mpe_rollout's bit for bit.  Needs
 * a policy and a critic (MPE_ESTATE if one is missing); with several runs num_envs must be a
 * multiple of 16 (fastest: of 256; 4 and more agents: of 64, of 32 with 8 agents and bf16 weights or 7
 * agents and fp32 weights, of 16 with 8 to 10 agents and fp32 weights;
 * MPE_SCENARIO_TAG: fastest with multiples of 512 / num_agents where that divides 64, else of 64, of 32
 * with 10 agents), MPE_EINVAL
 * otherwise. */
int mpe_rollout_ac(mpe_env* env, int32_t T, float* obs_traj, uint8_t* act_traj, float* logp_traj,
                   float* value_traj, float* rew_traj, uint8_t* done_traj, float* last_obs,
                   float* last_value, void* stream);

/* The environment state as an explicit value (App. C: step takes the state and returns the new one;
 * "the state is passed explicitly"): here it lives in the handle and is copied out / in on request, which is
 * also what a checkpoint or a teacher-forced test needs.
 * Copy the state out / in (device to device, on `stream`).  Layouts: pos_a, vel_a
 * [2][N][TE], pos_l [2][L][TE] fp32 (coordinate-major, env fastest), ep_step [TE] int32.
 * Output pointers of mpe_get_state may be NULL individually; abs_step is a HOST pointer
 * (may be NULL).  mpe_set_state needs all four arrays (pos_l may be NULL when there are no
 * landmarks), replaces seed and absolute step counter, and makes the handle steppable. */
int mpe_get_state(mpe_env* env, float* pos_a, float* vel_a, float* pos_l, int32_t* ep_step,
                  uint32_t* abs_step, void* stream);
int mpe_set_state(mpe_env* env, const float* pos_a, const float* vel_a, const float* pos_l,
                  const int32_t* ep_step, uint32_t seed, uint32_t abs_step, void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: mpe_create + mpe_reset(seed) + mpe_set_policy + mpe_rollout(T) in ONE
 * call that allocates nothing (no hipMalloc / hipFree / hipHostMalloc, no handle).  The memory that the
 * handle-based calls own -- the SoA state of the TE environments (pos_a, vel_a, pos_l, ep_step), the packed
 * policy image, one fault word -- is a static device array of MPE_NOALLOC_SCRATCH_BYTES inside the library,
 * one copy per GPU, held until the process ends.
 * cfg: as for mpe_create, MPE_SCENARIO_SPREAD only.  W1..b3: fp32 device pointers laid out as for
 * mpe_set_policy (shapes as there), or all six NULL for seeded uniform actions.  Outputs as for mpe_rollout
 * (any may be NULL); they are bit-identical to those of the four calls above, and the absolute step
 * counter runs 0..T-1.  Nothing survives the call: the final state stays in the scratch array only until
 * the next call on that GPU.
 * MPE_EINVAL if the state of TE environments plus the packed policy does not fit the array
 * (256 + 4 regions rounded up to 256 bytes: 2 x 8 N TE, 8 L TE + 16, 4 TE bytes; + the packed image:
 * 33,344 bytes per run for the fp32 64-wide policies, up to 53,824 for the bf16 ones; 65,536 envs of 3
 * agents need 5.0 MB), and for every argument mpe_create, mpe_set_policy or mpe_rollout would refuse.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 * threads) race, and so would a replay of a captured graph overlapping another call; order them. */
#define MPE_NOALLOC_SCRATCH_BYTES (8u << 20)
int mpe_rollout_noalloc(const mpe_config* cfg, uint32_t seed, const float* W1, const float* b1,
                        const float* W2, const float* b2, const float* W3, const float* b3, int32_t T,
                        float* obs_traj, uint8_t* act_traj, float* rew_traj, uint8_t* done_traj,
                        float* last_obs, void* stream);

/* Text of the calling thread's most recent error ("" if none). Never NULL; static storage.  (C stand-in for
 * the exceptions of the paper's Python interface, App. C.) */
const char* mpe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MPE_H_ */
