/*
 * tianji.h - C ABI of the MI355X (gfx950) learner hot path of the TianJi RL
 * training system (arXiv 2502.20190).
 *
 * The library implements what the paper's Learner does with the Buffer
 * (Section 3.1: the learner loop loads trajectories, then learns and updates the
 * model; the buffer loop receives what actors push): a device-resident replay
 * ring whose transitions carry the policy version that produced them
 * (Section 2.2: actors hold different policy versions at any time), a
 * staleness-gated uniform minibatch sample (uniform rather than prioritised,
 * Section 2.2), and one batched double-DQN update generalising the TD(0) policy
 * update of Algorithm 1, with the Adam settings of Appendix E, Table 2.
 *
 * Conventions
 *  - Every function returns TJ_OK (0) or a negative tj_status; none throws or
 *    exits.  tj_strerror() names a status.
 *  - "device pointer" = HIP device memory on the current device; "host pointer"
 *    = ordinary host memory.  All bulk device memory (ring arena, minibatch,
 *    learner arena) is owned by the caller and must outlive the handle; the
 *    library never allocates or frees device memory.  Handles are small host
 *    objects owned by the library until the matching destroy call.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *    insert / sample / learner_step only enqueue work on that stream and return
 *    argument errors at once; data-dependent errors are reported through a
 *    sticky device status word read by tj_buffer_status().
 *  - Calls on one handle must be ordered by the caller (same stream, or events).
 */
#ifndef TIANJI_H
#define TIANJI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TJ_OK = 0,
    TJ_ERR_INVALID_ARG = -1,     /* null pointer, zero size, bad enum            */
    TJ_ERR_SHAPE = -2,           /* dimensions the kernels do not support        */
    TJ_ERR_ARENA_TOO_SMALL = -3, /* arena_bytes < tj_*_arena_bytes()             */
    TJ_ERR_NO_ELIGIBLE = -4,     /* a sample found no slot inside the gate       */
    TJ_ERR_CAPACITY = -5,        /* insert of more rows than the ring holds      */
    TJ_ERR_DEVICE = -6,          /* a HIP call failed                            */
    TJ_ERR_SCRATCH_LIMIT = -7    /* tj_sample_noalloc on a ring beyond its limit */
} tj_status;

enum { TJ_OBS_F32 = 0, TJ_OBS_U8 = 1 };
enum { TJ_PRECISION_FP32 = 0, TJ_PRECISION_BF16 = 1 };
enum { TJ_LAYER_LINEAR = 0, TJ_LAYER_CONV2D = 1 };
enum { TJ_MAX_LAYERS = 8 };

typedef struct tj_buffer tj_buffer;
typedef struct tj_learner tj_learner;

/* ---------------------------------------------------------------- buffer */

typedef struct {
    uint64_t capacity;  /* ring slots N, 1 <= N < 2^32 - 1                      */
    uint32_t obs_elems; /* elements of one observation (D, or C*H*W)            */
    uint32_t obs_dtype; /* TJ_OBS_F32 or TJ_OBS_U8                              */
} tj_buffer_desc;

/* A minibatch in caller-owned device memory (structure of arrays):
 * obs, next_obs [batch][obs_elems] in the ring's dtype; action i32, reward f32,
 * done u8, idx u32 [batch] (idx = the sampled ring slots).
 *
 * Indirect form (row_index != NULL, read by tj_learner_step only): obs and
 * next_obs are tables of n_rows rows of obs_elems elements, and row j of the
 * minibatch is row min(row_index[j], n_rows - 1) of each; action, reward and
 * done stay dense.  With obs / next_obs the ring's own arrays
 * (tj_buffer_field_ptr 0 and 1), n_rows the ring's capacity and row_index the
 * idx a tj_sample call produced, the learner's first kernels read the sampled
 * transitions where they lie and no copy of their observations is made: the
 * "load" of the learner loop (Section 3.1) happens inside the update.
 *
 * Indirect by planes (plane_index != NULL; pixel networks only): obs and
 * next_obs both point at one table of n_rows planes of H*W elements (the
 * frame ring's frames, tj_frame_buffer_field_ptr 0), and with C the network's
 * input channels, channel c of s_j is plane
 * min(plane_index[2*C*j + c], n_rows - 1) and channel c of s'_j plane
 * min(plane_index[2*C*j + C + c], n_rows - 1).  tj_frame_sample fills
 * plane_index when it is given no observation destinations.
 * row_index == plane_index == NULL: the dense form, n_rows is ignored; giving
 * both is an error. */
typedef struct {
    void *obs;
    void *next_obs;
    int32_t *action;
    float *reward;
    uint8_t *done;
    uint32_t *idx;
    uint32_t batch;
    uint32_t *row_index;
    uint64_t n_rows;
    uint32_t *plane_index;
} tj_minibatch;

typedef struct {
    uint64_t capacity, head, count; /* ring state (host side)                    */
    uint64_t last_n_eligible;       /* K of the most recent tj_sample            */
    int32_t sticky_error;           /* TJ_OK or TJ_ERR_NO_ELIGIBLE               */
    uint64_t last_excluded_begin;   /* arc of slots the last tj_sample left out   */
    uint64_t last_excluded_len;     /* because an insert into them was in flight  */
} tj_buffer_info;

/* Bytes of device memory tj_buffer_create needs for `desc` (0 if desc is bad). */
size_t tj_buffer_arena_bytes(const tj_buffer_desc *desc);

/* The Buffer component (Section 3.1).  `dev_arena` (device pointer, 256-byte
 * aligned, arena_bytes >= tj_buffer_arena_bytes) holds the ring as a structure
 * of arrays plus the sampler's scratch; the library zeroes its scratch on
 * `hip_stream` and keeps the arena pointer, it does not own it. */
int tj_buffer_create(const tj_buffer_desc *desc, void *dev_arena, size_t arena_bytes,
                     void *hip_stream, tj_buffer **out);

/* Releases the handle; never touches the arena. */
int tj_buffer_destroy(tj_buffer *buf);

/* Buffer receive (Section 3.1, buffer loop): append n transitions, each tagged
 * with the version of the policy that produced it (Section 2.2).  Row i goes to
 * slot (head+i) mod capacity; then head advances and count saturates at
 * capacity.  All six sources are device pointers: d_obs/d_next_obs
 * [n][obs_elems] in the ring's dtype, the others [n].  n > capacity returns
 * TJ_ERR_CAPACITY and writes nothing; n == 0 is a no-op. */
int tj_buffer_insert(tj_buffer *buf, uint32_t n, const void *d_obs, const void *d_next_obs,
                     const int32_t *d_action, const float *d_reward, const uint8_t *d_done,
                     const int32_t *d_version, void *hip_stream);

/* Buffer receive while the learner keeps sampling (Section 3.1: the buffer
 * loop and the learner loop run asynchronously, the learner does not wait for
 * the actors' pushes).  Same effect as tj_buffer_insert, but `insert_stream`
 * may differ from the stream tj_sample runs on, and the library orders the
 * two itself:
 *  - the copy waits, on the device, for every tj_sample issued before this
 *    call (it may overwrite slots those samples still read);
 *  - a later tj_sample leaves out the slots of every insert that was issued
 *    before it but had not finished when its first kernel ran on the device:
 *    slot s is skipped iff (s - begin) mod capacity < len for the arc
 *    [begin, begin+len) those inserts cover, which holds the oldest
 *    transitions of the ring.  The arc the last tj_sample used is reported by
 *    tj_buffer_status.
 * head and count advance at the call, as for tj_buffer_insert.  All concurrent
 * inserts of one buffer go to the same insert_stream; tj_sample calls of one
 * buffer go to one stream at a time (they share the sampler's scratch).  The
 * source rows must stay valid until the copy has run. */
int tj_buffer_insert_concurrent(tj_buffer *buf, uint32_t n, const void *d_obs, const void *d_next_obs,
                                const int32_t *d_action, const float *d_reward, const uint8_t *d_done,
                                const int32_t *d_version, void *insert_stream);

/* Learner load (Section 3.1, learner loop): a slot i < count is eligible iff
 * 0 <= current_version - version[i] <= max_staleness.  With E the ascending
 * list of eligible slots and K = |E|, draw j (0 <= j < batch) takes
 * E[floor(SplitMix64(seed, j) * K / 2^64)] (uniform, with replacement), and
 * minibatch row j is a copy of that ring row.  out->batch must equal `batch`
 * and every pointer in *out is a device pointer of that many rows; out->obs
 * and out->next_obs may both be NULL, then only idx, action, reward and done
 * are produced (for the indirect minibatch form above).  out->row_index and
 * out->n_rows are not read.  The mask is
 * recomputed from the version tags on every call.  Slots under an unfinished
 * tj_buffer_insert_concurrent are not eligible.  K == 0: idx is filled with
 * 0xFFFFFFFF, the other minibatch fields are left untouched and the sticky
 * status becomes TJ_ERR_NO_ELIGIBLE (see tj_buffer_status). */
int tj_sample(tj_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
              uint64_t seed, const tj_minibatch *out, void *hip_stream);

/* tj_sample for callers that cannot allocate device memory or let a library do
 * so on their behalf (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it).  Same arguments, same result, same reporting
 * through tj_buffer_status as tj_sample, but the sampler's scratch (eligibility
 * mask, per-tile counts and offsets) is not taken from the ring arena: it lives
 * in a fixed array inside the library's device image, 557 056 bytes that every
 * GPU the library runs on holds until the process ends.  The call allocates
 * nothing, frees nothing and creates no HIP object.
 *  - Rings of more than TJ_SAMPLE_NOALLOC_MAX_CAPACITY slots are refused with
 *    TJ_ERR_SCRATCH_LIMIT.
 *  - Once tj_buffer_insert_concurrent has been used on `buf`, the first sample
 *    after it must be a tj_sample (it creates the event that orders later
 *    inserts); before that, this call returns TJ_ERR_INVALID_ARG.
 *  - All calls on one GPU share the one array, whatever the buffer or stream:
 *    calls that overlap in time on the same GPU race.  Order them on one stream
 *    or with events.  The array keeps the last call's contents; every word a
 *    call reads it has written itself before. */
#define TJ_SAMPLE_NOALLOC_MAX_CAPACITY 4194304ull
int tj_sample_noalloc(tj_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
                      uint64_t seed, const tj_minibatch *out, void *hip_stream);

/* For callers that hand the ring's own arrays to tj_learner_step (indirect
 * minibatch) while tj_buffer_insert_concurrent is in use: declares that
 * everything enqueued on `hip_stream` so far has finished reading the ring once
 * the stream gets here.  Later concurrent inserts wait for that point, as they
 * wait for the end of a tj_sample, before they overwrite slots.  Call it after
 * the tj_learner_step that consumed the indices, on the same stream, and issue
 * no tj_buffer_insert_concurrent between that tj_sample and this call: such an
 * insert would wait for the sample only and could overwrite rows the update is
 * still reading. */
int tj_buffer_reads_done(tj_buffer *buf, void *hip_stream);

/* Synchronises `hip_stream`, then reports ring state, the last K and the sticky
 * status (which it clears).  Returns the sticky status. */
int tj_buffer_status(tj_buffer *buf, tj_buffer_info *h_out, void *hip_stream);

/* Device pointers into the arena, for tests: field 0 obs, 1 next_obs, 2 action,
 * 3 reward, 4 done, 5 version.  NULL on a bad argument. */
void *tj_buffer_field_ptr(tj_buffer *buf, int field);

/* ---------------------------------------------------------------- frame ring */

/* Replay ring for pixel observations that stores every frame once (Section 4.1
 * evaluates on Atari, whose network input is a stack of the last k frames, so
 * consecutive transitions share k-1 frames of s and s').  Rows are inserted in
 * time order of ONE environment stream: row t holds the u8 frame f_t, a_t, r_t,
 * done_t and the version tag.  Transition t, rebuilt at sampling time, is
 *   s  = (f_{t-b(0)}, ..., f_{t-b(k-1)}),  b(p) = min(k-1-p, age_t),
 *   s' = the stack of row t+1 built in the same way,
 * with age_t = rows since the start of row t's episode, capped at k-1 (a row
 * starts an episode if it is the first ever or follows done = 1), i.e. early in
 * an episode the first frame is repeated.  A slot is eligible iff it passes the
 * staleness gate of tj_sample, is not the newest row, and, once the ring has
 * wrapped, its look-back does not reach past the oldest slot.  Everything else
 * (arena ownership, streams, error reporting, the draw of the indices, the
 * minibatch layout with obs rows of k * frame_elems bytes) is as for tj_buffer. */
typedef struct tj_frame_buffer tj_frame_buffer;

typedef struct {
    uint64_t capacity;    /* ring slots, 2 * stack <= capacity < 2^32 - 1        */
    uint32_t frame_elems; /* bytes of one u8 frame                               */
    uint32_t stack;       /* k, 1 <= k <= 16                                     */
} tj_frame_buffer_desc;

size_t tj_frame_buffer_arena_bytes(const tj_frame_buffer_desc *desc);
int tj_frame_buffer_create(const tj_frame_buffer_desc *desc, void *dev_arena, size_t arena_bytes,
                           void *hip_stream, tj_frame_buffer **out);
int tj_frame_buffer_destroy(tj_frame_buffer *buf);
/* d_frame: device, u8 [n][frame_elems]; the others device [n].  n > capacity
 * returns TJ_ERR_CAPACITY and writes nothing. */
int tj_frame_buffer_insert(tj_frame_buffer *buf, uint32_t n, const uint8_t *d_frame, const int32_t *d_action,
                           const float *d_reward, const uint8_t *d_done, const int32_t *d_version,
                           void *hip_stream);
/* As tj_sample.  With out->obs == out->next_obs == NULL no stack is rebuilt:
 * out->plane_index (device, u32 [batch][2 * stack], required then) receives the
 * slot of every frame of s (positions 0 .. k-1) and of s' (k .. 2k-1) of each
 * drawn transition, all ones where nothing was eligible, for the minibatch
 * form that is indirect by planes. */
int tj_frame_sample(tj_frame_buffer *buf, uint32_t batch, int64_t current_version, int64_t max_staleness,
                    uint64_t seed, const tj_minibatch *out, void *hip_stream);
int tj_frame_buffer_status(tj_frame_buffer *buf, tj_buffer_info *h_out, void *hip_stream);
/* Device pointers for tests: 0 frames, 1 ages (u8), 2 action, 3 reward, 4 done, 5 version. */
void *tj_frame_buffer_field_ptr(tj_frame_buffer *buf, int field);

/* ---------------------------------------------------------------- learner */

typedef struct {
    uint32_t kind;   /* TJ_LAYER_LINEAR or TJ_LAYER_CONV2D (valid padding)       */
    uint32_t out;    /* output features / channels                               */
    uint32_t kernel; /* conv: square kernel size; linear: 0                      */
    uint32_t stride; /* conv: stride; linear: 0                                  */
} tj_layer;

typedef struct {
    uint32_t n_layers;               /* ReLU after every layer but the last       */
    tj_layer layers[TJ_MAX_LAYERS];
    uint32_t in_c, in_h, in_w;       /* one observation; vectors: (D, 1, 1)       */
    uint32_t obs_dtype;              /* TJ_OBS_F32, or TJ_OBS_U8 (scaled by 1/255) */
    uint32_t precision;              /* TJ_PRECISION_FP32 / _BF16 (GEMM operands
                                        bf16, fp32 accumulate, fp32 master)       */
    uint32_t max_batch;
    float gamma, huber_delta;        /* discount (Table 2: 0.99), Huber kappa      */
    float lr, beta1, beta2, eps;     /* Adam (Table 2: eps 1e-8)                   */
    uint32_t target_interval;        /* hard target update period (Table 2), 0 = never */
} tj_learner_desc;

/* Written to device memory by tj_learner_step. */
typedef struct {
    float loss;        /* mean Huber loss of the minibatch                        */
    uint32_t step;     /* t after this step (Adam's step count)                   */
} tj_step_stats;

enum {
    TJ_STATE_PARAMS = 0,  /* online parameters, fp32 master [P]                   */
    TJ_STATE_TARGET = 1,  /* target parameters [P]                                */
    TJ_STATE_GRADS = 2,   /* gradient of the last step [P] (get only)             */
    TJ_STATE_ADAM_M = 3,  /* first moment [P]                                     */
    TJ_STATE_ADAM_V = 4,  /* second moment [P]                                    */
    TJ_STATE_QVALS = 5,   /* last step: Q_online(s), Q_online(s'), Q_target(s'),
                             each [batch][A], concatenated (get only)             */
    TJ_STATE_ASTAR = 6,   /* last step: greedy next actions as floats [batch]
                             (get only)                                           */
    /* The weights as the contraction kernels read them (get only, [P], flat
     * order of TJ_STATE_PARAMS): every weight is the compute-type copy converted
     * back to float (bf16 precision: the round-to-nearest-even image of the
     * master weight; fp32: the master weight itself), biases are the master's.
     * _T reads the transposed copies the input-gradient kernels contract over
     * (layers that keep none read as the straight copy). */
    TJ_STATE_WEIGHTS_COMPUTE = 7,        /* online network                        */
    TJ_STATE_WEIGHTS_COMPUTE_T = 8,      /* online network, transposed copies     */
    TJ_STATE_WEIGHTS_COMPUTE_TARGET = 9  /* target network                        */
};

/* Number of parameters P of the network in `desc` (0 if desc is bad).  Flat
 * order: layer by layer, weight [out][in] (conv [Cout][Cin][kh][kw]; a linear
 * layer after a conv sees its input flattened as (C, H, W)), then bias [out]. */
size_t tj_learner_num_params(const tj_learner_desc *desc);

size_t tj_learner_arena_bytes(const tj_learner_desc *desc);

/* The Learner's model state (Section 3.1).  h_init_online / h_init_target: host
 * pointers to P floats each.  Adam moments start at zero, t at 0.  Copies are
 * enqueued on hip_stream and complete before this returns. */
int tj_learner_create(const tj_learner_desc *desc, void *dev_arena, size_t arena_bytes,
                      const float *h_init_online, const float *h_init_target, void *hip_stream,
                      tj_learner **out);

int tj_learner_destroy(tj_learner *lrn);

/* One policy update (Algorithm 1, "Policy update", batched): with Q_on / Q_tg
 * the online and target networks,
 *   a*_j = argmax_a Q_on(s'_j, a)            (lowest index on ties)
 *   y_j  = r_j + gamma (1 - done_j) Q_tg(s'_j, a*_j)
 *   d_j  = Q_on(s_j, a_j) - y_j
 *   L    = mean_j Huber_kappa(d_j)
 * gradients of L flow through Q_on(s) only; then Adam (bias-corrected, eps added
 * outside the square root) with t = 1, 2, ...; then, if t is a multiple of
 * target_interval, the target parameters become a copy of the online ones.
 * `mb` holds device pointers (idx is not read); mb->batch <= max_batch.  Both
 * forms of the minibatch are accepted (the form by planes by networks whose
 * first layer is a convolution); with an indirect form the tables must
 * stay unchanged until the step's kernels have run (a network whose first
 * layer is a convolution reads them again in its backward pass), and
 * n_rows == 0 is TJ_ERR_INVALID_ARG.
 * Actions are expected in [0, A); the kernels cannot report a bad one, so an
 * action outside that range is read as the nearest valid one (0 or A - 1).
 * d_stats (device pointer, may be NULL) receives loss and t. */
int tj_learner_step(tj_learner *lrn, const tj_minibatch *mb, tj_step_stats *d_stats,
                    void *hip_stream);

/* Policy inference (Algorithm 1, step 1: choose the action with the
 * epsilon-greedy policy of the current weights) for n observations, with the
 * learner's online network: greedy_j = argmax_a Q(s_j, a), lowest index on
 * ties.  Draw j uses two outputs of tj_sample's generator: u = SplitMix64(seed,
 * 2j) decides (explore iff its top 24 bits are below floor(epsilon * 2^24)),
 * v = SplitMix64(seed, 2j+1) gives the uniform action floor(v * A / 2^64).
 * d_obs: device, [n][obs elements] in the learner's observation dtype;
 * d_action, d_version: device int32[n] (the version is the learner's step
 * count, i.e. the version of the weights that chose the action: Section 2.2,
 * actors hold different policy versions); d_q: optional device float[n][A].
 * n <= 2 * max_batch.  Runs on hip_stream in the learner's activation
 * buffers: never concurrently with tj_learner_step of the same handle. */
int tj_actor_act(tj_learner *lrn, uint32_t n, const void *d_obs, float epsilon, uint64_t seed,
                 int32_t *d_action, int32_t *d_version, float *d_q, void *hip_stream);

/* Synchronising host copies of learner state (h_out / h_in: host pointers to n
 * floats; n must match the size given at the enum).  set_state accepts PARAMS,
 * TARGET, ADAM_M, ADAM_V and refreshes the derived weight copies. */
int tj_learner_get_state(tj_learner *lrn, int which, float *h_out, size_t n, void *hip_stream);
int tj_learner_set_state(tj_learner *lrn, int which, const float *h_in, size_t n,
                         void *hip_stream);

/* Adam's step count t (set it together with the moments when resuming). */
int tj_learner_get_step(tj_learner *lrn, uint64_t *h_t);
int tj_learner_set_step(tj_learner *lrn, uint64_t t);

/* ---------------------------------------------------------------- on-policy */

/* The paper's on-policy workload (Section 4 and the PPO column of the appendix
 * hyperparameter table: gamma 0.99, GAE 0.95, rollout length 512, buffer size =
 * batch size, Adam eps 1e-5, lr 1e-4, hidden width 256).  The paper names the
 * algorithm only; the estimator is generalised advantage estimation (Schulman
 * et al. 2016, Eq. 16), the objective PPO's clipped surrogate with value and
 * entropy terms (Schulman et al. 2017, Eq. 7 and 9). */

/* Advantages and returns of n_env rollouts of T steps, environment-major device
 * arrays: d_reward, d_done [n_env][T]; d_value [n_env][T + 1] (what the
 * behaviour policy's critic said at every step, last column = the state after
 * the rollout); outputs d_adv, d_ret float [n_env][T]:
 *   delta_t = r_t + gamma V_{t+1} (1 - done_t) - V_t
 *   A_t     = delta_t + gamma lambda (1 - done_t) A_{t+1},  A_T = 0
 *   ret_t   = A_t + V_t
 * fp32; the recursion is evaluated as a scan of affine maps, so its rounding
 * order differs from the serial one.  n_env == 0 or T == 0: nothing is done. */
int tj_gae(uint32_t n_env, uint32_t T, const float *d_reward, const float *d_value,
           const uint8_t *d_done, float gamma, float lambda, float *d_adv, float *d_ret,
           void *hip_stream);

typedef struct {
    uint32_t obs_dim;                  /* fp32 vector observations                  */
    uint32_t n_hidden;                 /* shared trunk: ReLU layers                 */
    uint32_t hidden[TJ_MAX_LAYERS - 1];
    uint32_t n_actions;                /* 1..63; the head has n_actions + 1 outputs:
                                          logits, then the state value              */
    uint32_t precision;                /* TJ_PRECISION_FP32 / _BF16                 */
    uint32_t max_batch;
    float lr, beta1, beta2, eps;       /* Adam                                      */
    float clip, c_v, c_e;              /* clipping range, value and entropy weights */
} tj_ppo_desc;

/* Device pointers of one batch (the whole buffer: rollouts flattened). */
typedef struct {
    uint32_t batch;
    const float *obs;        /* [batch][obs_dim]                                   */
    const int32_t *action;   /* [batch], in [0, n_actions)                         */
    const float *old_logp;   /* [batch] log-probability under the behaviour policy */
    const float *adv, *ret;  /* [batch] from tj_gae                                */
} tj_ppo_batch;

typedef struct {
    float loss_pi;   /* mean of -min(rho Adv, clip(rho, 1-c, 1+c) Adv)             */
    float loss_v;    /* mean of (V - ret)^2                                        */
    float entropy;   /* mean policy entropy                                        */
    float loss;      /* loss_pi + c_v loss_v - c_e entropy (before the update)     */
    uint32_t step;   /* t after this step                                          */
} tj_ppo_stats;

/* Parameters of the actor-critic network, flat order as tj_learner_num_params. */
size_t tj_ppo_num_params(const tj_ppo_desc *desc);
size_t tj_ppo_arena_bytes(const tj_ppo_desc *desc);

/* An on-policy learner.  The handle is a tj_learner: tj_learner_destroy,
 * tj_learner_get_state / set_state (PARAMS, GRADS, ADAM_M, ADAM_V),
 * tj_learner_get_step / set_step and tj_learner_set_phase_events apply;
 * tj_learner_step and tj_actor_act return TJ_ERR_INVALID_ARG for it.
 * h_init: host pointer to tj_ppo_num_params floats. */
int tj_ppo_create(const tj_ppo_desc *desc, void *dev_arena, size_t arena_bytes, const float *h_init,
                  void *hip_stream, tj_learner **out);

/* One update on the whole batch: with p = softmax(logits(s_j)), rho_j =
 * p[a_j] / exp(old_logp_j) and H_j the entropy of p,
 *   loss = mean_j ( -min(rho_j Adv_j, clip(rho_j, 1-c, 1+c) Adv_j)
 *                   + c_v (V(s_j) - ret_j)^2 - c_e H_j )
 * (where both terms of the minimum are equal the unclipped one carries the
 * gradient), backward through the shared network, Adam as in tj_learner_step.
 * batch->batch <= max_batch; d_stats: optional device pointer. */
int tj_ppo_step(tj_learner *lrn, const tj_ppo_batch *batch, tj_ppo_stats *d_stats, void *hip_stream);

/* Forward pass only, n <= max_batch observations: d_logits float [n][n_actions]
 * and d_value float [n] (either may be NULL).  What an actor needs to act and
 * to fill old_logp and the value columns of tj_gae.  Uses the learner's
 * activation buffers: never concurrently with tj_ppo_step of the same handle. */
int tj_ppo_evaluate(tj_learner *lrn, uint32_t n, const float *d_obs, float *d_logits, float *d_value,
                    void *hip_stream);

/* Acting under the stochastic policy, n <= max_batch observations: with p =
 * softmax(logits(s_j)) and u_j = (top 24 bits of SplitMix64(seed, j)) / 2^24
 * (tj_sample's generator), the action is the first a whose cumulative
 * probability p_0 + ... + p_a exceeds u_j (the last action if rounding leaves
 * none).  d_action int32[n]; d_logp float[n] = log p[action], what
 * tj_ppo_batch.old_logp expects; d_value float[n] (may be NULL) = V(s_j), the
 * value columns of tj_gae.  Same buffers and the same rule about overlapping
 * calls as tj_ppo_evaluate. */
int tj_ppo_act(tj_learner *lrn, uint32_t n, const float *d_obs, uint64_t seed, int32_t *d_action,
               float *d_logp, float *d_value, void *hip_stream);

/* ---------------------------------------------------------------- timing */

/* ---------------------------------------------------------------- balance */

/* Production / consumption balance (Section 3.3, Eq. 2-3; Appendix D.1).  From
 * the measured consumption throughput TR_L of the learner and production
 * throughput TR_A of the actors (transitions per second), the batch B of this
 * deployment and the serial reference (batch B_s, buffer N_s, staleness ratio
 * P = B_s / N_s, Eq. 2), computes the staleness gate for tj_sample that keeps
 * the consumed share of the eligible pool at P:  each policy version tags
 * R = B * TR_A / TR_L transitions, v = max_staleness + 1 versions are
 * eligible, and N_c / N_s' = B / (v R) = P gives v = (N_s / B_s) * TR_L / TR_A,
 * rounded to the nearest whole number, at least 1, and cut to what `capacity`
 * ring slots can hold.  Host arithmetic; all pointers are host pointers.
 * Returns TJ_ERR_INVALID_ARG for non-positive rates or sizes or N_s < B_s. */
typedef struct {
    double tr_learner, tr_actor;          /* TR_L, TR_A: transitions per second  */
    uint64_t batch;                       /* B                                    */
    uint64_t serial_batch, serial_buffer; /* B_s, N_s                             */
    uint64_t capacity;                    /* ring slots                           */
} tj_balance_in;

typedef struct {
    int64_t max_staleness;           /* the gate: v - 1                               */
    double rows_per_version;         /* R                                              */
    double window;                   /* N_s' = v R, transitions eligible when steady   */
    double ratio, target_ratio;      /* B / N_s' achieved, and P                       */
    double throughput;               /* min(TR_L, TR_A), the objective of Eq. 3        */
    int32_t bottleneck;              /* 0 balanced within 5 %, 1 production, 2 consumption */
    int32_t window_exceeds_capacity; /* 1 if v was cut to fit the ring                 */
} tj_balance_out;

int tj_balance_plan(const tj_balance_in *in, tj_balance_out *out);

/* Optional phase timing for benchmarks.  `hip_events` is a host array of
 * hipEvent_t (created by the caller with timing enabled, passed as void*), or
 * NULL / n == 0 to switch timing off.  While set, every tj_sample (and
 * tj_frame_sample of a frame ring) records
 *   [0] start, [1] after mask + scan + select, [2] after the row gather
 * (n must be 3), and every tj_learner_step records
 *   [0] after the input cast, [1] after the forward GEMMs (before the fused
 *   head-layer + TD kernel where that is used, else after the head GEMM),
 *   [2] after the TD / Huber kernel, [3] after the weight- and input-
 *   gradient GEMMs (on a bf16 MLP of three layers or more the last of those
 *   launches also adds up the slices of the hidden layers' split weight
 *   gradients), [4] after the Adam kernel, which for MLPs sums the
 *   slices of the split weight gradients that are still apart (where a layer
 *   still keeps a weight copy that kernel does not write, a copy kernel
 *   follows it) (n must be 5);
 *   every tj_ppo_step records [0] after the input cast, [1] after the forward
 *   GEMMs including the head, [2] after the objective kernel, [3] and [4] as
 *   above (the Adam kernel also finalises the step's statistics),
 * on the call's stream.  The caller reads them after synchronising. */
int tj_buffer_set_phase_events(tj_buffer *buf, void *const *hip_events, uint32_t n);
int tj_frame_buffer_set_phase_events(tj_frame_buffer *buf, void *const *hip_events, uint32_t n);
int tj_learner_set_phase_events(tj_learner *lrn, void *const *hip_events, uint32_t n);

const char *tj_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TIANJI_H */
