/*
 * CPU oracle for the learner's sample-consumption path of the TianJi training
 * system (arXiv 2502.20190): replay ring buffer with policy-version tags,
 * staleness-gated uniform minibatch sampling, and one double-DQN update
 * (online/target forward, TD target, Huber loss, backward, Adam, target sync).
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, fp64 statement of what the
 * path computes, written to be checked against the paper by eye.  Only tests,
 * the smoke check and the CPU-baseline leg of the benchmark may call it.  It
 * shares no code with the HIP library and must never be used as a fallback.
 *
 * What the paper fixes, and where each function takes it from:
 *   - the Buffer component receives transitions pushed by actors holding
 *     different policy versions, and the Learner loads batches from it
 *     (Section 3.1, learner/buffer loops; Section 2.2 on version inconsistency);
 *   - sampling is uniform, not prioritised (Section 2.2, discussion of PER);
 *   - the TD error  delta = r + gamma V(s') - V(s)  and the semi-gradient
 *     update  theta += alpha delta grad V(s)  (Algorithm 1, "Policy update");
 *   - Adam with eps = 1e-8, gamma = 0.99, a periodic hard target update
 *     (Appendix E, Table 2).
 * Everything the paper leaves open (the per-sample staleness gate, double-DQN,
 * Huber, the counter-based generator, Adam's betas) follows textbook
 * definitions; every such reading is listed in the repository's design notes.
 *
 * Parity pins (tests marked "not gpu"): SplitMix64 published vectors, brute-force
 * sampling on tiny rings, the Lag-k closed form of Appendix D.1 / Eq. 2,
 * hand-computed TD targets, Algorithm 1 as a special case, finite differences,
 * numpy / torch library routines for single layers and for a whole step, and
 * Adam closed forms.  The optional bf16-rounding mode is pinned only through
 * the fp64 mode plus a rounding bound: its bit-level behaviour is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Counter-based generator and range reduction                          */
/* ------------------------------------------------------------------ */

/* SplitMix64 (Steele, Lea, Flood 2014): the j-th output of the stream whose
 * state starts at `seed`; the state after j+1 increments is
 * seed + (j+1)*golden-gamma, and the output is its finalised mix. */
uint64_t orc_rng64(uint64_t seed, uint64_t j)
{
    uint64_t z = seed + (j + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* floor(a*b / 2^64): maps a uniform 64-bit draw a onto [0, b). */
uint64_t orc_mulhi64(uint64_t a, uint64_t b)
{
    return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

/* ------------------------------------------------------------------ */
/* Staleness-gated uniform sampling                                      */
/* ------------------------------------------------------------------ */

/* A slot i < count is eligible iff 0 <= cur - version[i] <= max_st.
 * E is the ascending list of eligible slots, K = |E|.  Draw j picks
 * E[ mulhi64(rng64(seed, j), K) ], with replacement.
 * Returns 0 on success, -4 if K == 0 (idx filled with 0xFFFFFFFF). */
/* Sampling while an insert into the arc [ex_begin, ex_begin + ex_len) (mod capacity) has not
 * finished (Section 3.1: buffer and learner loops run asynchronously): slots of the arc are not
 * eligible; everything else as orc_sample. */
int orc_sample_excluding(const int32_t *version, uint64_t count, uint64_t capacity, uint64_t ex_begin,
                         uint64_t ex_len, int64_t cur, int64_t max_st, uint64_t seed, uint32_t batch,
                         uint32_t *idx, uint64_t *K_out)
{
    uint64_t *E = (uint64_t *)malloc((count ? count : 1) * sizeof(uint64_t));
    uint64_t K = 0;
    for (uint64_t i = 0; i < count; ++i) {
        /* i = (ex_begin + t) mod capacity for some t < ex_len  <=>  (i - ex_begin) mod capacity < ex_len */
        int in_arc = ((i + capacity - ex_begin % capacity) % capacity) < ex_len;
        int64_t staleness = cur - (int64_t)version[i];
        if (!in_arc && staleness >= 0 && staleness <= max_st) E[K++] = i;
    }
    if (K_out) *K_out = K;
    if (K == 0) {
        for (uint32_t j = 0; j < batch; ++j) idx[j] = 0xFFFFFFFFu;
        free(E);
        return -4;
    }
    for (uint32_t j = 0; j < batch; ++j) {
        uint64_t k = orc_mulhi64(orc_rng64(seed, j), K);
        idx[j] = (uint32_t)E[k];
    }
    free(E);
    return 0;
}

int orc_sample(const int32_t *version, uint64_t count, int64_t cur, int64_t max_st,
               uint64_t seed, uint32_t batch, uint32_t *idx, uint64_t *K_out)
{
    return orc_sample_excluding(version, count, count ? count : 1, 0, 0, cur, max_st, seed, batch, idx, K_out);
}

/* ------------------------------------------------------------------ */
/* Ring buffer                                                           */
/* ------------------------------------------------------------------ */

typedef struct {
    uint64_t capacity, head, count;
    uint32_t obs_elems, elem_bytes; /* elem_bytes: 4 (f32) or 1 (u8) */
    uint8_t *obs, *next_obs;
    int32_t *action, *version;
    float *reward;
    uint8_t *done;
} orc_buffer;

orc_buffer *orc_buffer_create(uint64_t capacity, uint32_t obs_elems, uint32_t obs_dtype)
{
    orc_buffer *b = (orc_buffer *)calloc(1, sizeof(orc_buffer));
    b->capacity = capacity;
    b->obs_elems = obs_elems;
    b->elem_bytes = obs_dtype == 0 ? 4u : 1u;
    size_t row = (size_t)obs_elems * b->elem_bytes;
    b->obs = (uint8_t *)calloc(capacity, row);
    b->next_obs = (uint8_t *)calloc(capacity, row);
    b->action = (int32_t *)calloc(capacity, sizeof(int32_t));
    b->version = (int32_t *)calloc(capacity, sizeof(int32_t));
    b->reward = (float *)calloc(capacity, sizeof(float));
    b->done = (uint8_t *)calloc(capacity, 1);
    return b;
}

void orc_buffer_destroy(orc_buffer *b)
{
    if (!b) return;
    free(b->obs); free(b->next_obs); free(b->action); free(b->version);
    free(b->reward); free(b->done); free(b);
}

/* Rows go to slots (head+i) mod capacity in order i = 0..n-1, so that on a
 * wrap later rows overwrite earlier ones; then head advances and count
 * saturates at capacity.  Returns -5 (nothing written) if n > capacity. */
int orc_buffer_insert(orc_buffer *b, uint32_t n, const void *obs, const void *next_obs,
                      const int32_t *action, const float *reward, const uint8_t *done,
                      const int32_t *version)
{
    if ((uint64_t)n > b->capacity) return -5;
    size_t row = (size_t)b->obs_elems * b->elem_bytes;
    for (uint32_t i = 0; i < n; ++i) {
        uint64_t s = (b->head + i) % b->capacity;
        memcpy(b->obs + s * row, (const uint8_t *)obs + (size_t)i * row, row);
        memcpy(b->next_obs + s * row, (const uint8_t *)next_obs + (size_t)i * row, row);
        b->action[s] = action[i];
        b->reward[s] = reward[i];
        b->done[s] = done[i];
        b->version[s] = version[i];
    }
    b->head = (b->head + n) % b->capacity;
    b->count = b->count + n < b->capacity ? b->count + n : b->capacity;
    return 0;
}

uint64_t orc_buffer_count(const orc_buffer *b) { return b->count; }
uint64_t orc_buffer_head(const orc_buffer *b) { return b->head; }
const int32_t *orc_buffer_versions(const orc_buffer *b) { return b->version; }

int orc_buffer_sample(const orc_buffer *b, uint32_t batch, int64_t cur, int64_t max_st,
                      uint64_t seed, uint32_t *idx, uint64_t *K_out)
{
    return orc_sample(b->version, b->count, cur, max_st, seed, batch, idx, K_out);
}

/* Minibatch row j is a copy of ring row idx[j], field by field. */
void orc_buffer_gather(const orc_buffer *b, const uint32_t *idx, uint32_t batch, void *obs,
                       void *next_obs, int32_t *action, float *reward, uint8_t *done)
{
    size_t row = (size_t)b->obs_elems * b->elem_bytes;
    for (uint32_t j = 0; j < batch; ++j) {
        uint64_t s = idx[j];
        memcpy((uint8_t *)obs + (size_t)j * row, b->obs + s * row, row);
        memcpy((uint8_t *)next_obs + (size_t)j * row, b->next_obs + s * row, row);
        action[j] = b->action[s];
        reward[j] = b->reward[s];
        done[j] = b->done[s];
    }
}

/* ------------------------------------------------------------------ */
/* Frame ring: one frame per slot, observation stacks rebuilt at sampling  */
/* ------------------------------------------------------------------ */

/* Pixel observations are stacks of the last k frames, so consecutive transitions share k-1 frames
 * of s and s' (Section 4.1 uses Atari with the usual stacked-frame network input).  This ring
 * stores each frame once.  Rows are inserted in time order of one environment stream; row t holds
 * frame f_t, action a_t, reward r_t, done_t and the version tag.  Transition t is
 *   s = (f_{t-b(0)}, ..., f_{t-b(k-1)}),  b(p) = min(k-1-p, age_t),
 *   s' = the stack of row t+1 built the same way with age_{t+1},
 * where age_t = steps since the start of row t's episode, capped at k-1 (a row starts an episode
 * if it is the first ever or follows a row with done = 1): early in an episode the first frame is
 * repeated.  A slot is usable iff it is valid, is not the newest row (its successor is missing),
 * and, once the ring has wrapped, its look-back does not reach past the oldest slot. */
typedef struct {
    uint64_t capacity, head, count;
    uint32_t frame_elems, stack;
    uint8_t *frame, *done, *age;
    int32_t *action, *version;
    float *reward;
    int has_prev;
    uint8_t prev_done, prev_age;
} orc_frame_buffer;

orc_frame_buffer *orc_frame_buffer_create(uint64_t capacity, uint32_t frame_elems, uint32_t stack)
{
    orc_frame_buffer *b = (orc_frame_buffer *)calloc(1, sizeof(orc_frame_buffer));
    b->capacity = capacity; b->frame_elems = frame_elems; b->stack = stack;
    b->frame = (uint8_t *)calloc(capacity, frame_elems);
    b->done = (uint8_t *)calloc(capacity, 1);
    b->age = (uint8_t *)calloc(capacity, 1);
    b->action = (int32_t *)calloc(capacity, 4);
    b->version = (int32_t *)calloc(capacity, 4);
    b->reward = (float *)calloc(capacity, 4);
    return b;
}

void orc_frame_buffer_destroy(orc_frame_buffer *b)
{
    if (!b) return;
    free(b->frame); free(b->done); free(b->age); free(b->action); free(b->version); free(b->reward);
    free(b);
}

int orc_frame_buffer_insert(orc_frame_buffer *b, uint32_t n, const uint8_t *frames, const int32_t *action,
                            const float *reward, const uint8_t *done, const int32_t *version)
{
    if ((uint64_t)n > b->capacity) return -5;
    for (uint32_t i = 0; i < n; ++i) {
        uint64_t s = b->head;
        uint8_t age = 0;
        if (b->has_prev && !b->prev_done) age = (uint32_t)b->prev_age + 1 < b->stack ? (uint8_t)(b->prev_age + 1) : (uint8_t)(b->stack - 1);
        memcpy(b->frame + s * b->frame_elems, frames + (size_t)i * b->frame_elems, b->frame_elems);
        b->action[s] = action[i]; b->reward[s] = reward[i]; b->done[s] = done[i]; b->version[s] = version[i];
        b->age[s] = age;
        b->has_prev = 1; b->prev_done = done[i]; b->prev_age = age;
        b->head = (b->head + 1) % b->capacity;
        if (b->count < b->capacity) b->count += 1;
    }
    return 0;
}

uint64_t orc_frame_buffer_count(const orc_frame_buffer *b) { return b->count; }
uint64_t orc_frame_buffer_head(const orc_frame_buffer *b) { return b->head; }
const uint8_t *orc_frame_buffer_ages(const orc_frame_buffer *b) { return b->age; }
const int32_t *orc_frame_buffer_versions(const orc_frame_buffer *b) { return b->version; }

static int frame_slot_usable(const orc_frame_buffer *b, uint64_t i)
{
    if (i >= b->count) return 0;
    uint64_t newest = (b->head + b->capacity - 1) % b->capacity;
    if (i == newest) return 0;
    if (b->count == b->capacity) {
        uint64_t from_oldest = (i + b->capacity - b->head) % b->capacity;   /* the oldest slot is at head */
        if (from_oldest < b->age[i]) return 0;
    }
    return 1;
}

int orc_frame_buffer_sample(const orc_frame_buffer *b, uint32_t batch, int64_t cur, int64_t max_st,
                            uint64_t seed, uint32_t *idx, uint64_t *K_out)
{
    uint64_t *E = (uint64_t *)malloc((b->count ? b->count : 1) * sizeof(uint64_t));
    uint64_t K = 0;
    for (uint64_t i = 0; i < b->count; ++i) {
        int64_t staleness = cur - (int64_t)b->version[i];
        if (frame_slot_usable(b, i) && staleness >= 0 && staleness <= max_st) E[K++] = i;
    }
    if (K_out) *K_out = K;
    if (K == 0) {
        for (uint32_t j = 0; j < batch; ++j) idx[j] = 0xFFFFFFFFu;
        free(E);
        return -4;
    }
    for (uint32_t j = 0; j < batch; ++j) idx[j] = (uint32_t)E[orc_mulhi64(orc_rng64(seed, j), K)];
    free(E);
    return 0;
}

static void frame_stack_of(const orc_frame_buffer *b, uint64_t t, uint8_t *out)
{
    for (uint32_t p = 0; p < b->stack; ++p) {
        uint32_t back = b->stack - 1 - p;
        if (back > b->age[t]) back = b->age[t];
        uint64_t src = (t + b->capacity - back) % b->capacity;
        memcpy(out + (size_t)p * b->frame_elems, b->frame + src * b->frame_elems, b->frame_elems);
    }
}

void orc_frame_buffer_gather(const orc_frame_buffer *b, const uint32_t *idx, uint32_t batch, uint8_t *obs,
                             uint8_t *next_obs, int32_t *action, float *reward, uint8_t *done)
{
    size_t row = (size_t)b->stack * b->frame_elems;
    for (uint32_t j = 0; j < batch; ++j) {
        uint64_t t = idx[j];
        frame_stack_of(b, t, obs + (size_t)j * row);
        frame_stack_of(b, (t + 1) % b->capacity, next_obs + (size_t)j * row);
        action[j] = b->action[t]; reward[j] = b->reward[t]; done[j] = b->done[t];
    }
}

/* ------------------------------------------------------------------ */
/* Q-network: a chain of conv2d / linear layers, ReLU after all but last */
/* ------------------------------------------------------------------ */

typedef struct {
    int kind; /* 0 linear, 1 conv2d (valid padding, square kernel) */
    int in_c, in_h, in_w;
    int out_c, out_h, out_w;
    int k, stride;
    size_t in_size, out_size, w_off, w_size, b_off;
} orc_layer;

enum { ORC_PARAMS = 0, ORC_TARGET = 1, ORC_GRADS = 2, ORC_ADAM_M = 3, ORC_ADAM_V = 4 };

typedef struct {
    int n_layers;
    orc_layer *L;
    size_t n_params, in_size;
    int n_actions, obs_is_u8, emulate_bf16;
    double gamma, kappa, lr, beta1, beta2, eps;
    int64_t target_interval, t;
    double *theta, *target, *grad, *m, *v;
    /* outputs of the last step, kept for the parity protocol */
    uint32_t last_batch;
    double *q_s, *q_next_online, *q_next_target, *y, *delta;
    int32_t *a_star;
} orc_learner;

/* Round a double to the nearest bfloat16 (ties to even), via fp32. */
static double bf16_round(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan */
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* spec: n_layers rows of 4 ints {kind, out_channels_or_features, kernel, stride}. */
orc_learner *orc_learner_create(const int32_t *spec, int n_layers, int in_c, int in_h, int in_w,
                                int obs_is_u8, double gamma, double kappa, double lr,
                                double beta1, double beta2, double eps, int64_t target_interval,
                                int emulate_bf16)
{
    orc_learner *l = (orc_learner *)calloc(1, sizeof(orc_learner));
    l->n_layers = n_layers;
    l->L = (orc_layer *)calloc((size_t)n_layers, sizeof(orc_layer));
    int c = in_c, h = in_h, w = in_w;
    size_t off = 0;
    l->in_size = (size_t)c * h * w;
    for (int i = 0; i < n_layers; ++i) {
        orc_layer *L = &l->L[i];
        L->kind = spec[4 * i];
        L->out_c = spec[4 * i + 1];
        L->k = spec[4 * i + 2];
        L->stride = spec[4 * i + 3];
        if (L->kind == 1) {
            L->in_c = c; L->in_h = h; L->in_w = w;
            L->out_h = (h - L->k) / L->stride + 1;
            L->out_w = (w - L->k) / L->stride + 1;
            L->w_size = (size_t)L->out_c * c * L->k * L->k;
        } else { /* a linear layer sees its input flattened in (c, h, w) order */
            L->in_c = c * h * w; L->in_h = 1; L->in_w = 1;
            L->out_h = 1; L->out_w = 1;
            L->k = 1; L->stride = 1;
            L->w_size = (size_t)L->out_c * L->in_c;
        }
        L->in_size = (size_t)L->in_c * L->in_h * L->in_w;
        L->out_size = (size_t)L->out_c * L->out_h * L->out_w;
        L->w_off = off; off += L->w_size;
        L->b_off = off; off += (size_t)L->out_c;
        c = L->out_c; h = L->out_h; w = L->out_w;
    }
    l->n_params = off;
    l->n_actions = (int)l->L[n_layers - 1].out_size;
    l->obs_is_u8 = obs_is_u8;
    l->emulate_bf16 = emulate_bf16;
    l->gamma = gamma; l->kappa = kappa; l->lr = lr;
    l->beta1 = beta1; l->beta2 = beta2; l->eps = eps;
    l->target_interval = target_interval;
    l->t = 0;
    l->theta = (double *)calloc(off, sizeof(double));
    l->target = (double *)calloc(off, sizeof(double));
    l->grad = (double *)calloc(off, sizeof(double));
    l->m = (double *)calloc(off, sizeof(double));
    l->v = (double *)calloc(off, sizeof(double));
    return l;
}

static void free_step_outputs(orc_learner *l)
{
    free(l->q_s); free(l->q_next_online); free(l->q_next_target);
    free(l->y); free(l->delta); free(l->a_star);
    l->q_s = l->q_next_online = l->q_next_target = l->y = l->delta = NULL;
    l->a_star = NULL;
}

void orc_learner_destroy(orc_learner *l)
{
    if (!l) return;
    free_step_outputs(l);
    free(l->theta); free(l->target); free(l->grad); free(l->m); free(l->v);
    free(l->L); free(l);
}

uint64_t orc_learner_num_params(const orc_learner *l) { return l->n_params; }
int orc_learner_num_actions(const orc_learner *l) { return l->n_actions; }
int64_t orc_learner_get_t(const orc_learner *l) { return l->t; }
void orc_learner_set_t(orc_learner *l, int64_t t) { l->t = t; }

static double *state_ptr(orc_learner *l, int which)
{
    switch (which) {
    case ORC_PARAMS: return l->theta;
    case ORC_TARGET: return l->target;
    case ORC_GRADS: return l->grad;
    case ORC_ADAM_M: return l->m;
    case ORC_ADAM_V: return l->v;
    default: return NULL;
    }
}

int orc_learner_set_state(orc_learner *l, int which, const double *in)
{
    double *p = state_ptr(l, which);
    if (!p) return -1;
    memcpy(p, in, l->n_params * sizeof(double));
    return 0;
}

int orc_learner_get_state(orc_learner *l, int which, double *out)
{
    double *p = state_ptr(l, which);
    if (!p) return -1;
    memcpy(out, p, l->n_params * sizeof(double));
    return 0;
}

/* z = W x + b for one sample.  Linear: W[out][in].  Conv: W[oc][ic][ky][kx],
 * x[ic][y][x], z[oc][oy][ox], valid padding, stride s. */
static void layer_forward(const orc_layer *L, const double *W, const double *b,
                          const double *x, double *z)
{
    if (L->kind == 0) {
        for (int o = 0; o < L->out_c; ++o) {
            double acc = 0.0;
            for (int i = 0; i < L->in_c; ++i) acc += W[(size_t)o * L->in_c + i] * x[i];
            z[o] = acc + b[o];
        }
        return;
    }
    const int k = L->k, s = L->stride;
    for (int oc = 0; oc < L->out_c; ++oc)
        for (int oy = 0; oy < L->out_h; ++oy)
            for (int ox = 0; ox < L->out_w; ++ox) {
                double acc = 0.0;
                for (int ic = 0; ic < L->in_c; ++ic)
                    for (int ky = 0; ky < k; ++ky)
                        for (int kx = 0; kx < k; ++kx)
                            acc += W[(((size_t)oc * L->in_c + ic) * k + ky) * k + kx] *
                                   x[((size_t)ic * L->in_h + (oy * s + ky)) * L->in_w + (ox * s + kx)];
                z[((size_t)oc * L->out_h + oy) * L->out_w + ox] = acc + b[oc];
            }
}

/* dx = W^T dz for one sample (the transpose of layer_forward without bias). */
static void layer_backward_input(const orc_layer *L, const double *W, const double *dz, double *dx)
{
    memset(dx, 0, L->in_size * sizeof(double));
    if (L->kind == 0) {
        for (int o = 0; o < L->out_c; ++o)
            for (int i = 0; i < L->in_c; ++i) dx[i] += W[(size_t)o * L->in_c + i] * dz[o];
        return;
    }
    const int k = L->k, s = L->stride;
    for (int oc = 0; oc < L->out_c; ++oc)
        for (int oy = 0; oy < L->out_h; ++oy)
            for (int ox = 0; ox < L->out_w; ++ox) {
                double g = dz[((size_t)oc * L->out_h + oy) * L->out_w + ox];
                for (int ic = 0; ic < L->in_c; ++ic)
                    for (int ky = 0; ky < k; ++ky)
                        for (int kx = 0; kx < k; ++kx)
                            dx[((size_t)ic * L->in_h + (oy * s + ky)) * L->in_w + (ox * s + kx)] +=
                                W[(((size_t)oc * L->in_c + ic) * k + ky) * k + kx] * g;
            }
}

/* Gradient of one output channel's weights and bias, summed over the batch in
 * sample order: dW[o] = sum_j dz_j[o] (x) x_j,  db[o] = sum_j dz_j[o]. */
static void layer_backward_params(const orc_layer *L, int o, uint32_t batch, const double *x_all,
                                  const double *dz_all, double *dW, double *db)
{
    if (L->kind == 0) {
        double *row = dW + (size_t)o * L->in_c;
        double bsum = 0.0;
        for (int i = 0; i < L->in_c; ++i) row[i] = 0.0;
        for (uint32_t j = 0; j < batch; ++j) {
            const double *x = x_all + (size_t)j * L->in_size;
            double g = dz_all[(size_t)j * L->out_size + o];
            bsum += g;
            for (int i = 0; i < L->in_c; ++i) row[i] += g * x[i];
        }
        db[o] = bsum;
        return;
    }
    const int k = L->k, s = L->stride;
    double *wo = dW + (size_t)o * L->in_c * k * k;
    double bsum = 0.0;
    for (size_t i = 0; i < (size_t)L->in_c * k * k; ++i) wo[i] = 0.0;
    for (uint32_t j = 0; j < batch; ++j) {
        const double *x = x_all + (size_t)j * L->in_size;
        const double *dz = dz_all + (size_t)j * L->out_size;
        for (int oy = 0; oy < L->out_h; ++oy)
            for (int ox = 0; ox < L->out_w; ++ox) {
                double g = dz[((size_t)o * L->out_h + oy) * L->out_w + ox];
                bsum += g;
                for (int ic = 0; ic < L->in_c; ++ic)
                    for (int ky = 0; ky < k; ++ky)
                        for (int kx = 0; kx < k; ++kx)
                            wo[((size_t)ic * k + ky) * k + kx] +=
                                g * x[((size_t)ic * L->in_h + (oy * s + ky)) * L->in_w + (ox * s + kx)];
            }
    }
    db[o] = bsum;
}

/* Network input h0 for one observation: fp32 values as they are, bytes scaled
 * by 1/255; in bf16 mode the input is rounded like every other GEMM operand. */
static void load_input(const orc_learner *l, const void *obs, size_t j, double *h0)
{
    size_t n = l->in_size;
    if (l->obs_is_u8) {
        const uint8_t *p = (const uint8_t *)obs + j * n;
        for (size_t i = 0; i < n; ++i) h0[i] = (double)p[i] / 255.0;
    } else {
        const float *p = (const float *)obs + j * n;
        for (size_t i = 0; i < n; ++i) h0[i] = (double)p[i];
    }
    if (l->emulate_bf16)
        for (size_t i = 0; i < n; ++i) h0[i] = bf16_round(h0[i]);
}

/* Forward pass of the whole batch with parameters `theta`.
 * acts[i] (optional) receives the input of layer i for every sample,
 * acts[i][j*in_size_i ...]; q receives the head output [batch][n_actions].
 * Hidden layers apply ReLU; the head is linear.  In bf16 mode the weights and
 * the post-ReLU activations are rounded to bf16; bias add and the head output
 * are not. */
static void forward_batch(const orc_learner *l, const double *theta, const void *obs,
                          uint32_t batch, double **acts, double *q, double *min_abs_preact)
{
    double *Wr = NULL;
    const double *P = theta;
    if (l->emulate_bf16) {
        Wr = (double *)malloc(l->n_params * sizeof(double));
        memcpy(Wr, theta, l->n_params * sizeof(double));
        for (int i = 0; i < l->n_layers; ++i)
            for (size_t e = 0; e < l->L[i].w_size; ++e)
                Wr[l->L[i].w_off + e] = bf16_round(Wr[l->L[i].w_off + e]);
        P = Wr;
    }
    size_t max_size = l->in_size;
    for (int i = 0; i < l->n_layers; ++i)
        if (l->L[i].out_size > max_size) max_size = l->L[i].out_size;

#pragma omp parallel
    {
        double *a = (double *)malloc(max_size * sizeof(double));
        double *z = (double *)malloc(max_size * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t j = 0; j < (int64_t)batch; ++j) {
            load_input(l, obs, (size_t)j, a);
            for (int i = 0; i < l->n_layers; ++i) {
                const orc_layer *L = &l->L[i];
                if (acts) memcpy(acts[i] + (size_t)j * L->in_size, a, L->in_size * sizeof(double));
                layer_forward(L, P + L->w_off, P + L->b_off, a, z);
                if (i + 1 < l->n_layers) {
                    if (min_abs_preact)
                        for (size_t e = 0; e < L->out_size; ++e)
                            if (fabs(z[e]) < min_abs_preact[j]) min_abs_preact[j] = fabs(z[e]);
                    for (size_t e = 0; e < L->out_size; ++e) {
                        double r = z[e] > 0.0 ? z[e] : 0.0;
                        a[e] = l->emulate_bf16 ? bf16_round(r) : r;
                    }
                } else {
                    memcpy(q + (size_t)j * L->out_size, z, L->out_size * sizeof(double));
                }
            }
        }
        free(a); free(z);
    }
    free(Wr);
}

/* Q-values of a batch under the online (which = 0) or target (1) network. */
void orc_learner_forward(orc_learner *l, int which, const void *obs, uint32_t batch, double *q)
{
    forward_batch(l, which == 0 ? l->theta : l->target, obs, batch, NULL, q, NULL);
}

/* Policy inference (Algorithm 1, step 1): an epsilon-greedy action for each observation under
 * the online network.  greedy_j = argmax_a Q(s_j, a), lowest index on ties.  Draw j takes two
 * outputs of the sampler's generator: u = rng64(seed, 2j) decides (explore iff its top 24 bits are
 * below floor(epsilon * 2^24)), v = rng64(seed, 2j + 1) picks the uniform action floor(v * A / 2^64).
 * q (optional) receives the Q-values, greedy (optional) the greedy actions. */
void orc_actor_act(orc_learner *l, const void *obs, uint32_t n, double epsilon, uint64_t seed,
                   int32_t *action, double *q, int32_t *greedy)
{
    const int A = l->n_actions;
    double *qq = (double *)malloc((size_t)n * A * sizeof(double));
    forward_batch(l, l->theta, obs, n, NULL, qq, NULL);
    double scaled = epsilon * 16777216.0;
    uint64_t threshold = scaled <= 0.0 ? 0 : (scaled >= 16777216.0 ? 16777216u : (uint64_t)scaled);
    for (uint32_t j = 0; j < n; ++j) {
        int best = 0;
        for (int a = 1; a < A; ++a)
            if (qq[(size_t)j * A + a] > qq[(size_t)j * A + best]) best = a;
        if (greedy) greedy[j] = best;
        uint64_t u = orc_rng64(seed, 2 * (uint64_t)j), v = orc_rng64(seed, 2 * (uint64_t)j + 1);
        action[j] = (u >> 40) < threshold ? (int32_t)orc_mulhi64(v, (uint64_t)A) : best;
    }
    if (q) memcpy(q, qq, (size_t)n * A * sizeof(double));
    free(qq);
}

/* Distance of a batch from the ReLU kinks: the smallest |pre-activation| over
 * all hidden units and samples under the online network.  At a kink the loss
 * gradient jumps, so a comparison of gradients at 1e-4 is only meaningful for
 * inputs that stay clear of them; tests use this to choose such inputs.
 * per_sample (optional) receives the minimum of each sample. */
double orc_learner_min_abs_preactivation(orc_learner *l, const void *obs, uint32_t batch,
                                         double *per_sample)
{
    double *mins = (double *)malloc(batch * sizeof(double));
    double *q = (double *)malloc((size_t)batch * l->n_actions * sizeof(double));
    for (uint32_t j = 0; j < batch; ++j) mins[j] = INFINITY;
    forward_batch(l, l->theta, obs, batch, NULL, q, mins);
    double m = INFINITY;
    for (uint32_t j = 0; j < batch; ++j) {
        if (mins[j] < m) m = mins[j];
        if (per_sample) per_sample[j] = mins[j];
    }
    free(mins); free(q);
    return m;
}

/* Backward pass from dz = dLoss/d(head output) [batch][head width] (consumed) through the
 * network whose layer inputs are acts[i] (freed here), leaving the gradient in l->grad, then one
 * Adam update of l->theta (bias-corrected, eps outside the square root, t counts from 1). */
static void backward_and_adam(orc_learner *l, uint32_t batch, double **acts, double *dz)
{
    const int nl = l->n_layers;
    double *Wr = NULL;
    const double *P = l->theta;
    if (l->emulate_bf16) {
        Wr = (double *)malloc(l->n_params * sizeof(double));
        memcpy(Wr, l->theta, l->n_params * sizeof(double));
        for (int i = 0; i < nl; ++i)
            for (size_t e = 0; e < l->L[i].w_size; ++e)
                Wr[l->L[i].w_off + e] = bf16_round(Wr[l->L[i].w_off + e]);
        P = Wr;
    }
    for (int i = nl - 1; i >= 0; --i) {
        const orc_layer *L = &l->L[i];
        if (l->emulate_bf16)
            for (size_t e = 0; e < (size_t)batch * L->out_size; ++e) dz[e] = bf16_round(dz[e]);
#pragma omp parallel for schedule(static)
        for (int o = 0; o < L->out_c; ++o)
            layer_backward_params(L, o, batch, acts[i], dz, l->grad + L->w_off, l->grad + L->b_off);
        if (i == 0) break;
        double *dx = (double *)malloc((size_t)batch * L->in_size * sizeof(double));
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < (int64_t)batch; ++j) {
            double *dxj = dx + (size_t)j * L->in_size;
            layer_backward_input(L, P + L->w_off, dz + (size_t)j * L->out_size, dxj);
            /* ReLU of the previous layer: derivative 0 where its output is <= 0 */
            const double *h = acts[i] + (size_t)j * L->in_size;
            for (size_t e = 0; e < L->in_size; ++e)
                if (!(h[e] > 0.0)) dxj[e] = 0.0;
        }
        free(dz);
        dz = dx;
    }
    free(dz);
    free(Wr);
    for (int i = 0; i < nl; ++i) free(acts[i]);
    free(acts);

    l->t += 1;
    double c1 = 1.0 - pow(l->beta1, (double)l->t);
    double c2 = 1.0 - pow(l->beta2, (double)l->t);
    for (size_t p = 0; p < l->n_params; ++p) {
        double g = l->grad[p];
        l->m[p] = l->beta1 * l->m[p] + (1.0 - l->beta1) * g;
        l->v[p] = l->beta2 * l->v[p] + (1.0 - l->beta2) * g * g;
        double mhat = l->m[p] / c1, vhat = l->v[p] / c2;
        l->theta[p] -= l->lr * mhat / (sqrt(vhat) + l->eps);
    }
}

/* One learner step on a minibatch.  Returns the loss.
 * astar_override is NULL in normal use.  CPU-only tests that compare the two
 * rounding modes of this file pass one mode's greedy actions to the other, so
 * that a near-tie in the argmax does not turn rounding noise into a jump of
 * the target; values from any other implementation are never passed here. */
double orc_learner_step(orc_learner *l, uint32_t batch, const void *obs, const void *next_obs,
                        const int32_t *action, const float *reward, const uint8_t *done,
                        const int32_t *astar_override)
{
    const int nl = l->n_layers, A = l->n_actions;
    free_step_outputs(l);
    l->last_batch = batch;
    l->q_s = (double *)malloc((size_t)batch * A * sizeof(double));
    l->q_next_online = (double *)malloc((size_t)batch * A * sizeof(double));
    l->q_next_target = (double *)malloc((size_t)batch * A * sizeof(double));
    l->y = (double *)malloc(batch * sizeof(double));
    l->delta = (double *)malloc(batch * sizeof(double));
    l->a_star = (int32_t *)malloc(batch * sizeof(int32_t));

    double **acts = (double **)malloc((size_t)nl * sizeof(double *));
    for (int i = 0; i < nl; ++i)
        acts[i] = (double *)malloc((size_t)batch * l->L[i].in_size * sizeof(double));

    /* forward: Q_online(s) keeps its activations, Q_online(s'), Q_target(s') */
    forward_batch(l, l->theta, obs, batch, acts, l->q_s, NULL);
    forward_batch(l, l->theta, next_obs, batch, NULL, l->q_next_online, NULL);
    forward_batch(l, l->target, next_obs, batch, NULL, l->q_next_target, NULL);

    /* double-DQN target, TD error, Huber loss and its gradient wrt Q(s_j, a_j) */
    double *dz = (double *)calloc((size_t)batch * A, sizeof(double));
    double loss_sum = 0.0;
    for (uint32_t j = 0; j < batch; ++j) {
        const double *qn = l->q_next_online + (size_t)j * A;
        int best = 0;
        for (int a = 1; a < A; ++a)
            if (qn[a] > qn[best]) best = a; /* lowest index wins ties */
        if (astar_override) best = astar_override[j];
        l->a_star[j] = best;
        double not_done = done[j] ? 0.0 : 1.0;
        double y = (double)reward[j] + l->gamma * not_done * l->q_next_target[(size_t)j * A + best];
        double d = l->q_s[(size_t)j * A + action[j]] - y;
        double ad = fabs(d);
        l->y[j] = y;
        l->delta[j] = d;
        loss_sum += ad <= l->kappa ? 0.5 * d * d : l->kappa * (ad - 0.5 * l->kappa);
        double clipped = d > l->kappa ? l->kappa : (d < -l->kappa ? -l->kappa : d);
        dz[(size_t)j * A + action[j]] = clipped / (double)batch;
    }
    double loss = loss_sum / (double)batch;

    /* backward through Q_online(s) only: y is a constant */
    backward_and_adam(l, batch, acts, dz);
    /* periodic hard target update */
    if (l->target_interval > 0 && l->t % l->target_interval == 0)
        memcpy(l->target, l->theta, l->n_params * sizeof(double));
    return loss;
}

/* ------------------------------------------------------------------ */
/* On-policy workload (the PPO column of the appendix hyperparameter    */
/* table: gamma 0.99, GAE 0.95, rollout 512, Adam eps 1e-5).  The paper */
/* names the algorithm only; the estimator is Schulman et al. 2016      */
/* (GAE, Eq. 16) and the objective Schulman et al. 2017 (Eq. 7 and 9).  */
/* ------------------------------------------------------------------ */

/* Generalised advantage estimates of n_env rollouts of T steps each, stored environment-major:
 * reward[e][t], done[e][t], value[e][0..T] (value[e][T] bootstraps the step after the rollout).
 *   delta_t = r_t + gamma * V_{t+1} * (1 - done_t) - V_t
 *   A_t     = delta_t + gamma * lambda * (1 - done_t) * A_{t+1},   A_T = 0
 *   ret_t   = A_t + V_t
 * done_t = 1 means the episode ended with the transition at t: nothing after it leaks back. */
void orc_gae(uint32_t n_env, uint32_t T, const float *reward, const float *value, const uint8_t *done,
             double gamma, double lambda, double *adv, double *ret)
{
    for (uint32_t e = 0; e < n_env; ++e) {
        const float *r = reward + (size_t)e * T, *v = value + (size_t)e * (T + 1);
        const uint8_t *d = done + (size_t)e * T;
        double next = 0.0;
        for (int64_t t = (int64_t)T - 1; t >= 0; --t) {
            double nd = d[t] ? 0.0 : 1.0;
            double delta = (double)r[t] + gamma * (double)v[t + 1] * nd - (double)v[t];
            next = delta + gamma * lambda * nd * next;
            adv[(size_t)e * T + t] = next;
            ret[(size_t)e * T + t] = next + (double)v[t];
        }
    }
}

/* Actor-critic head: the network's last layer has A + 1 outputs, policy logits z_0..z_{A-1} and
 * the state value.  Per sample, with p = softmax(z), rho = p[a] / exp(old_logp):
 *   L_pi = -min(rho * Adv, clip(rho, 1 - c, 1 + c) * Adv)       (clipped surrogate)
 *   L_v  = (V - ret)^2
 *   H    = -sum_a p_a log p_a
 *   loss = mean_j (L_pi + c_v * L_v - c_e * H)
 * out = {mean L_pi, mean L_v, mean H, loss}.  dz (optional) receives dloss/d(head output). */
static void ppo_head(const double *z_all, uint32_t batch, int A, const int32_t *action,
                     const float *old_logp, const float *adv, const float *ret, double clip,
                     double c_v, double c_e, double out[4], double *dz_all)
{
    double s_pi = 0.0, s_v = 0.0, s_h = 0.0;
    for (uint32_t j = 0; j < batch; ++j) {
        const double *z = z_all + (size_t)j * (A + 1);
        double mx = z[0];
        for (int a = 1; a < A; ++a)
            if (z[a] > mx) mx = z[a];
        double se = 0.0;
        for (int a = 0; a < A; ++a) se += exp(z[a] - mx);
        double lse = mx + log(se);
        double H = 0.0;
        for (int a = 0; a < A; ++a) H -= exp(z[a] - lse) * (z[a] - lse);
        double logp = z[action[j]] - lse;
        double rho = exp(logp - (double)old_logp[j]);
        double rc = rho < 1.0 - clip ? 1.0 - clip : (rho > 1.0 + clip ? 1.0 + clip : rho);
        double s1 = rho * (double)adv[j], s2 = rc * (double)adv[j];
        int unclipped = s1 <= s2; /* the minimum is the unclipped term: it carries the gradient */
        double verr = z[A] - (double)ret[j];
        s_pi += -(unclipped ? s1 : s2);
        s_v += verr * verr;
        s_h += H;
        if (dz_all) {
            double *dz = dz_all + (size_t)j * (A + 1);
            for (int a = 0; a < A; ++a) {
                double pa = exp(z[a] - lse);
                double g = 0.0;
                if (unclipped) g += -(double)adv[j] * rho * ((a == action[j] ? 1.0 : 0.0) - pa);
                g += c_e * pa * ((z[a] - lse) + H); /* d(-H)/dz_a = p_a (log p_a + H) */
                dz[a] = g / (double)batch;
            }
            dz[A] = 2.0 * c_v * verr / (double)batch;
        }
    }
    out[0] = s_pi / (double)batch;
    out[1] = s_v / (double)batch;
    out[2] = s_h / (double)batch;
    out[3] = out[0] + c_v * out[1] - c_e * out[2];
}

/* The objective on a batch under the current parameters, nothing updated. */
void orc_ppo_loss(orc_learner *l, uint32_t batch, const void *obs, const int32_t *action,
                  const float *old_logp, const float *adv, const float *ret, double clip, double c_v,
                  double c_e, double out[4])
{
    const int A = l->n_actions - 1;
    double *z = (double *)malloc((size_t)batch * (A + 1) * sizeof(double));
    forward_batch(l, l->theta, obs, batch, NULL, z, NULL);
    ppo_head(z, batch, A, action, old_logp, adv, ret, clip, c_v, c_e, out, NULL);
    free(z);
}

/* One update on the whole batch: forward, objective, backward, Adam. */
void orc_ppo_step(orc_learner *l, uint32_t batch, const void *obs, const int32_t *action,
                  const float *old_logp, const float *adv, const float *ret, double clip, double c_v,
                  double c_e, double out[4])
{
    const int nl = l->n_layers, A = l->n_actions - 1;
    double **acts = (double **)malloc((size_t)nl * sizeof(double *));
    for (int i = 0; i < nl; ++i)
        acts[i] = (double *)malloc((size_t)batch * l->L[i].in_size * sizeof(double));
    double *z = (double *)malloc((size_t)batch * (A + 1) * sizeof(double));
    double *dz = (double *)malloc((size_t)batch * (A + 1) * sizeof(double));
    forward_batch(l, l->theta, obs, batch, acts, z, NULL);
    ppo_head(z, batch, A, action, old_logp, adv, ret, clip, c_v, c_e, out, dz);
    free(z);
    backward_and_adam(l, batch, acts, dz);
}

/* Acting under the stochastic policy (what an actor does between updates): for observation j,
 * p = softmax(logits(s_j)), u_j = (top 24 bits of rng64(seed, j)) / 2^24, the action is the
 * smallest a whose cumulative probability p_0 + ... + p_a exceeds u_j (the last action if rounding
 * leaves none), logp its log-probability, value the head's last output.  margin (optional)
 * receives the distance from u_j to the nearest cumulative probability: a comparison in another
 * precision may legitimately pick a neighbouring action when it is within rounding of zero. */
void orc_ppo_act(orc_learner *l, const void *obs, uint32_t n, uint64_t seed, int32_t *action,
                 double *logp, double *value, double *margin)
{
    const int A = l->n_actions - 1;
    double *z = (double *)malloc((size_t)n * (A + 1) * sizeof(double));
    forward_batch(l, l->theta, obs, n, NULL, z, NULL);
    for (uint32_t j = 0; j < n; ++j) {
        const double *zj = z + (size_t)j * (A + 1);
        double mx = zj[0];
        for (int a = 1; a < A; ++a)
            if (zj[a] > mx) mx = zj[a];
        double se = 0.0;
        for (int a = 0; a < A; ++a) se += exp(zj[a] - mx);
        double lse = mx + log(se);
        double u = (double)(orc_rng64(seed, j) >> 40) / 16777216.0;
        double cdf = 0.0, best = INFINITY;
        int pick = A - 1, found = 0;
        for (int a = 0; a < A; ++a) {
            cdf += exp(zj[a] - lse);
            if (a + 1 < A && fabs(cdf - u) < best) best = fabs(cdf - u);
            if (!found && cdf > u) { pick = a; found = 1; }
        }
        action[j] = pick;
        logp[j] = zj[pick] - lse;
        value[j] = zj[A];
        if (margin) margin[j] = best;
    }
    free(z);
}

/* Per-row outputs of the last step: which = 0 Q_online(s) [B*A], 1 Q_online(s')
 * [B*A], 2 Q_target(s') [B*A], 3 y [B], 4 delta [B]. */
int orc_learner_last(orc_learner *l, int which, double *out)
{
    size_t BA = (size_t)l->last_batch * l->n_actions, B = l->last_batch;
    switch (which) {
    case 0: memcpy(out, l->q_s, BA * sizeof(double)); return 0;
    case 1: memcpy(out, l->q_next_online, BA * sizeof(double)); return 0;
    case 2: memcpy(out, l->q_next_target, BA * sizeof(double)); return 0;
    case 3: memcpy(out, l->y, B * sizeof(double)); return 0;
    case 4: memcpy(out, l->delta, B * sizeof(double)); return 0;
    default: return -1;
    }
}

int orc_learner_last_astar(orc_learner *l, int32_t *out)
{
    memcpy(out, l->a_star, l->last_batch * sizeof(int32_t));
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Production / consumption balance (Section 3.3, Eq. 2-3; Appendix D.1) */
/* ------------------------------------------------------------------ */

/* Serial staleness ratio P = B_s / N_s (Eq. 2).  The learner makes TR_L / B policy versions per
 * second while TR_A transitions per second arrive, so R = TR_A / (TR_L / B) transitions carry one
 * version tag; with v versions inside the gate the eligible pool is v R and one batch is the
 * share B / (v R) of it.  Setting that share to P: v = B / (P R).  v is rounded to the nearest
 * whole number, is at least 1, and v R may not exceed the ring.  out: {max_staleness, R, pool,
 * share, P, min(TR_L, TR_A), cut flag}. */
int orc_balance_plan(double tr_learner, double tr_actor, uint64_t batch, uint64_t serial_batch,
                     uint64_t serial_buffer, uint64_t capacity, double *out)
{
    if (!(tr_learner > 0) || !(tr_actor > 0) || !batch || !serial_batch || serial_buffer < serial_batch || !capacity)
        return -1;
    double P = (double)serial_batch / (double)serial_buffer;
    double versions_per_s = tr_learner / (double)batch;
    double R = tr_actor / versions_per_s;
    double v = floor((double)batch / (P * R) + 0.5);
    if (v < 1) v = 1;
    double cut = 0;
    if (v * R > (double)capacity) {
        cut = 1;
        v = floor((double)capacity / R);
        if (v < 1) v = 1;
    }
    out[0] = v - 1; out[1] = R; out[2] = v * R; out[3] = (double)batch / (v * R); out[4] = P;
    out[5] = tr_learner < tr_actor ? tr_learner : tr_actor; out[6] = cut;
    return 0;
}
