/*
 * CPU ORACLE for the Ape-X replay-memory hot path  --  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded C implementation of what the replay memory of
 * "Distributed Prioritized Experience Replay" computes.  It exists so that the HIP
 * library can be checked against something written independently from the paper.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * product path never does.  It shares no source, header or generator with the HIP code.
 * One thing is alike by specification: the mass of a priority has to be the same integer
 * on both sides, so the power p^alpha is ONE specified sequence of fp32 operations with 19
 * specified polynomial coefficients (oracle_pow_spec), typed in here and, again, in the
 * library; what makes that sequence trustworthy is not the library but the pins against
 * the double-precision pow of libm and the exact special cases.
 *
 * Data structures are the textbook ones: a binary array sum-tree of uint64 masses
 * (node[i] = node[2i] + node[2i+1], leaves at node[P2 + slot]) and a ring of slots
 * addressed by monotonically increasing keys (slot = key mod P).
 *
 * Every function names the passage of the paper it follows.  Where the paper is
 * silent the reading taken is written next to the code.
 *
 * Parity pins: every function here is pinned by tests that do not call it back
 * (closed-form n-step returns, brute-force inverse CDF, exact expected sampling
 * frequencies, double-precision pow, hand-worked fixtures; the observation codec by a
 * hand-worked row, closed-form sizes, a second derivation of its mask and counts and the
 * lossless round trip).  Nothing is "parity unpinned".
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -mfma -shared -fPIC apex_oracle.c -lm
 * (-ffp-contract=off: every floating-point rounding below is written out by hand;
 *  -mfma only makes fmaf() a single instruction, it is correctly rounded either way.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
  ORACLE_OK = 0,
  ORACLE_ERR_INVALID_ARG = -1,
  ORACLE_ERR_FULL = -2,
  ORACLE_ERR_NOT_READY = -3,
  ORACLE_ERR_EMPTY = -4,
};

/* ------------------------------------------------------------------------- */
/* p^alpha in fixed point                                                      */
/* ------------------------------------------------------------------------- */

static float f32_from_bits(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t bits_from_f32(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/*
 * x^alpha for x in [2^-100, 2^100], |alpha| <= 1, as a fixed sequence of correctly
 * rounded fp32 operations (Appendix "Implementation", paragraph "Sampling Data":
 * a transition is drawn with probability p^alpha / sum p^alpha).
 *
 * The paper does not say how the power is evaluated.  Because the result is turned
 * into an integer mass that decides sampled indices, it is evaluated here in a way
 * that has one answer on any IEEE-754 machine: x = m * 2^e with m in (sqrt(1/2),
 * sqrt(2)], log2(m) by a degree-10 polynomial in m-1, alpha*(e + log2 m) carried
 * as an unevaluated sum hi + zl, and 2^frac by a degree-7 polynomial.
 */
float oracle_pow_spec(float x, float alpha)
{
  /* log2(1+f)/f on [sqrt(1/2)-1, sqrt(2)-1], least-squares fit at Chebyshev nodes */
  static const float LG[11] = {
    0x1.715476p+0f, -0x1.715476p-1f, 0x1.ec707ep-2f, -0x1.71548cp-2f,
    0x1.2780bap-2f, -0x1.ec7be2p-3f, 0x1.a3e68ap-3f, -0x1.6e459ap-3f,
    0x1.60767ep-3f, -0x1.5b108p-3f,  0x1.8efecp-4f };
  /* 2^r on [-0.53, 0.53] */
  static const float EX[8] = {
    0x1.0p+0f,      0x1.62e43p-1f,  0x1.ebfbep-3f,  0x1.c6b08ep-5f,
    0x1.3b299ep-7f, 0x1.5d8716p-10f, 0x1.449884p-13f, 0x1.00faccp-16f };

  uint32_t u = bits_from_f32(x);
  int e = (int)((u >> 23) & 0xffu) - 127;
  float m = f32_from_bits((u & 0x007fffffu) | 0x3f800000u);   /* [1,2) */
  if (m > 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }           /* (sqrt2/2, sqrt2] */
  float f = m - 1.0f;                                          /* exact */

  float poly = LG[10];
  for (int i = 9; i >= 0; --i) poly = fmaf(poly, f, LG[i]);
  float lm = f * poly;                                         /* log2(m) */

  float ef = (float)e;
  float hi = ef * alpha;
  float lo = fmaf(ef, alpha, -hi);                             /* exact residual of the product */
  float zl = fmaf(alpha, lm, lo);
  float t  = hi + zl;
  float n  = rintf(t);                                         /* round to nearest, ties to even */
  float r  = (hi - n) + zl;

  float ex = EX[7];
  for (int i = 6; i >= 0; --i) ex = fmaf(ex, r, EX[i]);
  float scale = f32_from_bits((uint32_t)((int)n + 127) << 23); /* 2^n, exact */
  return ex * scale;
}

/*
 * Fixed-point mass of a priority p (Appendix "Implementation", "Sampling Data":
 * priority p_k = |delta_k|, sampling weight p_k^alpha).
 * Readings: eps is added to |p| so that a zero TD error keeps a non-zero chance;
 * the mass is floor(p^alpha * 2^F) clamped to [1, qmax]; NaN counts as the smallest
 * admissible input, +inf as the largest.
 */
uint64_t oracle_quantise(float p, float alpha, float eps, uint32_t frac_bits, uint64_t qmax, int *clamped)
{
  float x = fabsf(p) + eps;
  if (!(x >= 0x1p-100f)) x = 0x1p-100f;
  if (x > 0x1p+100f) x = 0x1p+100f;
  float y = oracle_pow_spec(x, alpha);
  float s = y * f32_from_bits((uint32_t)(frac_bits + 127u) << 23);   /* y * 2^F, exact */
  uint64_t q = (s >= 0x1p+62f) ? ((uint64_t)1 << 62) : (uint64_t)s;  /* truncation toward zero */
  int c = 0;
  if (q < 1) { q = 1; c = 1; }
  if (q > qmax) { q = qmax; c = 1; }
  if (clamped) *clamped = c;
  return q;
}

static uint32_t ceil_log2_u64(uint64_t v)
{
  uint32_t l = 0;
  while (((uint64_t)1 << l) < v) ++l;
  return l;
}

/* Largest mass one leaf may hold so that the sum over max_slots leaves stays below 2^63. */
uint64_t oracle_qmax(uint64_t max_slots)
{
  if (max_slots == 0) return (uint64_t)1 << 62;
  return (uint64_t)1 << (62 - ceil_log2_u64(max_slots));
}

/* ------------------------------------------------------------------------- */
/* n-step priorities                                                           */
/* ------------------------------------------------------------------------- */

/*
 * Absolute n-step TD errors of S streams x T transitions (Algorithm 1,
 * ComputePriorities; multi-step double-Q target of the Ape-X DQN section and the
 * critic target of the Ape-X DPG section; Appendix "Implementation", "Adding Data":
 * partial return and accumulated discount per transition, priorities computed in
 * batch from buffered Q-values).
 *
 * Row u of a stream holds what the actor saw when it acted in state S_u:
 * q_online[u,:], q_target[u,:], action[u], the reward received after that action
 * (the paper's R_{u+1}) and the discount returned with it (gamma, or 0 when the
 * episode ended on that step).  Each stream carries T+n rows: the last n are the
 * look-ahead of its final transitions.
 *
 *   R     = sum_{j<n} (prod_{i<j} d[t+i]) r[t+j]      partial return
 *   Gamma = prod_{j<n} d[t+j]                          accumulated discount
 *   boot  = q_target[t+n, argmax_a q_online[t+n,a]]    double-Q bootstrap
 *   delta = R + Gamma*boot - q_online[t, action[t]]
 *
 * A zero discount wipes out everything after it, which is the paper's rule that
 * returns are truncated when the episode ends within the n steps.  With A = 1 the
 * same arithmetic is the DPG critic target (q_target then holds
 * q(S, pi(S)) of the target networks).  Ties in the argmax go to the lowest action.
 * Rounding order: the return by Horner's rule with one fused multiply-add per step,
 * the discount product left to right, the target as one fused multiply-add.
 */
void oracle_nstep_priorities(uint32_t S, uint32_t T, uint32_t n, uint32_t A,
                             const float *q_online, const float *q_target, const int32_t *action,
                             const float *reward, const float *discount,
                             float alpha, float eps, uint32_t frac_bits, uint64_t max_slots,
                             float *prio, float *ret, float *gacc, uint64_t *prio_fx)
{
  const uint64_t qmax = oracle_qmax(max_slots);
  const uint32_t L = T + n;
  for (uint32_t s = 0; s < S; ++s) {
    const float *qo = q_online + (size_t)s * L * A;
    const float *qt = q_target + (size_t)s * L * A;
    const int32_t *ac = action + (size_t)s * L;
    const float *rw = reward + (size_t)s * L;
    const float *dc = discount + (size_t)s * L;
    for (uint32_t t = 0; t < T; ++t) {
      float R = 0.0f;
      for (int j = (int)n - 1; j >= 0; --j) R = fmaf(dc[t + j], R, rw[t + j]);
      float G = 1.0f;
      for (uint32_t j = 0; j < n; ++j) G = G * dc[t + j];
      const float *row = qo + (size_t)(t + n) * A;
      uint32_t best = 0;
      for (uint32_t a = 1; a < A; ++a) if (row[a] > row[best]) best = a;
      float boot = qt[(size_t)(t + n) * A + best];
      float target = fmaf(G, boot, R);
      float delta = target - qo[(size_t)t * A + (uint32_t)ac[t]];
      float p = fabsf(delta);
      size_t o = (size_t)s * T + t;
      ret[o] = R; gacc[o] = G; prio[o] = p;
      if (prio_fx) prio_fx[o] = oracle_quantise(p, alpha, eps, frac_bits, qmax, NULL);
    }
  }
}

/* ------------------------------------------------------------------------- */
/* the replay memory                                                           */
/* ------------------------------------------------------------------------- */

typedef struct oracle_replay {
  uint64_t capacity, max_slots, min_size;
  uint32_t obs_bytes, act_bytes, frac_bits;
  float alpha, eps;
  uint64_t qmax;
  uint64_t P2;            /* leaves of the binary tree: next power of two >= max_slots */
  uint64_t *node;         /* [2*P2] */
  uint64_t head, tail;    /* valid keys are head <= key < tail */
  uint64_t payload_slots; /* 0: no payload kept; else rows live at slot mod payload_slots */
  uint8_t *obs, *act;
  float *ret, *gacc;
  uint64_t n_stale, n_clamped;
} oracle_replay;

static void set_leaf(oracle_replay *r, uint64_t slot, uint64_t v)
{
  uint64_t j = r->P2 + slot;
  r->node[j] = v;
  for (j >>= 1; j >= 1; j >>= 1) r->node[j] = r->node[2 * j] + r->node[2 * j + 1];
}

oracle_replay *oracle_replay_create(uint64_t capacity, uint64_t max_slots, uint32_t obs_bytes, uint32_t act_bytes,
                                    float alpha, float eps, uint32_t frac_bits, uint64_t min_size,
                                    uint64_t payload_slots)
{
  if (capacity == 0 || max_slots < capacity || frac_bits > 32 || !(alpha >= -1.0f && alpha <= 1.0f) || !(eps >= 0.0f))
    return NULL;
  oracle_replay *r = (oracle_replay *)calloc(1, sizeof *r);
  if (!r) return NULL;
  r->capacity = capacity; r->max_slots = max_slots; r->min_size = min_size;
  r->obs_bytes = obs_bytes; r->act_bytes = act_bytes; r->frac_bits = frac_bits;
  r->alpha = alpha; r->eps = eps;
  r->qmax = oracle_qmax(max_slots);
  r->P2 = 1; while (r->P2 < max_slots) r->P2 <<= 1;
  r->node = (uint64_t *)calloc(2 * r->P2, sizeof(uint64_t));
  if (payload_slots > max_slots) payload_slots = max_slots;
  r->payload_slots = payload_slots;
  if (payload_slots) {
    r->obs = (uint8_t *)calloc(payload_slots, obs_bytes ? obs_bytes : 1);
    r->act = (uint8_t *)calloc(payload_slots, act_bytes ? act_bytes : 1);
    r->ret = (float *)calloc(payload_slots, sizeof(float));
    r->gacc = (float *)calloc(payload_slots, sizeof(float));
  }
  if (!r->node || (payload_slots && (!r->obs || !r->act || !r->ret || !r->gacc))) {
    free(r->node); free(r->obs); free(r->act); free(r->ret); free(r->gacc); free(r);
    return NULL;
  }
  return r;
}

void oracle_replay_destroy(oracle_replay *r)
{
  if (!r) return;
  free(r->node); free(r->obs); free(r->act); free(r->ret); free(r->gacc); free(r);
}

/*
 * replay.Add (Algorithm 1; Appendix "Implementation", "Adding Data"): every new
 * transition gets a unique key (here the running insertion count), is stored, and
 * enters the sampling distribution at once with the priority its actor computed.
 * Reading: the soft capacity never refuses data (Atari experiments: adding is always
 * permitted); only the physical ring can be full, and then nothing is written.
 */
int oracle_replay_add(oracle_replay *r, uint64_t count, const uint8_t *obs, const uint8_t *act,
                      const float *ret, const float *gacc, const float *prio, uint64_t *first_key)
{
  if (!r || (count && !prio)) return ORACLE_ERR_INVALID_ARG;
  if ((r->tail - r->head) + count > r->max_slots) return ORACLE_ERR_FULL;
  if (first_key) *first_key = r->tail;
  for (uint64_t i = 0; i < count; ++i) {
    uint64_t key = r->tail + i, slot = key % r->max_slots;
    if (r->payload_slots) {
      uint64_t ps = slot % r->payload_slots;
      if (obs) memcpy(r->obs + ps * r->obs_bytes, obs + i * r->obs_bytes, r->obs_bytes);
      if (act) memcpy(r->act + ps * r->act_bytes, act + i * r->act_bytes, r->act_bytes);
      if (ret) r->ret[ps] = ret[i];
      if (gacc) r->gacc[ps] = gacc[i];
    }
    int c;
    set_leaf(r, slot, oracle_quantise(prio[i], r->alpha, r->eps, r->frac_bits, r->qmax, &c));
    r->n_clamped += (uint64_t)c;
  }
  r->tail += count;
  return ORACLE_OK;
}

static uint64_t mulhi64(uint64_t a, uint64_t b) { return (uint64_t)(((unsigned __int128)a * b) >> 64); }

/*
 * replay.Sample (Algorithm 2; Appendix "Implementation", "Sampling Data"):
 * num_batches independent batches of k transitions, each transition drawn with
 * probability mass/total, all batches from the same state of the memory (the
 * learner prefetches several batches ahead of the updates they will receive).
 *
 * The paper names proportional prioritisation and gives the probability only.
 * Readings: a batch is stratified -- [0,total) is cut into k equal integer strata of
 * width w = floor(total/k) and sample j takes the point j*w + floor(rnd*w / 2^64) of
 * its own stratum; the transition drawn is the one whose interval of the cumulative
 * mass, in slot order, holds that point.  Importance weights are (N * P(i))^-beta
 * with N the number of stored transitions, divided by the largest weight in the same
 * batch of k.
 */
int oracle_replay_sample(oracle_replay *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                         uint64_t *key_out, uint32_t *slot_out, float *weight_out, uint64_t *mass_out,
                         uint8_t *obs_out, uint8_t *act_out, float *ret_out, float *gacc_out)
{
  if (!r || !k || !num_batches || !rnd || !slot_out) return ORACLE_ERR_INVALID_ARG;
  const uint64_t size = r->tail - r->head;
  if (size < r->min_size) return ORACLE_ERR_NOT_READY;
  if (size == 0) return ORACLE_ERR_EMPTY;
  const uint64_t total = r->node[1];
  const uint64_t w = total / k;
  const uint64_t P = r->max_slots;
  double *wt = (double *)malloc(sizeof(double) * k);
  if (!wt) return ORACLE_ERR_INVALID_ARG;
  for (uint32_t b = 0; b < num_batches; ++b) {
    double wmax = 0.0;
    for (uint32_t j = 0; j < k; ++j) {
      size_t o = (size_t)b * k + j;
      uint64_t x = (uint64_t)j * w + mulhi64(rnd[o], w);
      uint64_t node = 1;
      while (node < r->P2) {
        uint64_t left = r->node[2 * node];
        if (x < left) node = 2 * node;
        else { x -= left; node = 2 * node + 1; }
      }
      uint64_t slot = node - r->P2;
      uint64_t mass = r->node[node];
      uint64_t key = r->head + ((slot + P - r->head % P) % P);
      slot_out[o] = (uint32_t)slot;
      if (key_out) key_out[o] = key;
      if (mass_out) mass_out[o] = mass;
      double prob = (double)mass / (double)total;
      wt[j] = pow((double)size * prob, -(double)beta);
      if (wt[j] > wmax) wmax = wt[j];
      if (r->payload_slots) {
        uint64_t ps = slot % r->payload_slots;
        if (obs_out) memcpy(obs_out + o * r->obs_bytes, r->obs + ps * r->obs_bytes, r->obs_bytes);
        if (act_out) memcpy(act_out + o * r->act_bytes, r->act + ps * r->act_bytes, r->act_bytes);
        if (ret_out) ret_out[o] = r->ret[ps];
        if (gacc_out) gacc_out[o] = r->gacc[ps];
      }
    }
    if (weight_out)
      for (uint32_t j = 0; j < k; ++j) weight_out[(size_t)b * k + j] = (float)(wt[j] / wmax);
  }
  free(wt);
  return ORACLE_OK;
}

/*
 * The same draw by the plain definition, with no tree: walk the leaves in slot
 * order and stop where the running sum passes the stratum point.  Used to pin the
 * tree descent on small memories.
 */
int oracle_replay_sample_linear(const oracle_replay *r, uint32_t k, const uint64_t *rnd, uint32_t *slot_out)
{
  if (!r || !k) return ORACLE_ERR_INVALID_ARG;
  uint64_t total = 0;
  for (uint64_t i = 0; i < r->max_slots; ++i) total += r->node[r->P2 + i];
  const uint64_t w = total / k;
  for (uint32_t j = 0; j < k; ++j) {
    uint64_t x = (uint64_t)j * w + mulhi64(rnd[j], w);
    uint64_t run = 0, i = 0;
    for (; i < r->max_slots; ++i) {
      uint64_t m = r->node[r->P2 + i];
      if (x < run + m) break;
      run += m;
    }
    slot_out[j] = (uint32_t)i;
  }
  return ORACLE_OK;
}

/*
 * replay.SetPriority (Algorithm 2): the learner writes back new absolute TD errors
 * for the keys it sampled.  Readings: pairs are applied one after the other, so the
 * last of several pairs naming one key stands; a key that has been removed since it
 * was sampled is no longer in the set of valid keys and its pair is skipped.
 */
int oracle_replay_update_priorities(oracle_replay *r, uint64_t m, const uint64_t *key, const float *prio)
{
  if (!r || (m && (!key || !prio))) return ORACLE_ERR_INVALID_ARG;
  for (uint64_t i = 0; i < m; ++i) {
    if (key[i] < r->head || key[i] >= r->tail) { r->n_stale++; continue; }
    int c;
    set_leaf(r, key[i] % r->max_slots, oracle_quantise(prio[i], r->alpha, r->eps, r->frac_bits, r->qmax, &c));
    r->n_clamped += (uint64_t)c;
  }
  return ORACLE_OK;
}

/*
 * ComputePriorities of Algorithm 2 followed by replay.SetPriority: the learner's new priority of a
 * sampled transition is the absolute n-step TD error again, now with the Q-values of the current
 * networks, and with the partial return and accumulated discount that were stored with the
 * transition (Appendix "Implementation", "Adding Data"):
 *     | ret + gacc * q_target_next[argmax_a q_online_next[a]] - q_taken |
 * Needs a memory that keeps its payload un-aliased.  Pairs are applied one after the other; a
 * pair whose key is no longer valid is skipped and reports priority 0.
 */
int oracle_replay_update_from_q(oracle_replay *r, uint64_t m, const uint64_t *key, uint32_t A, const float *q_taken,
                                const float *q_online_next, const float *q_target_next, float *prio_out)
{
  if (!r || !A || r->payload_slots != r->max_slots || (m && (!key || !q_taken || !q_online_next || !q_target_next)))
    return ORACLE_ERR_INVALID_ARG;
  for (uint64_t i = 0; i < m; ++i) {
    if (key[i] < r->head || key[i] >= r->tail) {
      r->n_stale++;
      if (prio_out) prio_out[i] = 0.0f;
      continue;
    }
    const uint64_t slot = key[i] % r->max_slots;
    const float *row = q_online_next + i * A;
    uint32_t best = 0;
    for (uint32_t a = 1; a < A; ++a) if (row[a] > row[best]) best = a;
    const float boot = q_target_next[i * A + best];
    const float target = fmaf(r->gacc[slot], boot, r->ret[slot]);
    const float p = fabsf(target - q_taken[i]);
    if (prio_out) prio_out[i] = p;
    int c;
    set_leaf(r, slot, oracle_quantise(p, r->alpha, r->eps, r->frac_bits, r->qmax, &c));
    r->n_clamped += (uint64_t)c;
  }
  return ORACLE_OK;
}

/*
 * replay.RemoveToFit (Algorithm 2; Atari experiments): whatever exceeds the soft
 * capacity is removed in one go, oldest first.
 */
int oracle_replay_evict(oracle_replay *r, uint64_t *evicted)
{
  if (!r) return ORACLE_ERR_INVALID_ARG;
  uint64_t size = r->tail - r->head;
  uint64_t e = size > r->capacity ? size - r->capacity : 0;
  for (uint64_t key = r->head; key < r->head + e; ++key) set_leaf(r, key % r->max_slots, 0);
  r->head += e;
  if (evicted) *evicted = e;
  return ORACLE_OK;
}

/* read-only views for tests */
uint64_t oracle_replay_head(const oracle_replay *r) { return r->head; }
uint64_t oracle_replay_tail(const oracle_replay *r) { return r->tail; }
uint64_t oracle_replay_root(const oracle_replay *r) { return r->node[1]; }
uint64_t oracle_replay_n_stale(const oracle_replay *r) { return r->n_stale; }
uint64_t oracle_replay_n_clamped(const oracle_replay *r) { return r->n_clamped; }
uint64_t oracle_replay_tree_leaves(const oracle_replay *r) { return r->P2; }
const uint64_t *oracle_replay_nodes(const oracle_replay *r) { return r->node; }
void oracle_replay_leaves(const oracle_replay *r, uint64_t first, uint64_t count, uint64_t *out)
{
  memcpy(out, r->node + r->P2 + first, count * sizeof(uint64_t));
}

/* ------------------------------------------------------------------------- */
/* the replay memory with prioritized eviction                                 */
/* ------------------------------------------------------------------------- */

/*
 * Appendix "Continuous Control: Additional Details": to hold the memory at its capacity,
 * transitions are periodically evicted by proportional prioritized sampling with its own
 * exponent (alpha_evict = -0.4: transitions with small TD error go first), instead of oldest
 * first.  Sampling for the learner is unchanged.
 *
 * Readings (the paper gives the rule in one sentence):
 *  - a second sum tree holds the eviction masses Q(p; alpha_evict) of the same transitions;
 *  - slots freed by an eviction are re-used by later adds in the order in which they were freed
 *    (a ring of free slots, initially 0, 1, 2, ...), so a key can no longer be the insertion
 *    count: key = (generation of the slot << 32) | slot, the generation counting the slot's
 *    tenants; a key is valid while its generation is the slot's and the slot is occupied;
 *  - to evict e = size - capacity transitions without replacement: in each round draw as many
 *    stratified points as are still to go on the eviction tree as it stands at the start of the
 *    round (same stratum rule as for sampling); a transition drawn more than once counts once
 *    (such repeats are neighbours, the points being ordered); remove the distinct ones in the
 *    order of their points; repeat with what is left, for at most `rounds` rounds.
 */
typedef struct oracle_pe {
  uint64_t capacity, max_slots;
  uint32_t obs_bytes, act_bytes, frac_bits;
  float alpha, alpha_evict, eps;
  uint64_t qmax, P2;
  uint64_t *ts, *te;       /* sampling tree, eviction tree: [2*P2] each */
  uint32_t *gen;           /* [P] tenants seen by each slot */
  uint32_t *free_ring;     /* [P] */
  uint64_t free_head, free_tail, inserted, evicted;
  int payload;
  uint8_t *obs, *act;
  float *ret, *gacc;
  uint64_t n_stale, n_clamped;
} oracle_pe;

static void tree_set(uint64_t *node, uint64_t P2, uint64_t slot, uint64_t v)
{
  uint64_t j = P2 + slot;
  node[j] = v;
  for (j >>= 1; j >= 1; j >>= 1) node[j] = node[2 * j] + node[2 * j + 1];
}

static uint64_t tree_find(const uint64_t *node, uint64_t P2, uint64_t x)
{
  uint64_t j = 1;
  while (j < P2) {
    uint64_t left = node[2 * j];
    if (x < left) j = 2 * j;
    else { x -= left; j = 2 * j + 1; }
  }
  return j - P2;
}

void oracle_pe_destroy(oracle_pe *r)
{
  if (!r) return;
  free(r->ts); free(r->te); free(r->gen); free(r->free_ring);
  free(r->obs); free(r->act); free(r->ret); free(r->gacc); free(r);
}

oracle_pe *oracle_pe_create(uint64_t capacity, uint64_t max_slots, uint32_t obs_bytes, uint32_t act_bytes, float alpha,
                            float alpha_evict, float eps, uint32_t frac_bits, int payload)
{
  if (capacity == 0 || max_slots < capacity || max_slots > ((uint64_t)1 << 31) || frac_bits > 32 ||
      !(alpha >= -1.0f && alpha <= 1.0f) || !(alpha_evict >= -1.0f && alpha_evict <= 1.0f) || !(eps >= 0.0f))
    return NULL;
  oracle_pe *r = (oracle_pe *)calloc(1, sizeof *r);
  if (!r) return NULL;
  r->capacity = capacity; r->max_slots = max_slots;
  r->obs_bytes = obs_bytes; r->act_bytes = act_bytes; r->frac_bits = frac_bits;
  r->alpha = alpha; r->alpha_evict = alpha_evict; r->eps = eps;
  r->qmax = oracle_qmax(max_slots);
  r->P2 = 1; while (r->P2 < max_slots) r->P2 <<= 1;
  r->ts = (uint64_t *)calloc(2 * r->P2, 8);
  r->te = (uint64_t *)calloc(2 * r->P2, 8);
  r->gen = (uint32_t *)calloc(max_slots, 4);
  r->free_ring = (uint32_t *)calloc(max_slots, 4);
  r->payload = payload;
  if (payload) {
    r->obs = (uint8_t *)calloc(max_slots, obs_bytes ? obs_bytes : 1);
    r->act = (uint8_t *)calloc(max_slots, act_bytes ? act_bytes : 1);
    r->ret = (float *)calloc(max_slots, 4);
    r->gacc = (float *)calloc(max_slots, 4);
  }
  if (!r->ts || !r->te || !r->gen || !r->free_ring || (payload && (!r->obs || !r->act || !r->ret || !r->gacc))) {
    oracle_pe_destroy(r);
    return NULL;
  }
  for (uint64_t i = 0; i < max_slots; ++i) r->free_ring[i] = (uint32_t)i;
  r->free_head = 0;
  r->free_tail = max_slots;
  return r;
}

static uint64_t pe_size(const oracle_pe *r) { return r->max_slots - (r->free_tail - r->free_head); }

static void pe_set_priority(oracle_pe *r, uint64_t slot, float p)
{
  int c1, c2;
  tree_set(r->ts, r->P2, slot, oracle_quantise(p, r->alpha, r->eps, r->frac_bits, r->qmax, &c1));
  tree_set(r->te, r->P2, slot, oracle_quantise(p, r->alpha_evict, r->eps, r->frac_bits, r->qmax, &c2));
  r->n_clamped += (uint64_t)(c1 + c2);
}

int oracle_pe_add(oracle_pe *r, uint64_t count, const uint8_t *obs, const uint8_t *act, const float *ret,
                  const float *gacc, const float *prio, uint64_t *key_out)
{
  if (!r || (count && !prio)) return ORACLE_ERR_INVALID_ARG;
  if (pe_size(r) + count > r->max_slots) return ORACLE_ERR_FULL;
  for (uint64_t i = 0; i < count; ++i) {
    const uint64_t slot = r->free_ring[(r->free_head + i) % r->max_slots];
    r->gen[slot] += 1;
    if (r->payload) {
      if (obs) memcpy(r->obs + slot * r->obs_bytes, obs + i * r->obs_bytes, r->obs_bytes);
      if (act) memcpy(r->act + slot * r->act_bytes, act + i * r->act_bytes, r->act_bytes);
      if (ret) r->ret[slot] = ret[i];
      if (gacc) r->gacc[slot] = gacc[i];
    }
    pe_set_priority(r, slot, prio[i]);
    if (key_out) key_out[i] = ((uint64_t)r->gen[slot] << 32) | slot;
  }
  r->free_head += count;
  r->inserted += count;
  return ORACLE_OK;
}

int oracle_pe_sample(oracle_pe *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                     uint64_t *key_out, uint32_t *slot_out, float *weight_out, uint64_t *mass_out, uint8_t *obs_out,
                     uint8_t *act_out, float *ret_out, float *gacc_out)
{
  if (!r || !k || !num_batches || !rnd || !slot_out) return ORACLE_ERR_INVALID_ARG;
  const uint64_t size = pe_size(r);
  if (size == 0) return ORACLE_ERR_EMPTY;
  const uint64_t total = r->ts[1], w = total / k;
  double *wt = (double *)malloc(sizeof(double) * k);
  if (!wt) return ORACLE_ERR_INVALID_ARG;
  for (uint32_t b = 0; b < num_batches; ++b) {
    double wmax = 0.0;
    for (uint32_t j = 0; j < k; ++j) {
      const size_t o = (size_t)b * k + j;
      const uint64_t x = (uint64_t)j * w + mulhi64(rnd[o], w);
      const uint64_t slot = tree_find(r->ts, r->P2, x);
      const uint64_t mass = r->ts[r->P2 + slot];
      slot_out[o] = (uint32_t)slot;
      if (key_out) key_out[o] = ((uint64_t)r->gen[slot] << 32) | slot;
      if (mass_out) mass_out[o] = mass;
      wt[j] = pow((double)size * ((double)mass / (double)total), -(double)beta);
      if (wt[j] > wmax) wmax = wt[j];
      if (r->payload) {
        if (obs_out) memcpy(obs_out + o * r->obs_bytes, r->obs + slot * r->obs_bytes, r->obs_bytes);
        if (act_out) memcpy(act_out + o * r->act_bytes, r->act + slot * r->act_bytes, r->act_bytes);
        if (ret_out) ret_out[o] = r->ret[slot];
        if (gacc_out) gacc_out[o] = r->gacc[slot];
      }
    }
    if (weight_out)
      for (uint32_t j = 0; j < k; ++j) weight_out[(size_t)b * k + j] = (float)(wt[j] / wmax);
  }
  free(wt);
  return ORACLE_OK;
}

int oracle_pe_update_priorities(oracle_pe *r, uint64_t m, const uint64_t *key, const float *prio)
{
  if (!r || (m && (!key || !prio))) return ORACLE_ERR_INVALID_ARG;
  for (uint64_t i = 0; i < m; ++i) {
    const uint64_t slot = key[i] & 0xffffffffu, g = key[i] >> 32;
    if (slot >= r->max_slots || r->gen[slot] != g || r->ts[r->P2 + slot] == 0) { r->n_stale++; continue; }
    pe_set_priority(r, slot, prio[i]);
  }
  return ORACLE_OK;
}

/* rnd: [rounds, e] uniforms, e = size - capacity at the time of the call (row stride e). */
int oracle_pe_evict(oracle_pe *r, uint32_t rounds, const uint64_t *rnd, uint64_t *evicted_out)
{
  if (!r) return ORACLE_ERR_INVALID_ARG;
  const uint64_t size = pe_size(r);
  const uint64_t e = size > r->capacity ? size - r->capacity : 0;
  uint64_t remaining = e;
  if (e && !rnd) return ORACLE_ERR_INVALID_ARG;
  uint64_t *cand = (uint64_t *)malloc(sizeof(uint64_t) * (e ? e : 1));
  if (!cand) return ORACLE_ERR_INVALID_ARG;
  for (uint32_t rd = 0; rd < rounds && remaining > 0; ++rd) {
    const uint64_t k = remaining, total = r->te[1], w = total / k;
    for (uint64_t j = 0; j < k; ++j)
      cand[j] = tree_find(r->te, r->P2, j * w + mulhi64(rnd[(uint64_t)rd * e + j], w));
    for (uint64_t j = 0; j < k; ++j) {
      if (j > 0 && cand[j] == cand[j - 1]) continue;      /* drawn again: counts once */
      tree_set(r->ts, r->P2, cand[j], 0);
      tree_set(r->te, r->P2, cand[j], 0);
      r->free_ring[r->free_tail % r->max_slots] = (uint32_t)cand[j];
      r->free_tail++;
      r->evicted++;
      remaining--;
    }
  }
  free(cand);
  if (evicted_out) *evicted_out = e - remaining;
  return ORACLE_OK;
}

uint64_t oracle_pe_size(const oracle_pe *r) { return pe_size(r); }
uint64_t oracle_pe_root(const oracle_pe *r) { return r->ts[1]; }
uint64_t oracle_pe_root_evict(const oracle_pe *r) { return r->te[1]; }
uint64_t oracle_pe_inserted(const oracle_pe *r) { return r->inserted; }
uint64_t oracle_pe_evicted(const oracle_pe *r) { return r->evicted; }
uint64_t oracle_pe_free_head(const oracle_pe *r) { return r->free_head; }
uint64_t oracle_pe_free_tail(const oracle_pe *r) { return r->free_tail; }
uint64_t oracle_pe_n_stale(const oracle_pe *r) { return r->n_stale; }
uint64_t oracle_pe_n_clamped(const oracle_pe *r) { return r->n_clamped; }
void oracle_pe_leaves(const oracle_pe *r, int which, uint64_t *out)
{
  memcpy(out, (which ? r->te : r->ts) + r->P2, r->max_slots * sizeof(uint64_t));
}
void oracle_pe_nodes(const oracle_pe *r, int which, uint64_t *out)
{
  memcpy(out, which ? r->te : r->ts, 2 * r->P2 * sizeof(uint64_t));
}
uint64_t oracle_pe_tree_leaves(const oracle_pe *r) { return r->P2; }
void oracle_pe_gen(const oracle_pe *r, uint32_t *out) { memcpy(out, r->gen, r->max_slots * 4); }
void oracle_pe_free_ring(const oracle_pe *r, uint32_t *out) { memcpy(out, r->free_ring, r->max_slots * 4); }

/* ------------------------------------------------------------------------- */
/* Lossless codec of stored observations                                       */
/* ------------------------------------------------------------------------- */
/*
 * Section 4.1 (and Appendix "Atari: Additional Details"): observations are kept
 * compressed in the replay memory and decompressed by the learner as it prefetches
 * batches; the paper uses PNG and says no more.  The property that matters to the
 * method is that the codec is lossless.  The reading taken here is a codec that a
 * GPU can undo at memory speed: a row of raw_bytes = 64 * nb bytes is cut into nb
 * blocks of 64 bytes; a block whose 64 bytes are all equal ("flat": the background
 * of a game screen) is stored as that one byte, any other block as it is, and
 * every part of a block has a fixed place, so that nothing has to be looked up
 * before it can be fetched.
 *
 * Encoded row (all offsets and sizes in bytes, integers little-endian):
 *   0           mask: bit (b mod 64) of u64 word (b div 64) is 1 iff block b is not
 *               flat; ceil(nb/64) words, zero-padded to a multiple of 16 (M bytes)
 *   M           one byte per block, in block order: the common byte of block b if it
 *               is flat (else unspecified; the oracle writes 0); nb bytes, zero-padded
 *               to a multiple of 16 (V bytes)
 *   M + V       the image of the row: bytes [64 b, 64 b + 64) hold block b if it is not
 *               flat (else unspecified; the oracle writes 0)
 * A row takes M + V + 64 * nb bytes; that is the stride of the store.  What an encoder
 * has to write and a decoder to read is the mask, the bytes of the flat blocks and
 * the other blocks: M + (flat blocks) + 64 * (other blocks) bytes.
 */
static uint64_t pad16(uint64_t v) { return (v + 15) / 16 * 16; }

uint64_t oracle_codec_row_bytes(uint32_t raw_bytes)
{
  if (raw_bytes == 0 || raw_bytes % 64) return 0;
  const uint64_t nb = raw_bytes / 64;
  return pad16(8 * ((nb + 63) / 64)) + pad16(nb) + 64 * nb;
}

/* enc: oracle_codec_row_bytes(raw_bytes) bytes, all written.  *used: the bytes of it that carry data. */
int oracle_codec_encode_row(const uint8_t *raw, uint32_t raw_bytes, uint8_t *enc, uint64_t *used)
{
  const uint64_t cap = oracle_codec_row_bytes(raw_bytes);
  if (!cap) return ORACLE_ERR_INVALID_ARG;
  const uint64_t nb = raw_bytes / 64;
  const uint64_t M = pad16(8 * ((nb + 63) / 64)), V = pad16(nb);
  memset(enc, 0, cap);
  uint8_t *mask = enc, *flat = enc + M, *image = enc + M + V;
  uint64_t n_kept = 0;
  for (uint64_t b = 0; b < nb; ++b) {
    const uint8_t *blk = raw + 64 * b;
    int is_flat = 1;
    for (int j = 1; j < 64; ++j)
      if (blk[j] != blk[0]) is_flat = 0;
    if (is_flat) {
      flat[b] = blk[0];
    } else {
      mask[b / 8] |= (uint8_t)(1u << (b % 8)); /* little-endian words: bit b of the bit string */
      memcpy(image + 64 * b, blk, 64);
      ++n_kept;
    }
  }
  if (used) *used = M + (nb - n_kept) + 64 * n_kept;
  return ORACLE_OK;
}

int oracle_codec_decode_row(const uint8_t *enc, uint32_t raw_bytes, uint8_t *raw_out)
{
  const uint64_t cap = oracle_codec_row_bytes(raw_bytes);
  if (!cap) return ORACLE_ERR_INVALID_ARG;
  const uint64_t nb = raw_bytes / 64;
  const uint64_t M = pad16(8 * ((nb + 63) / 64)), V = pad16(nb);
  const uint8_t *mask = enc, *flat = enc + M, *image = enc + M + V;
  for (uint64_t b = 0; b < nb; ++b) {
    if (mask[b / 8] >> (b % 8) & 1)
      memcpy(raw_out + 64 * b, image + 64 * b, 64);
    else
      memset(raw_out + 64 * b, flat[b], 64);
  }
  return ORACLE_OK;
}
