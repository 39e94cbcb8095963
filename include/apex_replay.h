/*
 * apex_replay.h -- C ABI of an MI355X-resident replay memory for Ape-X
 * ("Distributed Prioritized Experience Replay").
 *
 * The library keeps the whole replay memory of the paper (Section 3, Figure 1: one shared,
 * centralized, prioritized memory that many actors fill and one learner samples) in the HBM
 * of one GPU and serves the paper's replay verbs as stream-ordered batches of HIP kernels:
 *
 *   apex_nstep_priorities          ComputePriorities of Algorithm 1 (actor side)
 *   apex_replay_add                replay.Add            (Algorithm 1)
 *   apex_replay_sample             replay.Sample         (Algorithm 2)
 *   apex_replay_update_priorities  replay.SetPriority    (Algorithm 2)
 *   apex_replay_evict              replay.RemoveToFit    (Algorithm 2)
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory that the caller allocated and still owns; the
 *     library never frees them and does not use them after the work it enqueued has finished.
 *     "host" pointers are ordinary host memory written before the call returns.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues kernels on that stream and returns; device outputs are valid once the stream has
 *     reached that point.  No call allocates or frees device memory, none synchronises except
 *     apex_replay_create and apex_replay_stats.  Calls on one memory must be issued in order
 *     on one stream (or be ordered by events): the memory holds no locks.  A memory object
 *     (and a pipeline on it) is used by one host thread at a time; different objects are
 *     independent.
 *   - Return value: APEX_OK or a negative apex_status; on error nothing has been enqueued and
 *     no state has changed.
 *   - Transitions are identified by a key: the running count of insertions (the first
 *     transition ever added has key 0).  The transition with key K lives in ring slot
 *     K mod max_slots.  Keys in [head, tail) are valid; eviction advances head.
 *   - Sampling mass.  A priority p is turned into the integer mass
 *         Q(p) = clamp( floor( (|p| + eps)^alpha * 2^frac_bits ), 1, QMAX ),
 *         QMAX = 2^(62 - ceil(log2(max_slots))),
 *     where the power is evaluated by a fixed sequence of IEEE fp32 operations, so that the
 *     same priorities give the same masses, tree sums and sampled indices on any machine.
 *     The probability of drawing a transition is mass / (sum of all masses), the paper's
 *     p^alpha / sum_k p_k^alpha (Appendix "Implementation", paragraph "Sampling Data").
 */
#ifndef APEX_REPLAY_H
#define APEX_REPLAY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum apex_status {
  APEX_OK = 0,
  APEX_ERR_INVALID_ARG = -1, /* null pointer, zero size, value out of its documented range          */
  APEX_ERR_FULL = -2,        /* add: size + count would exceed max_slots                             */
  APEX_ERR_NOT_READY = -3,   /* sample: fewer than min_size_to_sample transitions stored             */
  APEX_ERR_EMPTY = -4,       /* sample: nothing stored                                               */
  APEX_ERR_HIP = -5,         /* a HIP call failed; see apex_last_hip_error()                         */
  APEX_ERR_TOO_LARGE = -6    /* sample: more than APEX_MAX_SAMPLES_PER_CALL samples or
                                APEX_MAX_BATCHES_PER_CALL batches; update: m >= 2^32                 */
} apex_status;

#define APEX_MAX_SAMPLES_PER_CALL 65536u
#define APEX_MAX_BATCHES_PER_CALL 1024u
#define APEX_TREE_MAX_LEVELS 8u
#define APEX_NOALLOC_MAX_SAMPLES 16384u /* num_batches * k of apex_replay_sample_noalloc */

typedef struct apex_replay apex_replay_t; /* opaque host object; created and destroyed by the library */

typedef struct apex_replay_config {
  uint64_t capacity;           /* soft limit on stored transitions; apex_replay_evict trims to it
                                  (Section 4.1: 2,000,000)                                           */
  uint64_t max_slots;          /* physical ring size P, capacity <= P <= 2^31; slot = key mod P      */
  uint32_t obs_bytes;          /* opaque observation payload per transition (e.g. 84*84*4 = 28224)   */
  uint32_t act_bytes;          /* opaque action payload per transition (e.g. 4)                      */
  float alpha;                 /* priority exponent, in [-1, 1] (Section 4.1: 0.6)                   */
  float eps;                   /* added to |p| before the power, >= 0                                */
  uint32_t frac_bits;          /* F: fraction bits of the integer mass, <= 32 (24 recommended)       */
  uint32_t reserved;           /* must be 0                                                          */
  uint64_t min_size_to_sample; /* sample refuses below this size (Appendix "Atari: Additional
                                  Details": the learner waits for 50,000 transitions); 0 disables    */
} apex_replay_config_t;

typedef struct apex_replay_stats {
  uint64_t size, head, tail; /* stored transitions and the valid key range [head, tail)            */
  uint64_t root;             /* sum of all masses                                                   */
  uint64_t n_stale_dropped;  /* priority updates skipped because their key was no longer valid      */
  uint64_t n_clamped;        /* priorities whose mass had to be clamped to 1 or QMAX                */
} apex_replay_stats_t;

/* Where things live inside the caller's device regions (for inspection and tests). */
typedef struct apex_replay_layout {
  uint64_t obs_offset, act_offset, ret_offset, gacc_offset; /* byte offsets in d_storage; row strides
                                                               are obs_bytes, act_bytes, 4, 4       */
  uint32_t tree_levels;                                     /* level 0 = one uint64 mass per slot   */
  uint32_t tree_fanout;                                     /* node i of level l+1 = sum of nodes
                                                               [64 i, 64 i + 64) of level l         */
  uint64_t level_offset[APEX_TREE_MAX_LEVELS];              /* in uint64 units inside d_tree        */
  uint64_t level_size[APEX_TREE_MAX_LEVELS];                /* nodes in use (arrays are zero padded
                                                               to a multiple of 64)                 */
} apex_replay_layout_t;

/*
 * Sizes of the three device regions apex_replay_create adopts: the payload ring, the sum
 * tree (two copies: the second serves the pipeline's fused learner steps), and scratch
 * (device-side counters, per-call temporaries).  Any out pointer may be NULL.
 */
int apex_replay_workspace_bytes(const apex_replay_config_t *cfg, size_t *storage_bytes, size_t *tree_bytes,
                                size_t *scratch_bytes);

/*
 * Builds an empty replay memory inside three caller-allocated device regions of at least the
 * sizes reported above, each 256-byte aligned.  Zero-fills the tree and the scratch region and
 * synchronises the device once.  The regions must stay allocated until apex_replay_destroy,
 * which frees only the host object.
 */
int apex_replay_create(const apex_replay_config_t *cfg, void *d_storage, void *d_tree, void *d_scratch,
                       apex_replay_t **out);
int apex_replay_destroy(apex_replay_t *r);
int apex_replay_layout(const apex_replay_t *r, apex_replay_layout_t *out /*host*/);

/*
 * Actor-side priorities (Algorithm 1, ComputePriorities; Appendix "Implementation", "Adding
 * Data"): absolute n-step TD errors of S streams x T transitions, from Q-values the actors
 * already hold.  Stateless.
 *
 * All arrays are device, row-major.  Each stream carries T+n rows; row u holds what was known
 * when acting in state S_u: q_online[s,u,0..A), q_target[s,u,0..A), action[s,u] in [0,A),
 * reward[s,u] = the reward that followed (R_{u+1}), discount[s,u] = the discount that followed
 * (gamma, or 0 if the episode ended on that step).  For t in [0,T):
 *     ret   = sum_{j<n} (prod_{i<j} discount[t+i]) * reward[t+j]
 *     gacc  = prod_{j<n} discount[t+j]
 *     boot  = q_target[t+n, argmax_a q_online[t+n, a]]              (ties: lowest a)
 *     prio  = | ret + gacc * boot - q_online[t, action[t]] |
 * which is the multi-step double-Q target of Section 3.1; a zero discount truncates the return
 * at the end of an episode.  With A = 1 (q_* holding critic values) it is the target of
 * Section 3.2.  An actor with a single network passes the same pointer for q_online and
 * q_target.  Outputs prio, ret, gacc are [S,T] fp32; prio_fx (may be NULL) receives the integer
 * mass Q(prio) for a memory of max_slots slots (max_slots = 0: QMAX = 2^62).
 * fp32 arithmetic in a fixed order: ret by Horner's rule with one fused multiply-add per step,
 * gacc left to right, the target as one fused multiply-add.
 */
int apex_nstep_priorities(uint32_t S, uint32_t T, uint32_t n, uint32_t A, const float *q_online,
                          const float *q_target, const int32_t *action, const float *reward,
                          const float *discount, float alpha, float eps, uint32_t frac_bits,
                          uint64_t max_slots, float *prio, float *ret, float *gacc, uint64_t *prio_fx,
                          void *hip_stream);

/*
 * replay.Add (Algorithm 1; Appendix "Implementation", "Adding Data"): stores count transitions
 * under the next count keys and enters them into the sampling distribution with the priorities
 * the actors computed.  obs [count,obs_bytes], act [count,act_bytes], ret, gacc, prio [count]
 * are device arrays; obs, act, ret, gacc may each be NULL (that part of the payload is then
 * left as it is).  *first_key_out (host, may be NULL) receives the key of the first one.
 * Data beyond the soft capacity is accepted (Section 4.1: adding is always permitted); only a
 * full ring refuses, with APEX_ERR_FULL.
 */
int apex_replay_add(apex_replay_t *r, uint64_t count, const void *obs, const void *act, const float *ret,
                    const float *gacc, const float *prio, uint64_t *first_key_out, void *hip_stream);

/*
 * The two halves of apex_replay_add, for callers that overlap the large payload copy with other
 * work (Appendix "Implementation": the key-value store of transitions and the prioritized
 * distribution over its keys are separate structures; the distribution is updated once the batch
 * is in the store).  apex_replay_add_payload writes the rows of the next count keys into the ring
 * and publishes nothing; apex_replay_add_publish enters the same count keys into the sum tree and
 * advances tail.  The publish must be ordered after its payload (same stream, or an event), and
 * one payload/publish pair must complete before the next payload call is issued.
 *
 * Adding without a copy: a producer (a DMA from the host, a kernel of the caller's) may write a
 * column of the coming keys into the ring itself and pass NULL for it.  Key tail + i lives in
 * row (tail + i) mod max_slots of every column (apex_replay_layout gives the columns' offsets in
 * d_storage; tail is first_key_out + count of the last add, or apex_replay_stats).  No call
 * reads or writes the rows of keys that are not published yet.
 */
int apex_replay_add_payload(apex_replay_t *r, uint64_t count, const void *obs, const void *act, const float *ret,
                            const float *gacc, void *hip_stream);
int apex_replay_add_publish(apex_replay_t *r, uint64_t count, const float *prio, uint64_t *first_key_out,
                            void *hip_stream);

/*
 * replay.Sample (Algorithm 2; Appendix "Implementation", "Sampling Data"): num_batches
 * independent batches of k transitions, all drawn from the state of the memory at this point
 * of the stream (Section 4.1: the learner prefetches up to 16 batches of 512).
 *
 * Batch b, sample j: with total = sum of all masses and w = floor(total / k), the point
 *     x = j*w + floor(rnd[b,j] * w / 2^64)
 * lies in the j-th of k equal strata of [0,total); the transition drawn is the one whose
 * interval of the cumulative mass, taken in slot order, contains x.  rnd is a device array
 * [num_batches,k] of uniform 64-bit integers supplied by the caller.
 * weight_out[b,j] = (N * P(i))^-beta / max over the batch, N = size, P(i) = mass_i / total:
 * importance-sampling weights normalised by the largest weight of the same batch of k; beta in
 * [0, 1] (Section 4.1: 0.4), fp32, relative error below 1e-6.
 * Device outputs, each may be NULL except slot_out: key_out [nb,k] u64, slot_out [nb,k] u32,
 * weight_out [nb,k] f32, obs_out [nb,k,obs_bytes], act_out [nb,k,act_bytes], ret_out, gacc_out
 * [nb,k] f32 (copies of what apex_replay_add stored).
 */
int apex_replay_sample(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                       uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                       float *ret_out, float *gacc_out, void *hip_stream);

/*
 * apex_replay_sample for callers that cannot allocate device memory and do not want the call to touch
 * the memory's scratch region: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same results, same status codes as apex_replay_sample, with two
 * differences:
 *   - the per-call temporary (the mass of every drawn transition, which the draw writes and the
 *     importance weights read) lives in an array that is part of the library's code object:
 *     APEX_NOALLOC_MAX_SAMPLES * 8 bytes = 128 KB on every GPU the library runs on, held until the
 *     process ends.  Its device address is looked up once per GPU (by apex_replay_create on the GPU
 *     that is current then; else by the first call).  The call allocates nothing and frees nothing;
 *   - num_batches * k > APEX_NOALLOC_MAX_SAMPLES is refused with APEX_ERR_TOO_LARGE, nothing enqueued.
 * The GPU that holds the memory must be current in the calling thread (as for every call).  All calls
 * on one GPU share that GPU's array, whatever memory object or stream they name: two calls whose work
 * overlaps in time on one GPU race on it (order them on one stream or by an event); a later call simply
 * overwrites what an earlier one left, nothing has to start at zero.
 */
int apex_replay_sample_noalloc(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                               uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out,
                               void *act_out, float *ret_out, float *gacc_out, void *hip_stream);

/*
 * The two halves of apex_replay_sample, for callers that run the large copy on another stream
 * than the tree work (Section 4.1: the learner fetches batches asynchronously, ahead of use).
 * apex_replay_sample_begin does everything that reads the sum tree: it draws the samples and
 * writes key_out, slot_out, the small payload columns, and mass_out [nb,k] u64 (device,
 * required): the mass of every drawn transition.  It must be ordered with updates, adds and
 * evictions like apex_replay_sample.  apex_replay_sample_finish reads only slot and mass (device,
 * as written by begin) and the payload ring: it writes weight_out (may be NULL; needs mass) and
 * obs_out (may be NULL).  It may run on any stream once begin has completed, but before an add
 * re-uses the drawn slots.
 */
int apex_replay_sample_begin(apex_replay_t *r, uint32_t num_batches, uint32_t k, const uint64_t *rnd,
                             uint64_t *key_out, uint32_t *slot_out, uint64_t *mass_out, void *act_out, float *ret_out,
                             float *gacc_out, void *hip_stream);
int apex_replay_sample_finish(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint32_t *slot,
                              const uint64_t *mass, float *weight_out, void *obs_out, void *hip_stream);
/*
 * apex_replay_sample_finish followed by apex_replay_update_priorities(m, key, prio), as one call:
 * the two touch disjoint data (payload ring and caller buffers; sum tree), and for m <= 1024 and
 * long observation rows the update rides in one extra workgroup of the gather kernel instead of
 * a launch of its own.  key may be the key_out of the batch being finished, or an older one.
 */
int apex_replay_sample_finish_update(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta,
                                     const uint32_t *slot, const uint64_t *mass, float *weight_out, void *obs_out,
                                     uint64_t m, const uint64_t *key, const float *prio, void *hip_stream);
/*
 * apex_replay_sample_finish, and the new priorities of the very batch being finished written back
 * in the same launch: prio[i] (device, [nb*k]) becomes the priority of key[i], the transition
 * drawn as sample i (key, slot, mass as written by the matching apex_replay_sample_begin).
 * Allowed only if nothing has touched the sum tree since that apex_replay_sample_begin (no update,
 * add or eviction in between): the write-back then takes slot and mass as known, skipping the
 * loads key -> slot -> mass.  Result: that of apex_replay_sample_finish followed by
 * apex_replay_update_priorities(nb*k, key, prio).
 */
int apex_replay_sample_finish_writeback(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta,
                                        const uint64_t *key, const uint32_t *slot, const uint64_t *mass,
                                        float *weight_out, void *obs_out, const float *prio, void *hip_stream);

/*
 * The read half of replay.Sample on its own (Appendix "Implementation", "Data Storage": reading
 * batches of stored tensors): copies the payload of count ring slots, slot[i] < max_slots (device,
 * u32, e.g. the slot_out of an earlier apex_replay_sample), into obs_out [count,obs_bytes],
 * act_out [count,act_bytes], ret_out, gacc_out [count]; each output may be NULL.  Lets a caller put
 * the large copy on another stream than the tree work.  count <= APEX_MAX_SAMPLES_PER_CALL.
 */
int apex_replay_gather(apex_replay_t *r, uint64_t count, const uint32_t *slot, void *obs_out, void *act_out,
                       float *ret_out, float *gacc_out, void *hip_stream);

/*
 * replay.SetPriority (Algorithm 2): mass of key[i] becomes Q(prio[i]) for i in [0,m); key and
 * prio are device arrays.  The result is that of applying the pairs one after the other: of
 * several pairs naming one key the last stands; a pair whose key is not valid any more is
 * skipped and counted.
 */
int apex_replay_update_priorities(apex_replay_t *r, uint64_t m, const uint64_t *key, const float *prio,
                                  void *hip_stream);

/*
 * ComputePriorities and replay.SetPriority of Algorithm 2 as one call: the learner hands over the
 * Q-values it has just evaluated for a sampled batch and the library recomputes the priorities
 * from the partial return and accumulated discount it stores with every transition (Appendix
 * "Implementation", "Adding Data"): for i in [0,m), with ret and gacc those of key[i],
 *     prio = | ret + gacc * q_target_next[i, argmax_a q_online_next[i,a]] - q_taken[i] |
 * (the target of Section 3.1; A = 1 with critic values gives that of Section 3.2), fp32 in the same
 * order as apex_nstep_priorities, then exactly as apex_replay_update_priorities(m, key, prio).
 * Device arrays: key [m] u64, q_taken [m], q_online_next and q_target_next [m,A] fp32; prio_out
 * [m] (may be NULL) receives the priorities (0 for pairs skipped because their key is not valid).
 */
int apex_replay_update_from_q(apex_replay_t *r, uint64_t m, const uint64_t *key, uint32_t A, const float *q_taken,
                              const float *q_online_next, const float *q_target_next, float *prio_out,
                              void *hip_stream);

/*
 * replay.RemoveToFit (Algorithm 2; Section 4.1: excess above the soft capacity is removed en
 * masse, oldest first): removes the size - capacity oldest keys, if any.  *evicted_out (host,
 * may be NULL) receives their number.
 */
int apex_replay_evict(apex_replay_t *r, uint64_t *evicted_out, void *hip_stream);

/*
 * head and tail live in device memory and the kernels read them there, so launches captured in a
 * HIP graph stay correct when replayed.  The host keeps a mirror for its own checks (ring full,
 * eviction count, first_key_out), which replays do not advance: after replaying captured
 * launches, call this before the next direct call.  Synchronises hip_stream.
 */
int apex_replay_resync(apex_replay_t *r, void *hip_stream);

/* Synchronises hip_stream and reads the counters back. */
int apex_replay_stats(apex_replay_t *r, apex_replay_stats_t *out /*host*/, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Observations stored compressed (Section 4.1 and Appendix "Atari: Additional Details": the
 * replay memory keeps observations compressed, the learner decompresses them as it fetches
 * batches; the paper uses PNG).  Here: a lossless codec that is undone at memory speed.  A row
 * of raw_bytes = 64 * nb bytes is cut into nb blocks of 64 bytes; a block whose bytes are all
 * equal (flat background) is kept as that byte, any other block as it is, and every part has a
 * fixed place, so that nothing has to be looked up before it can be fetched.  Encoded row,
 * integers little-endian:
 *   0        mask, bit b set iff block b is kept as it is: ceil(nb/64) u64 words, zero-padded to a
 *            multiple of 16 bytes (M bytes in all)
 *   M        one byte per block: the byte of block b if it is not kept as it is (else unspecified);
 *            nb bytes, rounded up to a multiple of 16 (V bytes)
 *   M + V    the image of the row: bytes [64 b, 64 b + 64) hold block b if it is kept as it is (else
 *            unspecified)
 * apex_codec_row_bytes = M + V + 64 * nb is what a row takes; a memory that stores encoded rows
 * is created with obs_bytes >= that (a multiple of 16).  0 if raw_bytes is 0 or no multiple of 64.
 * The ring's row stride stays fixed, so the codec saves HBM traffic (an add writes, a fetch reads
 * only the parts that carry data), not capacity.
 *
 * apex_replay_add_payload_encoded is apex_replay_add_payload with raw_obs [count, raw_bytes]
 * (device, 16-byte aligned) encoded on its way into the ring; publish with
 * apex_replay_add_publish.  apex_replay_gather_decoded is apex_replay_gather with obs_out
 * [count, raw_bytes] (16-byte aligned, may be NULL) decoded on its way out.  Both:
 * APEX_ERR_INVALID_ARG for a raw_bytes the codec refuses or misaligned rows, APEX_ERR_TOO_LARGE
 * if the memory's rows are too short for raw_bytes.  With the plain calls a caller of the
 * codec draws with apex_replay_sample_begin and apex_replay_sample_finish (obs_out NULL) and
 * fetches with apex_replay_gather_decoded; the pipeline does both itself after
 * apex_pipeline_set_codec.
 * ---------------------------------------------------------------------------------------- */
size_t apex_codec_row_bytes(uint32_t raw_bytes);
int apex_replay_add_payload_encoded(apex_replay_t *r, uint64_t count, const void *raw_obs, uint32_t raw_bytes,
                                    const void *act, const float *ret, const float *gacc, void *hip_stream);
int apex_replay_gather_decoded(apex_replay_t *r, uint64_t count, const uint32_t *slot, uint32_t raw_bytes,
                               void *obs_out, void *act_out, float *ret_out, float *gacc_out, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Prefetch pipeline.  Section 4.1 and Appendix "Implementation" describe a learner that fetches
 * batches asynchronously, ahead of use, while priorities flow back and actors keep adding.  An
 * apex_pipeline_t issues the same verbs as above on two streams of its own (default priority),
 * ordered by events: learner steps and every other tree operation in program order on one (the
 * tree stream), the payload copies of large add rounds (with their n-step priorities) beside
 * them on the other (the copy stream).  A sequence of steps of one batch each is issued as one
 * launch per step (gather, weights and priority write-back of a batch together with the draw of
 * the next one; it uses the second copy of the sum tree held in the tree region); steps of
 * several batches put their gathers on the copy stream and on a third stream in turn, so that
 * one large gather follows the other without a gap; the payload of an add round is written
 * after the gathers of all batches drawn before it (it may land in slots that an eviction has
 * freed since).  Results are in every case those of the plain calls issued in the order: draw
 * batch, update, [publish add], [evict].
 * ---------------------------------------------------------------------------------------- */
typedef struct apex_pipeline apex_pipeline_t;

/* Device output buffers of one sample call of num_batches x k transitions ("a set"). */
typedef struct apex_batch_buffers {
  uint64_t *key;  /* [nb*k]            */
  uint32_t *slot; /* [nb*k]            */
  uint64_t *mass; /* [nb*k]            */
  float *weight;  /* [nb*k]            */
  void *obs;      /* [nb*k, obs_bytes] */
  void *act;      /* [nb*k, act_bytes] */
  float *ret;     /* [nb*k]            */
  float *gacc;    /* [nb*k]            */
} apex_batch_buffers_t;

/*
 * sets: host array of `depth` (1..64) buffer sets, all pointers non-NULL device memory owned by
 * the caller; step i fills set i mod depth.  The caller must have consumed a set before depth
 * further steps are issued.  Creates two streams (three for steps of several batches) and a few
 * events.
 */
int apex_pipeline_create(apex_replay_t *r, uint32_t depth, const apex_batch_buffers_t *sets, uint32_t num_batches,
                         uint32_t k, apex_pipeline_t **out);
/* Waits for the pipeline's streams, then destroys them. */
int apex_pipeline_destroy(apex_pipeline_t *p);
/* Everything enqueued so far on `after` (hipStream_t; NULL = the default stream) will precede
 * whatever the pipeline is given next. */
int apex_pipeline_fork(apex_pipeline_t *p, void *after);
/* `stream` (NULL = the default stream) waits, on the device, for everything the pipeline was given. */
int apex_pipeline_join(apex_pipeline_t *p, void *stream);

/*
 * n learner steps.  Step i draws num_batches x k transitions with the uniforms rnd[i] (device,
 * [n, nb*k]) into the next buffer set, gathers them, and, if new_prio is not NULL, writes
 * new_prio[i] (device, [n, nb*k]) back as the priorities of the keys just drawn, before the next
 * step draws.  *first_set_out (host, may be NULL) receives the index of the set
 * the first of these steps fills.  With the one-launch-per-step form the payload columns of a
 * set are complete when the launch after its draw has run, i.e. once the call's work is done.
 * Returns what apex_replay_sample returns for the same memory: APEX_ERR_NOT_READY below
 * min_size_to_sample, APEX_ERR_EMPTY if nothing is stored (decided from the host's mirror of head and
 * tail; none of the n steps has been enqueued then), APEX_ERR_INVALID_ARG for a NULL rnd or a beta
 * outside [0, 1].
 */
int apex_pipeline_steps(apex_pipeline_t *p, uint32_t n, float beta, const uint64_t *rnd, const float *new_prio,
                        uint32_t *first_set_out);

/*
 * An add round in two halves, so that its payload copy runs beside learner steps:
 * apex_pipeline_add_begin computes the n-step priorities of S x T transitions (arguments as for
 * apex_nstep_priorities; prio, ret, gacc are device scratch of S*T floats that must stay
 * untouched until the matching add_end has run) and copies obs, act, ret, gacc into the ring on
 * the add stream; apex_pipeline_add_end publishes them on the tree stream (after whatever steps
 * were issued in between) and, if evict is non-zero, then trims the memory to its capacity.
 * One round at a time.  Small rounds take shortcuts with the same result: below 4 MB of
 * observations the copies run on the tree stream (no events), and with rows of at most 1 KB the
 * whole round (priorities, payload, masses) is a single launch issued by add_end, which is why
 * every input of add_begin must stay untouched until add_end has run.  While a round is
 * open, apex_pipeline_steps holds the last launch of its call back until the next call on the
 * pipeline: add_end issues it with the round (a small one) or the round's masses (any other) in
 * further workgroups of the same launch (what a round adds to the tree commutes with that
 * step's write-back; the step draws nothing), every
 * other call (steps, join, fork, add_begin, capture_end, replay, destroy) issues it as it is.
 * A caller therefore orders its own stream after the pipeline with apex_pipeline_join, never
 * by waiting on the pipeline's streams themselves.
 */
int apex_pipeline_add_begin(apex_pipeline_t *p, uint32_t S, uint32_t T, uint32_t n, uint32_t A, const float *q_online,
                            const float *q_target, const int32_t *action, const float *reward,
                            const float *discount, const void *obs, const void *act, float *prio, float *ret,
                            float *gacc);
int apex_pipeline_add_end(apex_pipeline_t *p, int evict, uint64_t *first_key_out, uint64_t *evicted_out);

/*
 * Observations through the block codec (see apex_codec_row_bytes) on the pipeline's fast path: from
 * this call on the obs argument of apex_pipeline_add_begin is [S*T, raw_bytes] and is encoded on its
 * way into the ring, and the obs buffers of the sets are [k, raw_bytes] and receive decoded rows (the
 * step launch decodes as it copies; steps of several batches fetch theirs through the decoder on the
 * copy stream).  raw_bytes == 0 switches back.  Only for pipelines whose steps are single launches (one
 * batch per step, at least three sets) or go to the copy stream (many batches per step):
 * APEX_ERR_INVALID_ARG otherwise, APEX_ERR_TOO_LARGE if the memory's rows are too short.  Not while a
 * round is open or a capture is running.
 */
int apex_pipeline_set_codec(apex_pipeline_t *p, uint32_t raw_bytes);

/*
 * The same sequence as a HIP graph.  Between apex_pipeline_capture_begin and
 * apex_pipeline_capture_end the steps / add_begin / add_end calls are recorded instead of run
 * (stream capture across the pipeline's streams; fork and join are not allowed inside);
 * apex_pipeline_replay then launches the recorded sequence `times` times on the tree stream.
 * Because head and tail are read on the device, each replay continues where the last stopped;
 * the buffers, uniforms and priorities are those named at capture time.  The host mirror is
 * left as if the sequence had run once: replay at least once and call apex_replay_resync before
 * the next direct call.  capture_begin waits for the pipeline's streams to drain.  The counts
 * the recorded calls took from the host (eviction size) are frozen, so the sequence must leave
 * the memory at the size it found it.
 */
int apex_pipeline_capture_begin(apex_pipeline_t *p);
int apex_pipeline_capture_end(apex_pipeline_t *p);
int apex_pipeline_replay(apex_pipeline_t *p, uint32_t times);

/* ------------------------------------------------------------------------------------------
 * Replay memory with prioritized eviction (Appendix "Continuous Control: Additional Details": to
 * hold the capacity, transitions are periodically evicted by proportional prioritized sampling
 * with exponent alpha_evict = -0.4, instead of oldest first).  A separate object with the same
 * verbs.  What differs from apex_replay_t:
 *   - a second sum tree holds the eviction masses Q(p; alpha_evict) of the same transitions;
 *   - slots freed by an eviction are re-used by later adds in the order in which they were freed,
 *     so a key is (generation of the slot << 32) | slot, the generation counting the slot's
 *     tenants; a key is valid while its generation is the slot's and the slot is occupied.  Keys
 *     are handed out by apex_pe_sample only;
 *   - apex_pe_evict removes e = size - capacity transitions without replacement in rounds: each
 *     round draws as many stratified points as are still to go on the eviction tree as it stands
 *     (point j of k: j*w + floor(rnd*w / 2^64), w = floor(total / k)), counts a transition drawn
 *     more than once once, and removes the distinct ones in the order of their points.  rnd is a
 *     device array [rounds, e] of 64-bit uniforms (row stride e).  The call synchronises
 *     hip_stream and reports how many were removed (fewer than e only if `rounds` ran out).
 * Everything else (device pointers, streams, status codes, sampling rule, weights) is as above.
 * ---------------------------------------------------------------------------------------- */
#define APEX_PE_MAX_EVICT_PER_CALL 1048576u

typedef struct apex_pe_replay apex_pe_replay_t;

typedef struct apex_pe_config {
  uint64_t capacity;  /* apex_pe_evict trims to it (Appendix: 1,000,000)                          */
  uint64_t max_slots; /* physical slots P, capacity <= P <= 2^31                                  */
  uint32_t obs_bytes, act_bytes;
  float alpha;        /* sampling exponent, in [-1, 1] (Appendix: 0.6)                            */
  float alpha_evict;  /* eviction exponent, in [-1, 1] (Appendix: -0.4)                           */
  float eps;
  uint32_t frac_bits;
} apex_pe_config_t;

typedef struct apex_pe_stats {
  uint64_t size, inserted, evicted;
  uint64_t root, root_evict; /* sums of the sampling masses and of the eviction masses            */
  uint64_t free_head, free_tail;
  uint64_t n_stale_dropped, n_clamped;
} apex_pe_stats_t;

typedef struct apex_pe_layout {
  uint64_t obs_offset, act_offset, ret_offset, gacc_offset; /* in d_storage, as apex_replay_layout_t */
  uint32_t tree_levels, tree_fanout;
  uint64_t level_offset[APEX_TREE_MAX_LEVELS]; /* sampling tree, uint64 units inside d_tree        */
  uint64_t level_size[APEX_TREE_MAX_LEVELS];
  uint64_t evict_tree_offset;                  /* the eviction tree: same offsets, shifted by this  */
  uint64_t gen_offset, free_ring_offset;       /* byte offsets in d_scratch: u32 [P] each           */
} apex_pe_layout_t;

int apex_pe_workspace_bytes(const apex_pe_config_t *cfg, size_t *storage_bytes, size_t *tree_bytes,
                            size_t *scratch_bytes);
int apex_pe_create(const apex_pe_config_t *cfg, void *d_storage, void *d_tree, void *d_scratch,
                   apex_pe_replay_t **out);
int apex_pe_destroy(apex_pe_replay_t *r);
int apex_pe_layout(const apex_pe_replay_t *r, apex_pe_layout_t *out /*host*/);
int apex_pe_add(apex_pe_replay_t *r, uint64_t count, const void *obs, const void *act, const float *ret,
                const float *gacc, const float *prio, void *hip_stream);
int apex_pe_sample(apex_pe_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                   uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                   float *ret_out, float *gacc_out, void *hip_stream);
int apex_pe_update_priorities(apex_pe_replay_t *r, uint64_t m, const uint64_t *key, const float *prio,
                              void *hip_stream);
int apex_pe_evict(apex_pe_replay_t *r, uint32_t rounds, const uint64_t *rnd, uint64_t *evicted_out /*host*/,
                  void *hip_stream);
/*
 * apex_pe_evict without the host in the loop: enqueues the same rounds for e = size - capacity transitions and
 * returns; *requested_out (host, may be NULL) receives e.  rnd is [rounds, e] as above.  The host's own count of
 * stored transitions (which decides APEX_ERR_FULL, APEX_ERR_EMPTY and the next e) takes all e to be gone; behind
 * the rounds the call copies the device's counters into host memory of the library's, and the next calls look at
 * that copy once it has arrived: if the rounds ran out before e distinct transitions were found, the host's
 * count is corrected then (and the next eviction asks for the rest).  An add that would only fit if the
 * unconfirmed eviction was complete waits for the copy first, so a slot is never handed out twice; so does the
 * next apex_pe_evict_enqueue if the copy of the one before it has still not arrived (there is one such copy at a
 * time).  No device memory is allocated.  Not for HIP graph capture (the copy and its event would be recorded
 * once).
 */
int apex_pe_evict_enqueue(apex_pe_replay_t *r, uint32_t rounds, const uint64_t *rnd, uint64_t *requested_out /*host*/,
                          void *hip_stream);
/*
 * An actor round in one launch (Algorithm 1: ComputePriorities, then replay.Add): the n-step priorities of S x T
 * transitions (arguments and arithmetic as apex_nstep_priorities) and their insertion with obs [S*T, obs_bytes]
 * and act [S*T, act_bytes] (device; act may be NULL), partial return and accumulated discount as computed.
 * Result: that of apex_nstep_priorities followed by apex_pe_add.  Only for observation rows of at most 256
 * vectors (4 KB when rows and pointers are 16-byte aligned): APEX_ERR_TOO_LARGE otherwise.
 */
int apex_pe_add_round(apex_pe_replay_t *r, uint32_t S, uint32_t T, uint32_t n, uint32_t A, const float *q_online,
                      const float *q_target, const int32_t *action, const float *reward, const float *discount,
                      const void *obs, const void *act, void *hip_stream);
/*
 * A learner step in two launches (Algorithm 2: replay.Sample, replay.SetPriority): apex_pe_sample of one batch
 * of k <= 1024 with the uniforms rnd [k], then apex_pe_update_priorities(k, key_out, new_prio) with new_prio [k]
 * (device) - the gather, the weights and the write-back share the second launch.  key_out and slot_out are
 * required, the other outputs may be NULL.  Same row limit as apex_pe_add_round when obs_out is given.
 */
int apex_pe_sample_update(apex_pe_replay_t *r, uint32_t k, float beta, const uint64_t *rnd, const float *new_prio,
                          uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                          float *ret_out, float *gacc_out, void *hip_stream);
int apex_pe_stats(apex_pe_replay_t *r, apex_pe_stats_t *out /*host*/, void *hip_stream);

/* hipError_t of the last failed HIP call of the calling thread (0 if none). */
int apex_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* APEX_REPLAY_H */
