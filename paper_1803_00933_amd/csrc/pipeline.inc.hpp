// apex_pipeline_*: the replay verbs issued on two internal streams ordered by events (learner
// steps on one, the payload copies of add rounds on the other), and the same sequence captured
// once as a HIP graph and replayed.
// A step that draws several batches at once (the learner's prefetch, Section 4.1) is long enough
// to pay for two more events: its gather then runs on the copy stream, beside the write-back of
// its priorities and the next draw, which are all that the next step has to wait for.
// While an add round is open the last launch of a steps call is held back (HeldStep): add_end issues
// it with the round's tree work in further workgroups; every other entry point issues it first.
// Included by apex_replay.hip (one translation unit), after the plain entry points.

struct apex_pipeline {
  apex_replay *r;
  uint32_t depth, nb, k;
  std::vector<apex_batch_buffers_t> sets;
  hipStream_t tree, add;  // learner steps and every tree operation; add payloads
  // wide steps only: their gathers alternate between `add` and this stream, so that the next gather starts when
  // its draw is done, not when the one before it has been retired (no idle gap between two large copies)
  hipStream_t add2 = nullptr;

  // A "mark" is the latest record of one role (payload copied, tail advanced).  Outside a capture each
  // role re-records its own long-lived event; inside a capture every record gets a fresh event, so that
  // no event is recorded twice in one capture.
  struct Mark {
    hipEvent_t own = nullptr;  // long-lived
    hipEvent_t cur = nullptr;  // what a wait has to wait for; null: nothing to wait for
  };
  Mark payload_done, tail_ready;
  // wide steps only: the draw of a step (the copy stream's gather waits for it), and per buffer
  // set the gather that last read it (the next draw into that set waits for it)
  bool wide = false;
  Mark drawn;
  std::vector<Mark> gathered;
  // the latest gather on each of the two copy streams: an add round's payload may overwrite slots that an
  // eviction has just freed, so it waits for the gathers of batches drawn before that eviction
  hipEvent_t last_gather[2] = {nullptr, nullptr};
  hipEvent_t fork_ev = nullptr, join_ev = nullptr;
  std::vector<hipEvent_t> capture_events;

  uint64_t step = 0;          // learner steps issued so far
  uint64_t first_step = 0;    // steps before this one cannot be in flight (pipeline was drained)
  bool add_open = false;      // add_begin issued, add_end not yet
  bool add_on_tree = false;   // ... with its payload copy on the learner's stream (small rounds)
  bool tail_unmarked = false; // the tail has moved since tail_ready was last recorded
  bool add_deferred = false;  // the open round is issued as one launch by add_end
  HeldStep held;              // the last step launch of the latest steps call, if it waits for that launch
  uint32_t codec_raw_bytes = 0;  // != 0: observations pass through the block codec (apex_pipeline_set_codec)
  NstepArgs add_ns{};
  const void *add_obs = nullptr, *add_act = nullptr;
  uint64_t add_count = 0;
  float *add_prio = nullptr;

  bool capturing = false;
  hipGraph_t graph = nullptr;
  hipGraphExec_t graph_exec = nullptr;

  static constexpr int kStreams = 3;
  hipStream_t streams(int i) const { return i == 0 ? tree : i == 1 ? add : add2; }  // add2 may be null
};

namespace {

// Add rounds whose observations are smaller than this are issued on the learner's stream: the events that
// order the two streams would cost more than the copy.
constexpr uint64_t kSmallPayloadBytes = 4u << 20;

// From this many samples per step on, a step's gather goes to the copy stream.
constexpr uint64_t kWideStepSamples = 2048;
constexpr uint64_t kWideStepBytes = 8u << 20;  // ... and only if the gather moves enough to be worth two events

bool new_event(hipEvent_t *e) { return !hip_failed(hipEventCreateWithFlags(e, hipEventDisableTiming)); }

// Events that only order the pipeline's two streams on this device: no system-scope fence when
// they are recorded (the host and other devices never wait on them).
bool new_mark_event(hipEvent_t *e)
{
  return !hip_failed(hipEventCreateWithFlags(e, hipEventDisableTiming | hipEventDisableSystemFence));
}

int mark_record(apex_pipeline *p, apex_pipeline::Mark &m, hipStream_t s)
{
  hipEvent_t e = m.own;
  if (p->capturing) {
    if (!new_mark_event(&e)) return APEX_ERR_HIP;
    p->capture_events.push_back(e);
  }
  APEX_HIP(hipEventRecord(e, s));
  m.cur = e;
  return APEX_OK;
}

int mark_wait(apex_pipeline::Mark &m, hipStream_t s)
{
  if (m.cur) APEX_HIP(hipStreamWaitEvent(s, m.cur, 0));
  return APEX_OK;
}

void forget_marks(apex_pipeline *p)
{
  p->payload_done.cur = p->tail_ready.cur = p->drawn.cur = nullptr;
  for (apex_pipeline::Mark &m : p->gathered) m.cur = nullptr;
  p->last_gather[0] = p->last_gather[1] = nullptr;
  p->first_step = p->step;
}

// Stream s waits for the gathers of wide steps that are in flight on the other streams: what s is about to
// write into the ring (an add round's payload) may land in slots that an eviction has freed since those
// batches were drawn.
int wait_for_gathers(apex_pipeline *p, hipStream_t s)
{
  for (int i = 0; i < 2; ++i)
    if (p->last_gather[i] && p->streams(1 + i) != s) APEX_HIP(hipStreamWaitEvent(s, p->last_gather[i], 0));
  return APEX_OK;
}

void drop_graph(apex_pipeline *p)
{
  if (p->graph_exec) (void)hipGraphExecDestroy(p->graph_exec);
  if (p->graph) (void)hipGraphDestroy(p->graph);
  p->graph_exec = nullptr;
  p->graph = nullptr;
  for (hipEvent_t e : p->capture_events) (void)hipEventDestroy(e);
  p->capture_events.clear();
}

void pipeline_free(apex_pipeline *p)
{
  drop_graph(p);
  for (hipEvent_t e : {p->payload_done.own, p->tail_ready.own, p->drawn.own, p->fork_ev, p->join_ev})
    if (e) (void)hipEventDestroy(e);
  for (apex_pipeline::Mark &m : p->gathered)
    if (m.own) (void)hipEventDestroy(m.own);
  for (int i = 0; i < apex_pipeline::kStreams; ++i)
    if (p->streams(i)) (void)hipStreamDestroy(p->streams(i));
  delete p;
}

#define APEX_TRY(call)            \
  do {                            \
    const int rc_ = (call);       \
    if (rc_ != APEX_OK) return rc_; \
  } while (0)

}  // namespace

extern "C" {

int apex_pipeline_create(apex_replay_t *r, uint32_t depth, const apex_batch_buffers_t *sets, uint32_t num_batches,
                         uint32_t k, apex_pipeline_t **out)
{
  if (!r || !sets || !out || depth == 0 || depth > 64 || !num_batches || !k) return APEX_ERR_INVALID_ARG;
  if (num_batches > APEX_MAX_BATCHES_PER_CALL || (uint64_t)num_batches * k > APEX_MAX_SAMPLES_PER_CALL)
    return APEX_ERR_TOO_LARGE;
  for (uint32_t i = 0; i < depth; ++i) {
    const apex_batch_buffers_t &b = sets[i];
    if (!b.key || !b.slot || !b.mass || !b.weight || !b.obs || !b.act || !b.ret || !b.gacc) return APEX_ERR_INVALID_ARG;
  }
  apex_pipeline *p = new (std::nothrow) apex_pipeline();
  if (!p) return APEX_ERR_INVALID_ARG;
  p->r = r;
  p->depth = depth;
  p->nb = num_batches;
  p->k = k;
  p->sets.assign(sets, sets + depth);
  p->tree = p->add = nullptr;
  bool ok = true;
  for (hipStream_t *s : {&p->tree, &p->add})
    ok = ok && !hip_failed(hipStreamCreateWithFlags(s, hipStreamNonBlocking));  // default priority
  ok = ok && new_mark_event(&p->payload_done.own) && new_mark_event(&p->tail_ready.own) && new_event(&p->fork_ev) &&
       new_event(&p->join_ev) && new_mark_event(&p->drawn.own);
  p->wide = (uint64_t)num_batches * k >= kWideStepSamples && depth >= 2 &&
            (uint64_t)num_batches * k * r->cfg.obs_bytes >= kWideStepBytes;
  if (p->wide) {
    ok = ok && !hip_failed(hipStreamCreateWithFlags(&p->add2, hipStreamNonBlocking));
    p->gathered.resize(depth);
    for (apex_pipeline::Mark &m : p->gathered) ok = ok && new_mark_event(&m.own);
  }
  if (!ok) {
    pipeline_free(p);
    return APEX_ERR_HIP;
  }
  *out = p;
  return APEX_OK;
}

int apex_pipeline_destroy(apex_pipeline_t *p)
{
  if (!p || p->capturing) return APEX_ERR_INVALID_ARG;
  (void)issue_held_step(&p->held, p->tree);
  for (int i = 0; i < apex_pipeline::kStreams; ++i)
    if (p->streams(i)) (void)hipStreamSynchronize(p->streams(i));
  pipeline_free(p);
  return APEX_OK;
}

int apex_pipeline_fork(apex_pipeline_t *p, void *after)
{
  if (!p || p->capturing) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  APEX_HIP(hipEventRecord(p->fork_ev, static_cast<hipStream_t>(after)));
  for (int i = 0; i < apex_pipeline::kStreams; ++i)
    if (p->streams(i)) APEX_HIP(hipStreamWaitEvent(p->streams(i), p->fork_ev, 0));
  return APEX_OK;
}

int apex_pipeline_join(apex_pipeline_t *p, void *stream)
{
  if (!p || p->capturing) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  for (int i = 0; i < apex_pipeline::kStreams; ++i) {
    if (!p->streams(i)) continue;
    APEX_HIP(hipEventRecord(p->join_ev, p->streams(i)));
    APEX_HIP(hipStreamWaitEvent(static_cast<hipStream_t>(stream), p->join_ev, 0));
  }
  return APEX_OK;
}

int apex_pipeline_set_codec(apex_pipeline_t *p, uint32_t raw_bytes)
{
  if (!p || p->capturing || p->add_open) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  if (raw_bytes == 0) {
    p->codec_raw_bytes = 0;
    return APEX_OK;
  }
  const size_t stride = apex_codec_row_bytes(raw_bytes);
  if (!stride || (p->r->cfg.obs_bytes & 15)) return APEX_ERR_INVALID_ARG;
  if (stride > p->r->cfg.obs_bytes) return APEX_ERR_TOO_LARGE;
  if (!p->wide && !fused_steps_fit(p->r, p->nb, p->k, p->depth, p->sets.data())) return APEX_ERR_INVALID_ARG;
  for (const apex_batch_buffers_t &b : p->sets)
    if ((uintptr_t)b.obs & 15) return APEX_ERR_INVALID_ARG;
  p->codec_raw_bytes = raw_bytes;
  return APEX_OK;
}

int apex_pipeline_steps(apex_pipeline_t *p, uint32_t n, float beta, const uint64_t *rnd, const float *new_prio,
                        uint32_t *first_set_out)
{
  if (!p || (n && !rnd) || !(beta >= 0.0f) || !(beta <= 1.0f)) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  if (first_set_out) *first_set_out = (uint32_t)(p->step % p->depth);
  const uint64_t per = (uint64_t)p->nb * p->k;
  if (n && fused_steps_fit(p->r, p->nb, p->k, p->depth, p->sets.data())) {
    // With an add round open the last launch is held back: add_end issues it with the round (a small one)
    // or the round's masses (a large one, whose payload the other stream copies) inside.
    APEX_TRY(fused_steps(p->r, n, p->k, beta, rnd, new_prio, p->sets.data(), p->depth,
                         (uint32_t)(p->step % p->depth), p->add_open ? &p->held : nullptr, p->codec_raw_bytes,
                         p->tree));
    p->step += n;
    return APEX_OK;
  }
  if (n && p->codec_raw_bytes && !p->wide) return APEX_ERR_INVALID_ARG;  // set_codec has checked the step mode
  for (uint32_t i = 0; i < n; ++i) {
    const uint32_t set = (uint32_t)(p->step % p->depth);
    const apex_batch_buffers_t &b = p->sets[set];
    if (p->wide) {
      APEX_TRY(mark_wait(p->gathered[set], p->tree));  // the set's last gather has read slot and mass
      APEX_TRY(apex_replay_sample_begin(p->r, p->nb, p->k, rnd + i * per, b.key, b.slot, b.mass, b.act, b.ret, b.gacc,
                                        p->tree));
      APEX_TRY(mark_record(p, p->drawn, p->tree));
      hipStream_t gs = (p->step & 1) ? p->add2 : p->add;
      APEX_TRY(mark_wait(p->drawn, gs));
      if (p->codec_raw_bytes) {  // weights, then the rows through the decoder
        APEX_TRY(apex_replay_sample_finish(p->r, p->nb, p->k, beta, b.slot, b.mass, b.weight, nullptr, gs));
        APEX_TRY(apex_replay_gather_decoded(p->r, per, b.slot, p->codec_raw_bytes, b.obs, nullptr, nullptr, nullptr,
                                            gs));
      } else {
        APEX_TRY(apex_replay_sample_finish(p->r, p->nb, p->k, beta, b.slot, b.mass, b.weight, b.obs, gs));
      }
      APEX_TRY(mark_record(p, p->gathered[set], gs));
      p->last_gather[p->step & 1] = p->gathered[set].cur;
      if (new_prio) APEX_TRY(apex_replay_update_priorities(p->r, per, b.key, new_prio + i * per, p->tree));
      ++p->step;
      continue;
    }
    APEX_TRY(apex_replay_sample_begin(p->r, p->nb, p->k, rnd + i * per, b.key, b.slot, b.mass, b.act, b.ret, b.gacc,
                                      p->tree));
    // the gather of this batch, its weights, and the write-back of its priorities: one launch
    if (new_prio)
      APEX_TRY(apex_replay_sample_finish_writeback(p->r, p->nb, p->k, beta, b.key, b.slot, b.mass, b.weight, b.obs,
                                                   new_prio + i * per, p->tree));
    else
      APEX_TRY(apex_replay_sample_finish(p->r, p->nb, p->k, beta, b.slot, b.mass, b.weight, b.obs, p->tree));
    ++p->step;
  }
  return APEX_OK;
}

int apex_pipeline_add_begin(apex_pipeline_t *p, uint32_t S, uint32_t T, uint32_t n, uint32_t A, const float *q_online,
                            const float *q_target, const int32_t *action, const float *reward,
                            const float *discount, const void *obs, const void *act, float *prio, float *ret,
                            float *gacc)
{
  if (!p || p->add_open) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  apex_replay *r = p->r;
  const uint64_t count = (uint64_t)S * T;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  if (!S || !T || !n || !A || !q_online || !q_target || !action || !reward || !discount || !prio || !ret || !gacc)
    return APEX_ERR_INVALID_ARG;
  p->add_on_tree = count * r->cfg.obs_bytes < kSmallPayloadBytes;
  p->add_deferred = p->add_on_tree && obs && r->cfg.obs_bytes <= 1024 && !p->codec_raw_bytes;
  if (p->add_deferred) {
    // a small round of short rows is one launch, issued by add_end (the inputs stay untouched until then)
    p->add_ns = NstepArgs{S, T, n, A, q_online, q_target, action, reward, discount};
    p->add_obs = obs;
    p->add_act = act;
  } else {
    hipStream_t s = p->add_on_tree ? p->tree : p->add;
    if (!p->add_on_tree) {
      if (p->tail_unmarked) {  // small rounds have moved the tail since the last mark
        APEX_TRY(mark_record(p, p->tail_ready, p->tree));
        p->tail_unmarked = false;
      }
      APEX_TRY(mark_wait(p->tail_ready, p->add));  // the add stream reads tail on the device
    }
    APEX_TRY(wait_for_gathers(p, s));
    APEX_TRY(apex_nstep_priorities(S, T, n, A, q_online, q_target, action, reward, discount, r->cfg.alpha, r->cfg.eps,
                                   r->cfg.frac_bits, r->cfg.max_slots, prio, ret, gacc, nullptr, s));
    if (p->codec_raw_bytes && obs)
      APEX_TRY(apex_replay_add_payload_encoded(r, count, obs, p->codec_raw_bytes, act, ret, gacc, s));
    else
      APEX_TRY(apex_replay_add_payload(r, count, obs, act, ret, gacc, s));
    if (!p->add_on_tree) APEX_TRY(mark_record(p, p->payload_done, p->add));
  }
  p->add_open = true;
  p->add_count = count;
  p->add_prio = prio;
  return APEX_OK;
}

int apex_pipeline_add_end(apex_pipeline_t *p, int evict, uint64_t *first_key_out, uint64_t *evicted_out)
{
  if (!p || !p->add_open) return APEX_ERR_INVALID_ARG;
  if (!p->add_on_tree) APEX_TRY(mark_wait(p->payload_done, p->tree));
  if (p->add_deferred) {
    // in the launch of the step that was held back for it, if there is one and the two fit together
    int rc = issue_held_step_with_round(p->r, &p->held, p->add_ns, p->add_obs, p->add_act, first_key_out, p->tree);
    if (rc == APEX_ERR_NOT_READY) {
      APEX_TRY(issue_held_step(&p->held, p->tree));
      APEX_TRY(wait_for_gathers(p, p->tree));
      rc = add_round_small(p->r, p->add_ns, p->add_obs, p->add_act, first_key_out, p->tree);
    }
    APEX_TRY(rc);
  } else {
    int rc = issue_held_step_with_leaves(p->r, &p->held, p->add_count, p->add_prio, first_key_out, p->tree);
    if (rc == APEX_ERR_NOT_READY) rc = apex_replay_add_publish(p->r, p->add_count, p->add_prio, first_key_out, p->tree);
    APEX_TRY(rc);
  }
  p->add_open = false;
  if (evicted_out) *evicted_out = 0;
  if (evict) APEX_TRY(apex_replay_evict(p->r, evicted_out, p->tree));
  if (!p->add_on_tree) APEX_TRY(mark_record(p, p->tail_ready, p->tree));
  else p->tail_unmarked = true;
  return APEX_OK;
}

int apex_pipeline_capture_begin(apex_pipeline_t *p)
{
  if (!p || p->capturing || p->add_open) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  for (int i = 0; i < apex_pipeline::kStreams; ++i)  // drained: nothing older to wait for
    if (p->streams(i)) APEX_HIP(hipStreamSynchronize(p->streams(i)));
  drop_graph(p);
  forget_marks(p);
  APEX_HIP(hipStreamBeginCapture(p->tree, hipStreamCaptureModeRelaxed));
  p->capturing = true;
  p->r->second_version = 0;  // a replay cannot know the state it starts from: the record refreshes the second copy first
  // fork the other streams into the capture
  apex_pipeline::Mark origin;
  int rc = mark_record(p, origin, p->tree);
  for (int i = 1; i < apex_pipeline::kStreams && rc == APEX_OK; ++i)
    if (p->streams(i)) rc = mark_wait(origin, p->streams(i));
  return rc;
}

int apex_pipeline_capture_end(apex_pipeline_t *p)
{
  if (!p || !p->capturing || p->add_open) return APEX_ERR_INVALID_ARG;
  (void)issue_held_step(&p->held, p->tree);
  // join the other streams back into the origin of the capture
  int rc = APEX_OK;
  for (int i = 1; i < apex_pipeline::kStreams && rc == APEX_OK; ++i) {
    if (!p->streams(i)) continue;
    apex_pipeline::Mark done;
    rc = mark_record(p, done, p->streams(i));
    if (rc == APEX_OK) rc = mark_wait(done, p->tree);
  }
  hipGraph_t g = nullptr;
  const bool failed = hip_failed(hipStreamEndCapture(p->tree, &g));
  p->capturing = false;
  forget_marks(p);
  p->r->second_version = 0;  // what was recorded has not run
  if (failed || rc != APEX_OK || !g) {
    if (g) (void)hipGraphDestroy(g);
    return rc != APEX_OK ? rc : APEX_ERR_HIP;
  }
  p->graph = g;
  APEX_HIP(hipGraphInstantiate(&p->graph_exec, p->graph, nullptr, nullptr, 0));
  return APEX_OK;
}

int apex_pipeline_replay(apex_pipeline_t *p, uint32_t times)
{
  if (!p || p->capturing || !p->graph_exec) return APEX_ERR_INVALID_ARG;
  APEX_TRY(issue_held_step(&p->held, p->tree));
  for (uint32_t i = 0; i < times; ++i) APEX_HIP(hipGraphLaunch(p->graph_exec, p->tree));
  if (times) ++p->r->tree_version;
  return APEX_OK;
}

}  // extern "C"
