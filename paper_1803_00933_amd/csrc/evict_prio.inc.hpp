// apex_pe_*: a replay memory whose eviction is proportional prioritized sampling with its own
// exponent (Appendix "Continuous Control: Additional Details": alpha_evict = -0.4) instead of oldest
// first.  Included by apex_replay.hip (one translation unit).
//
// Two sum trees of the same shape over the same slots: sampling masses Q(p; alpha) and eviction
// masses Q(p; alpha_evict).  Slots freed by evictions go into a ring of free slots and are re-used
// by later adds in the order in which they were freed; a key is (generation of the slot << 32) |
// slot.  Evicting e transitions without replacement takes rounds: draw as many stratified points
// as are still to go on the eviction tree (the sampling kernel, pointed at that tree), drop
// repeats (they are neighbours, the points being ordered), remove the rest in the order of their
// points (a device-wide prefix sum gives each its place in the free ring), repeat.

namespace apex {

struct PeState {
  DeviceState base;  // head = evicted so far, tail = inserted so far, and the two counters
  uint64_t free_head, free_tail;   // the free ring holds slots free_ring[free_head .. free_tail) mod P
  uint64_t remaining;              // evictions still to go in the current call
};

struct PeView {
  TreeView ts, te;  // sampling masses, eviction masses
  uint32_t *gen;
  uint32_t *free_ring;
  QuantParams qs, qe;
};

__device__ __forceinline__ bool pe_key_valid(const PeView &v, uint64_t key, uint32_t *slot_out)
{
  const uint64_t slot = key & 0xffffffffu;
  if (slot >= v.ts.P) return false;
  *slot_out = (uint32_t)slot;
  return v.gen[slot] == (uint32_t)(key >> 32) && v.ts.level[0][slot] != 0;
}

__global__ __launch_bounds__(256) void pe_add_kernel(PeView v, PeState *__restrict__ st, uint64_t count,
                                                     const float *__restrict__ prio)
{
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t nclamp = 0, slot = 0;
  uint64_t q1 = 0, q2 = 0;
  if (i < count) {
    slot = v.free_ring[(st->free_head + i) % v.ts.P];
    v.gen[slot] += 1;
    bool c1, c2;
    const float p = prio[i];
    q1 = quantise_priority(p, v.qs, &c1), q2 = quantise_priority(p, v.qe, &c2);
    v.ts.level[0][slot] = q1;  // a free slot weighs nothing in either tree
    v.te.level[0][slot] = q2;
    nclamp = (uint32_t)c1 + (uint32_t)c2;
  }
  add_runs_to_ancestors(v.ts, i < count, slot, q1);
  add_runs_to_ancestors(v.te, i < count, slot, q2);
  const uint64_t nc = wave_sum(nclamp);
  if (nc && lane_id() == 0) atomic_add_u64(&st->base.n_clamped, nc);
  // the last workgroup to finish moves the free ring's head and the insertion count on
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t t = __hip_atomic_fetch_add(&st->base.ticket_add, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == gridDim.x - 1) {
      st->base.ticket_add = 0;
      st->free_head += count;
      st->base.tail += count;
    }
  }
}

// The same with the payload of short observation rows in the same launch, in workgroups of kPeAddThreads lanes.
// First 2^lanes_log2 lanes per transition copy its observation and action bytes into the next free slot; the
// first of them finds the priority - given (prio), or the n-step priority of an actor round (ns.S != 0:
// Algorithm 1, ComputePriorities; the partial return and accumulated discount are then the computed ones) - and
// leaves slot and priority in LDS.  Then one lane per transition enters the masses, whole waves of neighbouring
// transitions together (add_runs_to_ancestors).  act, ret, gacc may be null.
constexpr uint32_t kPeAddThreads = 1024;

template <typename Vec>
__global__ __launch_bounds__(kPeAddThreads) void pe_add_rows_kernel(PeView v, PeState *__restrict__ st, uint64_t count,
                                                                    NstepArgs ns, const float *__restrict__ prio,
                                                                    const uint8_t *__restrict__ obs,
                                                                    const uint8_t *__restrict__ act,
                                                                    const float *__restrict__ ret,
                                                                    const float *__restrict__ gacc,
                                                                    uint8_t *__restrict__ obs_ring,
                                                                    uint8_t *__restrict__ act_ring,
                                                                    float *__restrict__ ret_ring,
                                                                    float *__restrict__ gacc_ring, uint32_t vecs_per_row,
                                                                    uint32_t lanes_log2, uint64_t obs_bytes,
                                                                    uint32_t act_bytes)
{
  __shared__ uint32_t sh_slot[kPeAddThreads];
  __shared__ float sh_prio[kPeAddThreads];
  const uint32_t rows_per_block = blockDim.x >> lanes_log2, lanes = 1u << lanes_log2;
  const uint32_t r = threadIdx.x >> lanes_log2;
  const uint64_t i = (uint64_t)blockIdx.x * rows_per_block + r;
  const uint32_t vv = threadIdx.x & (lanes - 1);
  if (i < count) {
    const uint64_t slot = v.free_ring[(st->free_head + i) % v.ts.P];
    if (vv < vecs_per_row)
      reinterpret_cast<Vec *>(obs_ring + slot * obs_bytes)[vv] = reinterpret_cast<const Vec *>(obs + i * obs_bytes)[vv];
    if (act)
      for (uint32_t by = vv; by < act_bytes; by += lanes) act_ring[slot * act_bytes + by] = act[i * act_bytes + by];
    if (vv == 0) {
      float p;
      if (ns.S) {
        const NstepOut o = nstep_one(ns, i);
        ret_ring[slot] = o.R;
        gacc_ring[slot] = o.G;
        p = o.p;
      } else {
        if (ret) ret_ring[slot] = ret[i];
        if (gacc) gacc_ring[slot] = gacc[i];
        p = prio[i];
      }
      sh_slot[r] = (uint32_t)slot;
      sh_prio[r] = p;
    }
  }
  __syncthreads();
  if (threadIdx.x < ((rows_per_block + kWave - 1) & ~(uint32_t)(kWave - 1))) {  // whole waves
    const uint32_t e = threadIdx.x;
    const bool active = e < rows_per_block && (uint64_t)blockIdx.x * rows_per_block + e < count;
    uint32_t slot = 0, nclamp = 0;
    uint64_t q1 = 0, q2 = 0;
    if (active) {
      slot = sh_slot[e];
      v.gen[slot] += 1;
      bool c1, c2;
      q1 = quantise_priority(sh_prio[e], v.qs, &c1);
      q2 = quantise_priority(sh_prio[e], v.qe, &c2);
      v.ts.level[0][slot] = q1;  // a free slot weighs nothing in either tree
      v.te.level[0][slot] = q2;
      nclamp = (uint32_t)c1 + (uint32_t)c2;
    }
    add_runs_to_ancestors(v.ts, active, slot, q1);
    add_runs_to_ancestors(v.te, active, slot, q2);
    const uint64_t nc = wave_sum(nclamp);
    if (nc && lane_id() == 0) atomic_add_u64(&st->base.n_clamped, nc);
  }
  // the last workgroup to finish moves the free ring's head and the insertion count on
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t t = __hip_atomic_fetch_add(&st->base.ticket_add, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == gridDim.x - 1) {
      st->base.ticket_add = 0;
      st->free_head += count;
      st->base.tail += count;
    }
  }
}

// A learner batch of at most 1024 pairs in one workgroup of at least that many lanes: pairs naming one slot are
// resolved in an LDS hash table (the highest position wins), so the two passes below shrink to one launch.
// h_slot, h_pos: kDedupeSlots words of LDS each.  Called by every thread of the workgroup.
__device__ __forceinline__ void pe_update_small_block(const PeView &v, PeState *__restrict__ st, uint32_t m,
                                                      const uint64_t *__restrict__ key,
                                                      const float *__restrict__ prio, uint32_t *h_slot, uint32_t *h_pos)
{
  const uint32_t i = threadIdx.x;
  for (uint32_t t = i; t < kDedupeSlots; t += blockDim.x) {
    h_slot[t] = 0xffffffffu;
    h_pos[t] = 0;
  }
  __syncthreads();
  uint32_t slot = 0, h = 0, nclamp = 0;
  uint64_t q1 = 0, q2 = 0;
  const bool valid = i < m && pe_key_valid(v, key[i], &slot);
  const bool stale = i < m && !valid;
  if (valid) {
    h = (slot * 2654435761u) >> 21;  // top 11 bits
    for (;;) {
      const uint32_t prev = atomicCAS(&h_slot[h], 0xffffffffu, slot);
      if (prev == 0xffffffffu || prev == slot) break;
      h = (h + 1) & (kDedupeSlots - 1);
    }
    atomicMax(&h_pos[h], i + 1);
    bool c1, c2;
    const float p = prio[i];
    q1 = quantise_priority(p, v.qs, &c1);
    q2 = quantise_priority(p, v.qe, &c2);
    nclamp = (uint32_t)c1 + (uint32_t)c2;
  }
  __syncthreads();
  const bool wins = valid && h_pos[h] == i + 1;
  uint64_t d1 = 0, d2 = 0;
  if (wins) {
    d1 = q1 - v.ts.level[0][slot], d2 = q2 - v.te.level[0][slot];
    v.ts.level[0][slot] = q1;
    v.te.level[0][slot] = q2;
  }
  add_runs_to_ancestors(v.ts, wins, slot, d1);  // the keys of a drawn batch ascend: neighbours share their ancestors
  add_runs_to_ancestors(v.te, wins, slot, d2);
  const uint64_t ns = __popcll(__ballot(stale)), nc = wave_sum(nclamp);
  if (lane_id() == 0) {
    if (ns) atomic_add_u64(&st->base.n_stale, ns);
    if (nc) atomic_add_u64(&st->base.n_clamped, nc);
  }
}

__global__ __launch_bounds__(1024) void pe_update_small_kernel(PeView v, PeState *__restrict__ st, uint32_t m,
                                                               const uint64_t *__restrict__ key,
                                                               const float *__restrict__ prio)
{
  __shared__ uint32_t h_slot[kDedupeSlots];
  __shared__ uint32_t h_pos[kDedupeSlots];
  pe_update_small_block(v, st, m, key, prio, h_slot, h_pos);
}

// The write-back of the batch that the launch before has drawn, nothing having touched the trees since: pair i
// is valid, lives in slot[i] and weighs mass[i] in the sampling tree, so the loads key -> generation -> mass and
// the hash table are not needed; the drawn slots do not decrease (the strata ascend), so pairs naming one slot
// are neighbours and the last of them is the one that stands.  One workgroup of at least m lanes.
__device__ __forceinline__ void pe_writeback_block(const PeView &v, PeState *__restrict__ st, uint32_t m,
                                                   const uint32_t *__restrict__ slot, const uint64_t *__restrict__ mass,
                                                   const float *__restrict__ prio)
{
  const uint32_t i = threadIdx.x;
  const bool in = i < m;
  const uint32_t s = in ? slot[i] : 0, s_next = i + 1 < m ? slot[i + 1] : 0xffffffffu;
  const bool wins = in && s != s_next;
  uint64_t d1 = 0, d2 = 0;
  uint32_t nclamp = 0;
  if (in) {
    bool c1, c2;
    const float p = prio[i];
    const uint64_t q1 = quantise_priority(p, v.qs, &c1), q2 = quantise_priority(p, v.qe, &c2);
    nclamp = (uint32_t)c1 + (uint32_t)c2;  // counted for pairs that lose too, as when they are applied one by one
    if (wins) {
      d1 = q1 - mass[i], d2 = q2 - v.te.level[0][s];
      v.ts.level[0][s] = q1;
      v.te.level[0][s] = q2;
    }
  }
  add_runs_to_ancestors(v.ts, wins, s, d1);
  add_runs_to_ancestors(v.te, wins, s, d2);
  const uint64_t nc = wave_sum(nclamp);
  if (nc && lane_id() == 0) atomic_add_u64(&st->base.n_clamped, nc);
}

// Everything that follows the draw of one batch of short rows whose new priorities are known, in one launch of
// workgroups of 1024 lanes: workgroups [0, copy_blocks) gather the rows, the next one writes the importance
// weights, the last one writes the batch's new priorities back (m = k <= 1024 pairs).
template <typename Vec>
__global__ __launch_bounds__(1024) void pe_finish_update_kernel(ShortCopyArgs c, uint32_t copy_blocks, WeightArgs wa,
                                                                PeView v, PeState *__restrict__ st, uint32_t m,
                                                                const uint32_t *__restrict__ slot,
                                                                const float *__restrict__ prio)
{
  __shared__ uint64_t red[1024 / kWave];
  const uint32_t blk = blockIdx.x;
  if (blk < copy_blocks) {
    copy_rows_short_block<Vec>(c, blk);
  } else if (blk == copy_blocks && wa.weight_out) {
    batch_weights(wa, 0, red);
  } else if (blk == copy_blocks + 1) {
    pe_writeback_block(v, st, m, slot, wa.mass, prio);
  }
}

__global__ __launch_bounds__(256) void pe_update_claim_kernel(PeView v, PeState *__restrict__ st, uint32_t m,
                                                              const uint64_t *__restrict__ key,
                                                              uint32_t *__restrict__ claim)
{
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  bool stale = false;
  if (i < m) {
    uint32_t slot;
    if (pe_key_valid(v, key[i], &slot))
      __hip_atomic_fetch_max(claim + slot, i + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      stale = true;
  }
  const uint64_t ns = __popcll(__ballot(stale));
  if (ns && lane_id() == 0) atomic_add_u64(&st->base.n_stale, ns);
}

__global__ __launch_bounds__(256) void pe_update_apply_kernel(PeView v, PeState *__restrict__ st, uint32_t m,
                                                              const uint64_t *__restrict__ key,
                                                              const float *__restrict__ prio,
                                                              uint32_t *__restrict__ claim)
{
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t nclamp = 0;
  if (i < m) {
    uint32_t slot;
    if (pe_key_valid(v, key[i], &slot)) {  // a winner only ever writes non-zero masses, so this cannot flip
      bool c1, c2;
      const float p = prio[i];
      const uint64_t q1 = quantise_priority(p, v.qs, &c1), q2 = quantise_priority(p, v.qe, &c2);
      nclamp = (uint32_t)c1 + (uint32_t)c2;
      if (claim[slot] == i + 1) {
        const uint64_t o1 = v.ts.level[0][slot], o2 = v.te.level[0][slot];
        v.ts.level[0][slot] = q1;
        v.te.level[0][slot] = q2;
        add_to_ancestors(v.ts, slot, q1 - o1);
        add_to_ancestors(v.te, slot, q2 - o2);
        claim[slot] = 0;
      }
    }
  }
  const uint64_t nc = wave_sum(nclamp);
  if (nc && lane_id() == 0) atomic_add_u64(&st->base.n_clamped, nc);
}

__global__ void pe_begin_evict_kernel(PeState *st, uint64_t e)
{
  if (threadIdx.x == 0 && blockIdx.x == 0) st->remaining = e;
}

constexpr uint32_t kPeScanThreads = 1024;

// Which drawn candidates count (the first of each run of equal slots), and where each stands among
// those of its workgroup; the workgroup's count goes to block_sums.
__global__ __launch_bounds__(kPeScanThreads) void pe_flag_scan_kernel(const uint32_t *__restrict__ cand,
                                                                      const PeState *__restrict__ st,
                                                                      uint32_t *__restrict__ pos,
                                                                      uint32_t *__restrict__ block_sums)
{
  __shared__ uint32_t wave_tot[kPeScanThreads / kWave];
  const uint64_t rem = st->remaining;
  const uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool acc = j < rem && (j == 0 || cand[j] != cand[j - 1]);
  const uint64_t mask = __ballot(acc);
  const int lane = lane_id();
  const uint32_t wave = threadIdx.x / kWave;
  const uint32_t in_wave = __popcll(mask & ((1ull << lane) - 1));
  if (lane == 0) wave_tot[wave] = __popcll(mask);
  __syncthreads();
  uint32_t before = 0, total = 0;
  for (uint32_t w = 0; w < kPeScanThreads / kWave; ++w) {
    if (w < wave) before += wave_tot[w];
    total += wave_tot[w];
  }
  if (j < rem) pos[j] = acc ? before + in_wave : 0xffffffffu;
  if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// Removes the candidates that count, in the order of their points.  Every workgroup sums the counts of the
// workgroups before it (at most kPeScanThreads of them, one per lane) and of all of them, the round's total:
// cheaper than a launch that would do it once for all.
__global__ __launch_bounds__(kPeScanThreads) void pe_remove_kernel(PeView v, PeState *__restrict__ st,
                                                                   const uint32_t *__restrict__ cand,
                                                                   const uint32_t *__restrict__ pos,
                                                                   const uint32_t *__restrict__ block_sums)
{
  __shared__ uint32_t wave_before[kPeScanThreads / kWave], wave_all[kPeScanThreads / kWave];
  const uint32_t t = threadIdx.x, nblocks = gridDim.x;
  const uint32_t mine = t < nblocks ? block_sums[t] : 0;
  const uint32_t s_before = (uint32_t)wave_sum(t < blockIdx.x ? mine : 0), s_all = (uint32_t)wave_sum(mine);
  if (lane_id() == 0) {
    wave_before[t / kWave] = s_before;
    wave_all[t / kWave] = s_all;
  }
  __syncthreads();
  uint32_t offset = 0, round_total = 0;
  for (uint32_t w = 0; w < kPeScanThreads / kWave; ++w) {
    offset += wave_before[w];
    round_total += wave_all[w];
  }
  const uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t p = j < st->remaining ? pos[j] : 0xffffffffu;
  const bool counts = p != 0xffffffffu;
  uint32_t slot = 0;
  uint64_t o1 = 0, o2 = 0;
  if (counts) {
    slot = cand[j];
    o1 = v.ts.level[0][slot], o2 = v.te.level[0][slot];
    v.ts.level[0][slot] = 0;
    v.te.level[0][slot] = 0;
    v.free_ring[(st->free_tail + offset + p) % v.ts.P] = slot;
  }
  add_runs_to_ancestors(v.ts, counts, slot, 0 - o1);  // the candidates ascend: neighbours share their ancestors
  add_runs_to_ancestors(v.te, counts, slot, 0 - o2);
  // the last workgroup to have read the round's counters closes the round
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t tk = __hip_atomic_fetch_add(&st->base.ticket_evict, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tk == gridDim.x - 1) {
      st->base.ticket_evict = 0;
      st->free_tail += round_total;
      st->base.head += round_total;
      st->remaining -= round_total;
    }
  }
}

__global__ __launch_bounds__(256) void pe_init_free_ring_kernel(uint32_t *ring, uint64_t P, PeState *st)
{
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P) ring[i] = (uint32_t)i;
  if (i == 0) {
    st->free_head = 0;
    st->free_tail = P;
  }
}

}  // namespace apex

namespace {

struct PeGeometry {
  uint64_t obs_off, act_off, ret_off, gacc_off, storage_bytes;
  uint32_t nlev;
  uint64_t level_off[kMaxLevels], level_size[kMaxLevels], tree_words;  // of one tree; the second follows it
  uint64_t state_off, mass_off, cand_off, pos_off, sums_off, gen_off, ring_off, claim_off, scratch_bytes;
};

int pe_validate(const apex_pe_config_t *c)
{
  if (!c) return APEX_ERR_INVALID_ARG;
  if (c->capacity == 0 || c->max_slots < c->capacity || c->max_slots > (1ull << 31)) return APEX_ERR_INVALID_ARG;
  if (c->obs_bytes == 0 || c->act_bytes == 0 || c->frac_bits > 32) return APEX_ERR_INVALID_ARG;
  if (!(c->alpha >= -1.0f && c->alpha <= 1.0f) || !(c->alpha_evict >= -1.0f && c->alpha_evict <= 1.0f))
    return APEX_ERR_INVALID_ARG;
  if (!(c->eps >= 0.0f) || !(c->eps < 1e30f)) return APEX_ERR_INVALID_ARG;
  return APEX_OK;
}

int pe_geometry(const apex_pe_config_t *c, PeGeometry *g)
{
  apex_replay_config_t rc{};
  rc.capacity = c->capacity;
  rc.max_slots = c->max_slots;
  rc.obs_bytes = c->obs_bytes;
  rc.act_bytes = c->act_bytes;
  Geometry base;
  const int rv = geometry(&rc, &base);
  if (rv != APEX_OK) return rv;
  g->obs_off = base.obs_off;
  g->act_off = base.act_off;
  g->ret_off = base.ret_off;
  g->gacc_off = base.gacc_off;
  g->storage_bytes = base.storage_bytes;
  g->nlev = base.nlev;
  for (uint32_t l = 0; l < kMaxLevels; ++l) {
    g->level_off[l] = base.level_off[l];
    g->level_size[l] = base.level_size[l];
  }
  g->tree_words = base.tree_words;
  const uint64_t P = c->max_slots;
  g->state_off = 0;
  g->mass_off = 256;
  g->cand_off = g->mass_off + (uint64_t)APEX_PE_MAX_EVICT_PER_CALL * 8;  // also holds the masses of a sample call
  g->pos_off = g->cand_off + (uint64_t)APEX_PE_MAX_EVICT_PER_CALL * 4;
  g->sums_off = g->pos_off + (uint64_t)APEX_PE_MAX_EVICT_PER_CALL * 4;
  g->gen_off = g->sums_off + round_up(kPeScanThreads * 4, 256);
  g->ring_off = g->gen_off + round_up(P * 4, 256);
  g->claim_off = g->ring_off + round_up(P * 4, 256);
  g->scratch_bytes = g->claim_off + round_up(P * 4, 256);
  return APEX_OK;
}

}  // namespace

struct apex_pe_replay {
  apex_pe_config_t cfg;
  PeGeometry geo;
  uint8_t *storage;
  uint64_t *tree;
  uint8_t *scratch;
  // Host mirror.  `evicted` is what the host takes to have been evicted: exact after calls that report back
  // (apex_pe_evict, apex_pe_stats); after apex_pe_evict_enqueue it assumes that the eviction removed all it was
  // asked to, until the snapshot of the device's counters that the call left behind says otherwise.
  uint64_t inserted, evicted;
  uint64_t evicted_confirmed = 0;  // the last value read back from the device: evicted >= evicted_confirmed
  bool pending = false;            // a snapshot has been requested and not looked at yet
  uint64_t pending_claim = 0;      // what `evicted` was taken to be when it was requested
  PeState *snap = nullptr;         // pinned host memory that the snapshot lands in
  hipEvent_t snap_ev = nullptr;    // recorded behind the snapshot's copy
  PeView v;

  PeState *state() const { return reinterpret_cast<PeState *>(scratch + geo.state_off); }
  uint64_t *mass() const { return reinterpret_cast<uint64_t *>(scratch + geo.mass_off); }
  uint32_t *cand() const { return reinterpret_cast<uint32_t *>(scratch + geo.cand_off); }
  uint32_t *pos() const { return reinterpret_cast<uint32_t *>(scratch + geo.pos_off); }
  uint32_t *sums() const { return reinterpret_cast<uint32_t *>(scratch + geo.sums_off); }
  uint32_t *claim() const { return reinterpret_cast<uint32_t *>(scratch + geo.claim_off); }
  uint8_t *obs() const { return storage + geo.obs_off; }
  uint8_t *act() const { return storage + geo.act_off; }
  float *ret() const { return reinterpret_cast<float *>(storage + geo.ret_off); }
  float *gacc() const { return reinterpret_cast<float *>(storage + geo.gacc_off); }
  uint64_t size() const { return inserted - evicted; }
};

namespace {

// Looks at the snapshot that apex_pe_evict_enqueue requested, if it has arrived (wait: blocks until it has),
// and corrects the mirror if that eviction fell short of what it was asked for.
int pe_resolve(apex_pe_replay *r, bool wait)
{
  if (!r->pending) return APEX_OK;
  if (wait) {
    APEX_HIP(hipEventSynchronize(r->snap_ev));
  } else {
    const hipError_t e = hipEventQuery(r->snap_ev);
    if (e == hipErrorNotReady) {
      (void)hipGetLastError();  // not an error: nothing to report later
      return APEX_OK;
    }
    if (hip_failed(e)) return APEX_ERR_HIP;
  }
  r->pending = false;
  const uint64_t head = r->snap->base.head;
  r->evicted_confirmed = head;
  if (head < r->pending_claim) r->evicted -= r->pending_claim - head;  // the rounds ran out: fewer are gone
  return APEX_OK;
}

// Room for `count` more?  Decided from the mirror; where the mirror rests on an eviction that has not been
// confirmed and the answer depends on it, the confirmation is waited for.
int pe_check_room(apex_pe_replay *r, uint64_t count)
{
  APEX_TRY(pe_resolve(r, false));
  if (r->pending && r->inserted - r->evicted_confirmed + count > r->cfg.max_slots) APEX_TRY(pe_resolve(r, true));
  return r->size() + count > r->cfg.max_slots ? APEX_ERR_FULL : APEX_OK;
}

// The launches of an eviction of e transitions in `rounds` rounds.
int pe_enqueue_eviction(apex_pe_replay *r, uint64_t e, uint32_t rounds, const uint64_t *rnd, hipStream_t stream)
{
  PeState *st = r->state();
  pe_begin_evict_kernel<<<dim3(1), dim3(64), 0, stream>>>(st, e);
  SampleArgs a{};
  a.tv = r->v.te;
  a.st = &st->base;
  a.k = 0;
  a.k_dev = &st->remaining;
  a.gen = nullptr;
  a.key_out = nullptr;
  a.slot_out = r->cand();
  a.mass = r->mass();
  a.act = nullptr;
  a.act_bytes = 0;
  a.ret = a.gacc = nullptr;
  a.act_out = nullptr;
  a.ret_out = a.gacc_out = nullptr;
  const uint32_t waves = 4;  // (16 waves per workgroup, which stage the top level fewer times, measured 20 % slower)
  const size_t lds = ((size_t)a.tv.n_top + waves) * sizeof(uint64_t);
  const uint32_t scan_blocks = blocks_for(e, kPeScanThreads);  // <= 1024 since e <= 2^20
  for (uint32_t rd = 0; rd < rounds; ++rd) {
    a.rnd = rnd + (uint64_t)rd * e;
    sample_descent_kernel<<<dim3(blocks_for(e, waves), 1), dim3(waves * kWave), lds, stream>>>(a);
    pe_flag_scan_kernel<<<dim3(scan_blocks), dim3(kPeScanThreads), 0, stream>>>(r->cand(), st, r->pos(), r->sums());
    pe_remove_kernel<<<dim3(scan_blocks), dim3(kPeScanThreads), 0, stream>>>(r->v, st, r->cand(), r->pos(), r->sums());
  }
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

void pe_free(apex_pe_replay *r)
{
  if (r->snap_ev) (void)hipEventDestroy(r->snap_ev);
  if (r->snap) (void)hipHostFree(r->snap);
  delete r;
}

}  // namespace

extern "C" {

int apex_pe_workspace_bytes(const apex_pe_config_t *cfg, size_t *storage_bytes, size_t *tree_bytes,
                            size_t *scratch_bytes)
{
  int rc = pe_validate(cfg);
  if (rc != APEX_OK) return rc;
  PeGeometry g;
  rc = pe_geometry(cfg, &g);
  if (rc != APEX_OK) return rc;
  if (storage_bytes) *storage_bytes = g.storage_bytes;
  if (tree_bytes) *tree_bytes = 2 * g.tree_words * 8;
  if (scratch_bytes) *scratch_bytes = g.scratch_bytes;
  return APEX_OK;
}

int apex_pe_create(const apex_pe_config_t *cfg, void *d_storage, void *d_tree, void *d_scratch, apex_pe_replay_t **out)
{
  int rc = pe_validate(cfg);
  if (rc != APEX_OK) return rc;
  if (!d_storage || !d_tree || !d_scratch || !out) return APEX_ERR_INVALID_ARG;
  if (((uintptr_t)d_storage | (uintptr_t)d_tree | (uintptr_t)d_scratch) & 255) return APEX_ERR_INVALID_ARG;
  apex_pe_replay *r = new (std::nothrow) apex_pe_replay();
  if (!r) return APEX_ERR_INVALID_ARG;
  r->cfg = *cfg;
  rc = pe_geometry(cfg, &r->geo);
  if (rc != APEX_OK) {
    delete r;
    return rc;
  }
  r->storage = static_cast<uint8_t *>(d_storage);
  r->tree = static_cast<uint64_t *>(d_tree);
  r->scratch = static_cast<uint8_t *>(d_scratch);
  r->inserted = r->evicted = 0;
  const uint64_t qmax = qmax_for(cfg->max_slots);
  r->v.qs = QuantParams{cfg->alpha, cfg->eps, cfg->frac_bits, qmax};
  r->v.qe = QuantParams{cfg->alpha_evict, cfg->eps, cfg->frac_bits, qmax};
  for (TreeView *tv : {&r->v.ts, &r->v.te}) {
    tv->nlev = r->geo.nlev;
    tv->n_top = (uint32_t)r->geo.level_size[r->geo.nlev - 1];
    tv->P = cfg->max_slots;
    uint64_t *base = r->tree + (tv == &r->v.te ? r->geo.tree_words : 0);
    for (uint32_t l = 0; l < kMaxLevels; ++l) tv->level[l] = l < r->geo.nlev ? base + r->geo.level_off[l] : nullptr;
  }
  r->v.gen = reinterpret_cast<uint32_t *>(r->scratch + r->geo.gen_off);
  r->v.free_ring = reinterpret_cast<uint32_t *>(r->scratch + r->geo.ring_off);
  // (host memory and an event for apex_pe_evict_enqueue's snapshots: no device memory is allocated)
  if (hip_failed(hipHostMalloc(reinterpret_cast<void **>(&r->snap), sizeof(PeState), hipHostMallocDefault)) ||
      hip_failed(hipEventCreateWithFlags(&r->snap_ev, hipEventDisableTiming))) {
    pe_free(r);
    return APEX_ERR_HIP;
  }
  fill_zero_kernel<<<dim3(1024), dim3(256), 0, nullptr>>>(r->tree, 2 * r->geo.tree_words);
  fill_zero_kernel<<<dim3(1024), dim3(256), 0, nullptr>>>(reinterpret_cast<uint64_t *>(r->scratch),
                                                          r->geo.scratch_bytes / 8);
  pe_init_free_ring_kernel<<<dim3(blocks_for(cfg->max_slots, 256)), dim3(256), 0, nullptr>>>(
      r->v.free_ring, cfg->max_slots, r->state());
  if (hip_failed(hipGetLastError()) || hip_failed(hipDeviceSynchronize())) {
    pe_free(r);
    return APEX_ERR_HIP;
  }
  *out = r;
  return APEX_OK;
}

int apex_pe_destroy(apex_pe_replay_t *r)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  if (r->pending) (void)hipEventSynchronize(r->snap_ev);  // the snapshot's copy still names r->snap
  pe_free(r);
  return APEX_OK;
}

int apex_pe_layout(const apex_pe_replay_t *r, apex_pe_layout_t *out)
{
  if (!r || !out) return APEX_ERR_INVALID_ARG;
  out->obs_offset = r->geo.obs_off;
  out->act_offset = r->geo.act_off;
  out->ret_offset = r->geo.ret_off;
  out->gacc_offset = r->geo.gacc_off;
  out->tree_levels = r->geo.nlev;
  out->tree_fanout = kFanout;
  for (uint32_t l = 0; l < APEX_TREE_MAX_LEVELS; ++l) {
    out->level_offset[l] = l < r->geo.nlev ? r->geo.level_off[l] : 0;
    out->level_size[l] = l < r->geo.nlev ? r->geo.level_size[l] : 0;
  }
  out->evict_tree_offset = r->geo.tree_words;
  out->gen_offset = r->geo.gen_off;
  out->free_ring_offset = r->geo.ring_off;
  return APEX_OK;
}

int apex_pe_add(apex_pe_replay_t *r, uint64_t count, const void *obs, const void *act, const float *ret,
                const float *gacc, const float *prio, void *hip_stream)
{
  if (!r || (count && !prio)) return APEX_ERR_INVALID_ARG;
  APEX_TRY(pe_check_room(r, count));
  if (count == 0) return APEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const RowMap freed{r->v.free_ring, &r->state()->free_head, r->cfg.max_slots};  // the next free slots, in order
  const PayloadRing pr{r->obs(), r->act(), r->ret(), r->gacc(), r->cfg.obs_bytes, r->cfg.act_bytes};
  const uintptr_t mis = (uintptr_t)obs | (uintptr_t)r->obs() | (uintptr_t)r->cfg.obs_bytes;
  const uint32_t vb = (mis & 15) == 0 ? 16 : (mis & 3) == 0 ? 4 : 1;
  const uint32_t vpr = r->cfg.obs_bytes / vb;
  if (obs && vpr <= 256) {  // short rows: payload and masses in one launch
    uint32_t lanes_log2 = 0;
    while ((1u << lanes_log2) < vpr) ++lanes_log2;
    const uint64_t rows_per_block = kPeAddThreads >> lanes_log2;
    const uint64_t blocks = (count + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffffull) return APEX_ERR_TOO_LARGE;
    const dim3 grid((uint32_t)blocks), block(kPeAddThreads);
    const uint8_t *o8 = static_cast<const uint8_t *>(obs), *a8 = static_cast<const uint8_t *>(act);
#define APEX_PE_ADD_SHORT(Vec)                                                                                        \
  pe_add_rows_kernel<Vec><<<grid, block, 0, stream>>>(r->v, r->state(), count, NstepArgs{}, prio, o8, a8, ret, gacc,   \
                                                      pr.obs, pr.act, pr.ret, pr.gacc, vpr, lanes_log2, pr.obs_bytes, \
                                                      pr.act_bytes)
    if (vb == 16) APEX_PE_ADD_SHORT(u32x4);
    else if (vb == 4) APEX_PE_ADD_SHORT(uint32_t);
    else APEX_PE_ADD_SHORT(uint8_t);
#undef APEX_PE_ADD_SHORT
  } else {
    const int rc = add_payload_rows(pr, count, obs, act, ret, gacc, freed, stream);
    if (rc != APEX_OK) return rc;
    pe_add_kernel<<<dim3(blocks_for(count, 256)), dim3(256), 0, stream>>>(r->v, r->state(), count, prio);
  }
  APEX_HIP(hipGetLastError());
  r->inserted += count;
  return APEX_OK;
}

int apex_pe_sample(apex_pe_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                   uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                   float *ret_out, float *gacc_out, void *hip_stream)
{
  if (!r || !num_batches || !k || !rnd || !slot_out || !(beta >= 0.0f) || !(beta <= 1.0f)) return APEX_ERR_INVALID_ARG;
  if (num_batches > APEX_MAX_BATCHES_PER_CALL || (uint64_t)num_batches * k > APEX_MAX_SAMPLES_PER_CALL)
    return APEX_ERR_TOO_LARGE;
  if (r->size() == 0) return APEX_ERR_EMPTY;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  SampleArgs a{};
  a.tv = r->v.ts;
  a.st = &r->state()->base;
  a.k = k;
  a.k_dev = nullptr;
  a.gen = r->v.gen;
  a.rnd = rnd;
  a.key_out = key_out;
  a.slot_out = slot_out;
  a.mass = r->mass();
  a.act = r->act();
  a.act_bytes = r->cfg.act_bytes;
  a.ret = r->ret();
  a.gacc = r->gacc();
  a.act_out = static_cast<uint8_t *>(act_out);
  a.ret_out = ret_out;
  a.gacc_out = gacc_out;
  const uint32_t waves = 4;
  const size_t lds = ((size_t)a.tv.n_top + waves) * sizeof(uint64_t);
  sample_descent_kernel<<<dim3(blocks_for(k, waves), num_batches), dim3(waves * kWave), lds, stream>>>(a);
  APEX_HIP(hipGetLastError());
  SideJobs jobs;
  jobs.wa = WeightArgs{r->mass(), weight_out, k, beta};
  if (obs_out) {
    const RowMap by_slot{slot_out, nullptr, 0};
    const RowMap ident{nullptr, nullptr, 0};
    const int rc = launch_copy(r->obs(), by_slot, obs_out, ident, (uint64_t)num_batches * k, r->cfg.obs_bytes, stream, &jobs);
    if (rc != APEX_OK) return rc;
  }
  if (jobs.wa.weight_out) {
    batch_weights_kernel<<<dim3(num_batches, blocks_for(k, 512)), dim3(256), 0, stream>>>(jobs.wa);
    APEX_HIP(hipGetLastError());
  }
  return APEX_OK;
}

int apex_pe_update_priorities(apex_pe_replay_t *r, uint64_t m, const uint64_t *key, const float *prio,
                              void *hip_stream)
{
  if (!r || (m && (!key || !prio))) return APEX_ERR_INVALID_ARG;
  if (m >= 0xffffffffull) return APEX_ERR_TOO_LARGE;
  if (m == 0) return APEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (m <= 1024) {
    pe_update_small_kernel<<<dim3(1), dim3((uint32_t)round_up(m, kWave)), 0, stream>>>(r->v, r->state(), (uint32_t)m, key, prio);
    APEX_HIP(hipGetLastError());
    return APEX_OK;
  }
  const dim3 grid(blocks_for(m, 256)), block(256);
  pe_update_claim_kernel<<<grid, block, 0, stream>>>(r->v, r->state(), (uint32_t)m, key, r->claim());
  pe_update_apply_kernel<<<grid, block, 0, stream>>>(r->v, r->state(), (uint32_t)m, key, prio, r->claim());
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

int apex_pe_evict(apex_pe_replay_t *r, uint32_t rounds, const uint64_t *rnd, uint64_t *evicted_out, void *hip_stream)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  APEX_TRY(pe_resolve(r, true));  // this call reports back anyway: start from exact counts
  const uint64_t size = r->size();
  const uint64_t e = size > r->cfg.capacity ? size - r->cfg.capacity : 0;
  if (evicted_out) *evicted_out = 0;
  if (e == 0) return APEX_OK;
  if (!rnd || rounds == 0) return APEX_ERR_INVALID_ARG;
  if (e > APEX_PE_MAX_EVICT_PER_CALL) return APEX_ERR_TOO_LARGE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  APEX_TRY(pe_enqueue_eviction(r, e, rounds, rnd, stream));
  PeState h;
  APEX_HIP(hipMemcpyAsync(&h, r->state(), sizeof h, hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipStreamSynchronize(stream));
  r->evicted = r->evicted_confirmed = h.base.head;
  if (evicted_out) *evicted_out = e - h.remaining;
  return APEX_OK;
}

int apex_pe_evict_enqueue(apex_pe_replay_t *r, uint32_t rounds, const uint64_t *rnd, uint64_t *requested_out,
                          void *hip_stream)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  APEX_TRY(pe_resolve(r, true));  // the snapshot of the eviction before this one (long done by now) frees r->snap
  const uint64_t size = r->size();
  const uint64_t e = size > r->cfg.capacity ? size - r->cfg.capacity : 0;
  if (requested_out) *requested_out = e;
  if (e == 0) return APEX_OK;
  if (!rnd || rounds == 0) return APEX_ERR_INVALID_ARG;
  if (e > APEX_PE_MAX_EVICT_PER_CALL) return APEX_ERR_TOO_LARGE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  APEX_TRY(pe_enqueue_eviction(r, e, rounds, rnd, stream));
  APEX_HIP(hipMemcpyAsync(r->snap, r->state(), sizeof(PeState), hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipEventRecord(r->snap_ev, stream));
  r->evicted += e;
  r->pending = true;
  r->pending_claim = r->evicted;
  return APEX_OK;
}

int apex_pe_add_round(apex_pe_replay_t *r, uint32_t S, uint32_t T, uint32_t n, uint32_t A, const float *q_online,
                      const float *q_target, const int32_t *action, const float *reward, const float *discount,
                      const void *obs, const void *act, void *hip_stream)
{
  if (!r || !S || !T || !n || !A || !q_online || !q_target || !action || !reward || !discount || !obs)
    return APEX_ERR_INVALID_ARG;
  const uint64_t count = (uint64_t)S * T;
  if ((uint64_t)T + n > 0xffffffffull) return APEX_ERR_TOO_LARGE;
  const uintptr_t mis = (uintptr_t)obs | (uintptr_t)r->obs() | (uintptr_t)r->cfg.obs_bytes;
  const uint32_t vb = (mis & 15) == 0 ? 16 : (mis & 3) == 0 ? 4 : 1;
  const uint32_t vpr = r->cfg.obs_bytes / vb;
  if (vpr > 256) return APEX_ERR_TOO_LARGE;  // long rows: apex_nstep_priorities + apex_pe_add
  APEX_TRY(pe_check_room(r, count));
  uint32_t lanes_log2 = 0;
  while ((1u << lanes_log2) < vpr) ++lanes_log2;
  const uint64_t rows_per_block = kPeAddThreads >> lanes_log2;
  const uint64_t blocks = (count + rows_per_block - 1) / rows_per_block;
  if (blocks > 0x7fffffffull) return APEX_ERR_TOO_LARGE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const NstepArgs ns{S, T, n, A, q_online, q_target, action, reward, discount};
  const dim3 grid((uint32_t)blocks), block(kPeAddThreads);
  const uint8_t *o8 = static_cast<const uint8_t *>(obs), *a8 = static_cast<const uint8_t *>(act);
#define APEX_PE_ADD_ROUND(Vec)                                                                                          \
  pe_add_rows_kernel<Vec><<<grid, block, 0, stream>>>(r->v, r->state(), count, ns, nullptr, o8, a8, nullptr, nullptr,    \
                                                      r->obs(), r->act(), r->ret(), r->gacc(), vpr, lanes_log2,         \
                                                      r->cfg.obs_bytes, r->cfg.act_bytes)
  if (vb == 16) APEX_PE_ADD_ROUND(u32x4);
  else if (vb == 4) APEX_PE_ADD_ROUND(uint32_t);
  else APEX_PE_ADD_ROUND(uint8_t);
#undef APEX_PE_ADD_ROUND
  APEX_HIP(hipGetLastError());
  r->inserted += count;
  return APEX_OK;
}

int apex_pe_sample_update(apex_pe_replay_t *r, uint32_t k, float beta, const uint64_t *rnd, const float *new_prio,
                          uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                          float *ret_out, float *gacc_out, void *hip_stream)
{
  if (!r || !k || !rnd || !new_prio || !key_out || !slot_out || !(beta >= 0.0f) || !(beta <= 1.0f))
    return APEX_ERR_INVALID_ARG;
  if (k > 1024) return APEX_ERR_TOO_LARGE;
  const uintptr_t mis = (uintptr_t)obs_out | (uintptr_t)r->obs() | (uintptr_t)r->cfg.obs_bytes;
  const uint32_t vb = (mis & 15) == 0 ? 16 : (mis & 3) == 0 ? 4 : 1;
  const uint32_t vpr = r->cfg.obs_bytes / vb;
  if (obs_out && vpr > 256) return APEX_ERR_TOO_LARGE;  // long rows: apex_pe_sample + apex_pe_update_priorities
  if (r->size() == 0) return APEX_ERR_EMPTY;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  SampleArgs a{};
  a.tv = r->v.ts;
  a.st = &r->state()->base;
  a.k = k;
  a.gen = r->v.gen;
  a.rnd = rnd;
  a.key_out = key_out;
  a.slot_out = slot_out;
  a.mass = r->mass();
  a.act = r->act();
  a.act_bytes = r->cfg.act_bytes;
  a.ret = r->ret();
  a.gacc = r->gacc();
  a.act_out = static_cast<uint8_t *>(act_out);
  a.ret_out = ret_out;
  a.gacc_out = gacc_out;
  const uint32_t waves = 4;
  const size_t lds = ((size_t)a.tv.n_top + waves) * sizeof(uint64_t);
  sample_descent_kernel<<<dim3(blocks_for(k, waves), 1), dim3(waves * kWave), lds, stream>>>(a);
  // gather, weights and the write-back of the batch just drawn: one launch
  uint32_t lanes_log2 = 0;
  while ((1u << lanes_log2) < vpr) ++lanes_log2;
  const uint64_t rows_per_block = 1024u >> lanes_log2;
  const uint32_t copy_blocks = obs_out ? (uint32_t)((k + rows_per_block - 1) / rows_per_block) : 0;
  const ShortCopyArgs c{r->obs(), RowMap{slot_out, nullptr, 0}, static_cast<uint8_t *>(obs_out), RowMap{nullptr, nullptr, 0},
                        k, vpr, lanes_log2, r->cfg.obs_bytes};
  const WeightArgs wa{r->mass(), weight_out, k, beta};
  const dim3 grid(copy_blocks + 2), block(1024);
#define APEX_PE_FINISH(Vec) \
  pe_finish_update_kernel<Vec><<<grid, block, 0, stream>>>(c, copy_blocks, wa, r->v, r->state(), k, slot_out, new_prio)
  if (vb == 16) APEX_PE_FINISH(u32x4);
  else if (vb == 4) APEX_PE_FINISH(uint32_t);
  else APEX_PE_FINISH(uint8_t);
#undef APEX_PE_FINISH
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

int apex_pe_stats(apex_pe_replay_t *r, apex_pe_stats_t *out, void *hip_stream)
{
  if (!r || !out) return APEX_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  PeState h;
  static thread_local uint64_t top[2][kTopMax];
  const uint32_t n_top = r->v.ts.n_top;
  APEX_HIP(hipMemcpyAsync(&h, r->state(), sizeof h, hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipMemcpyAsync(top[0], r->v.ts.level[r->v.ts.nlev - 1], (size_t)n_top * 8, hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipMemcpyAsync(top[1], r->v.te.level[r->v.te.nlev - 1], (size_t)n_top * 8, hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipStreamSynchronize(stream));
  uint64_t root[2] = {0, 0};
  for (int t = 0; t < 2; ++t)
    for (uint32_t i = 0; i < n_top; ++i) root[t] += top[t][i];
  if (r->pending) APEX_TRY(pe_resolve(r, true));  // (an enqueued eviction's snapshot precedes this read on the stream
                                                  // only if it was enqueued on hip_stream; else it is simply waited for)
  out->size = h.base.tail - h.base.head;
  out->inserted = h.base.tail;
  out->evicted = h.base.head;
  out->root = root[0];
  out->root_evict = root[1];
  out->free_head = h.free_head;
  out->free_tail = h.free_tail;
  out->n_stale_dropped = h.base.n_stale;
  out->n_clamped = h.base.n_clamped;
  return APEX_OK;
}

}  // extern "C"
