// HIP kernels of the replay memory (gfx950).  Host-side entry points are in apex_replay.hip.
//
// Data layout in HBM
//   payload ring   obs[P][obs_bytes], act[P][act_bytes], ret[P], gacc[P]   (structure of arrays)
//   sum tree       level 0 = one uint64 mass per slot; node i of level l+1 = sum of nodes
//                  [64 i, 64 i + 64) of level l; levels are added until one has at most kTopMax
//                  nodes.  A wavefront reads the 64 children of a node as one coalesced 512-byte
//                  row; the top level is staged and prefix-summed in LDS by every workgroup.
//   device state   head, tail, counters: read by the kernels, so the same launches can be replayed.
// The set of transitions and the sampled indices do not depend on this shape: a sample is
// defined by the cumulative mass in slot order, whatever tree sums it up.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "quantise.hpp"
#include "wave.hpp"

namespace apex {

constexpr uint32_t kFanoutLog2 = 6;
constexpr uint32_t kFanout = 1u << kFanoutLog2;
constexpr uint32_t kTopMax = 4608;  // 36 KB of LDS; covers 2^24 + 2^20 slots with three levels
constexpr uint32_t kMaxLevels = 8;

struct DeviceState {
  uint64_t head, tail;      // valid keys: head <= key < tail
  uint64_t n_stale, n_clamped;
  uint32_t ticket_add;      // workgroups of the running add launch that are done with tail ...
  uint32_t ticket_evict;    // ... and of the running evict launch that are done with head (the two may overlap)
};

// Called by every thread of every workgroup of a launch once it has read what it needs of head or
// tail: the workgroup that arrives last moves that counter on, so that the launch needs no
// follow-up launch for it (the ticket is back at 0 afterwards).  Contains a barrier.
// n_wgs: the workgroups that take part (all of the launch unless stated).
__device__ __forceinline__ void advance_state_when_all_done(uint32_t *ticket, uint64_t *counter, uint64_t inc,
                                                            uint32_t n_wgs = gridDim.x)
{
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == n_wgs - 1) {
      *ticket = 0;
      *counter += inc;
    }
  }
}

struct TreeView {
  uint64_t *level[kMaxLevels];
  uint32_t nlev;   // level nlev-1 is the top
  uint32_t n_top;  // nodes of the top level
  uint64_t P;      // ring size
};

// Adds delta (mod 2^64) to every ancestor of `slot` above level 0.
__device__ __forceinline__ void add_to_ancestors(const TreeView &tv, uint64_t slot, uint64_t delta)
{
  uint64_t idx = slot;
  for (uint32_t l = 1; l < tv.nlev; ++l) {
    idx >>= kFanoutLog2;
    atomic_add_u64(tv.level[l] + idx, delta);
  }
}

// Same, for a wave whose active lanes hold neighbouring slots (adds, evictions): lanes under one
// level-1 node are summed first, so each node receives one atomic per wave instead of up to 64.
// Must be called by all 64 lanes; `active` marks the lanes that carry a delta.
// second: another copy of the same tree that receives the same sums, or null.
__device__ __forceinline__ void add_to_ancestors_grouped(const TreeView &tv, bool active, uint64_t slot, uint64_t delta,
                                                         const TreeView *second = nullptr)
{
  const int lane = lane_id();
  const uint64_t node1 = slot >> kFanoutLog2;
  uint64_t todo = __ballot(active);
  while (todo) {
    const int leader = __ffsll((unsigned long long)todo) - 1;
    const uint64_t node = __shfl(node1, leader, kWave);
    const bool mine = active && node1 == node;
    const uint64_t sum = wave_sum(mine ? delta : 0);
    if (lane == leader) {
      uint64_t idx = node;
      for (uint32_t l = 1; l < tv.nlev; ++l) {
        atomic_add_u64(tv.level[l] + idx, sum);
        if (second) atomic_add_u64(second->level[l] + idx, sum);
        idx >>= kFanoutLog2;
      }
    }
    todo &= ~__ballot(mine);
  }
}

// Same, for a wave whose lanes hold slots in any order (the free slots that a memory with prioritized
// eviction hands out, the candidates of an eviction round - both mostly ascending, so that neighbouring lanes
// mostly share their ancestors): on every level each run of neighbouring lanes under one node is summed with
// one prefix sum over the wave and sends one atomic.  A node that appears in several runs receives several
// atomics.  Sums are modulo 2^64, so a removal passes 0 - mass.  Must be called by all 64 lanes.
__device__ __forceinline__ void add_runs_to_ancestors(const TreeView &tv, bool active, uint64_t slot, uint64_t delta)
{
  const int lane = lane_id();
  const uint64_t incl = wave_inclusive_scan(active ? delta : 0);
  uint64_t idx = slot;
  for (uint32_t l = 1; l < tv.nlev; ++l) {
    idx >>= kFanoutLog2;
    const uint64_t node = active ? idx : ~0ull;  // lanes without a delta form runs of their own, which send nothing
    const uint64_t prev = __shfl_up(node, 1, kWave);
    const uint64_t starts = __ballot(lane == 0 || prev != node);
    const bool ends = lane == kWave - 1 || ((starts >> (lane + 1)) & 1);
    const int first = 63 - __builtin_clzll(starts & (~0ull >> (63 - lane)));  // where this lane's run starts (bit 0 is set)
    const uint64_t before = __shfl(incl, first > 0 ? first - 1 : 0, kWave);
    if (active && ends) atomic_add_u64(tv.level[l] + idx, incl - (first > 0 ? before : 0));
  }
}

// --------------------------------------------------------------------------------------------
// n-step priorities: one thread per transition (Algorithm 1, ComputePriorities; Sections 3.1, 3.2)
// --------------------------------------------------------------------------------------------
struct NstepArgs {
  uint32_t S, T, n, A;
  const float *q_online, *q_target;  // [S, T+n, A]
  const int32_t *action;             // [S, T+n]
  const float *reward, *discount;    // [S, T+n]
};

struct NstepOut {
  float p, R, G;  // priority |delta|, partial return, accumulated discount
};

// Transition gid = s * T + t of an add round (gid < S * T).
__device__ __forceinline__ NstepOut nstep_one(const NstepArgs &a, uint64_t gid)
{
  const uint32_t T = a.T, n = a.n, A = a.A;
  const uint32_t s = (uint32_t)(gid / T), t = (uint32_t)(gid - (uint64_t)s * T);
  const uint64_t row0 = (uint64_t)s * (T + n);  // first row of this stream
  const float *rw = a.reward + row0 + t;
  const float *dc = a.discount + row0 + t;

  float R = 0.0f;
  for (int j = (int)n - 1; j >= 0; --j) R = __builtin_fmaf(dc[j], R, rw[j]);  // Horner, one rounding per step
  float G = 1.0f;
  for (uint32_t j = 0; j < n; ++j) G = G * dc[j];

  const float *qrow = a.q_online + (row0 + t + n) * A;
  uint32_t best = 0;
  float vbest = qrow[0];
  for (uint32_t b = 1; b < A; ++b) {
    const float v = qrow[b];
    if (v > vbest) {
      vbest = v;
      best = b;
    }
  }
  const float boot = a.q_target[(row0 + t + n) * A + best];
  uint32_t at = (uint32_t)a.action[row0 + t];
  if (at >= A) at = A - 1;  // keeps a corrupt action index inside the row
  const float target = __builtin_fmaf(G, boot, R);
  const float delta = target - a.q_online[(row0 + t) * A + at];
  return NstepOut{__builtin_fabsf(delta), R, G};
}

__global__ __launch_bounds__(256) void nstep_kernel(NstepArgs a, QuantParams qp, float *__restrict__ prio,
                                                    float *__restrict__ ret, float *__restrict__ gacc,
                                                    uint64_t *__restrict__ prio_fx)
{
  const uint64_t gid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (uint64_t)a.S * a.T) return;
  const NstepOut o = nstep_one(a, gid);
  ret[gid] = o.R;
  gacc[gid] = o.G;
  prio[gid] = o.p;
  if (prio_fx) {
    bool c;
    prio_fx[gid] = quantise_priority(o.p, qp, &c);
  }
}

// --------------------------------------------------------------------------------------------
// row copies: payload into the ring (add) and out of it (gather)
// --------------------------------------------------------------------------------------------
// Row i of the source / destination is found through a RowMap: an index array (gather by slot),
// a ring position read from device memory (keys base+i, slot = key mod ring), or the identity.
struct RowMap {
  const uint32_t *index;     // row = index[i]
  const uint64_t *ring_key;  // row = (*ring_key + i) mod ring; with index: row = index[(*ring_key + i) mod ring]
  uint64_t ring;
};

__device__ __forceinline__ uint64_t map_row(const RowMap &m, uint64_t i)
{
  if (m.index) return m.ring_key ? m.index[(*m.ring_key + i) % m.ring] : m.index[i];
  if (m.ring_key) return (*m.ring_key + i) % m.ring;
  return i;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// --------------------------------------------------------------------------------------------
// Observations stored through the block codec (Section 4.1: observations are kept compressed in the
// replay memory): shape of an encoded row, and how a lane fetches a 16-byte piece of the raw row
// out of it.  The format is described in codec.inc.hpp: every part has a fixed place, so the three
// loads below depend on nothing but the row's address.
// --------------------------------------------------------------------------------------------
struct CodecShape {
  uint32_t raw_bytes, nb, mask_words;  // raw_bytes == 0: no codec
  uint32_t flat_off, image_off;        // M, M + V
  uint64_t stride;                     // M + V + 64 nb
};

__host__ __device__ inline CodecShape codec_shape(uint32_t raw_bytes)
{
  CodecShape c{};
  c.raw_bytes = raw_bytes;
  c.nb = raw_bytes / 64;
  c.mask_words = (c.nb + 63) / 64;
  const uint32_t M = (8 * c.mask_words + 15) / 16 * 16, V = (c.nb + 15) / 16 * 16;
  c.flat_off = M;
  c.image_off = M + V;
  c.stride = (uint64_t)c.image_off + 64ull * c.nb;
  return c;
}

// What a lane has asked for of piece v (16 bytes) of the raw row: the piece as the image holds it, its
// block's byte, and the word of the mask that says which of the two counts.
struct CodecFetched {
  u32x4 data;
  uint64_t word;
  uint32_t byte, bit;
};

// All three at once (for paths bound by latency: nothing waits for the mask).  v < raw_bytes / 16.
__device__ __forceinline__ CodecFetched codec_fetch_all(const uint8_t *e, const CodecShape &c, uint32_t v)
{
  CodecFetched f;
  const uint32_t b = v / 4;
  f.data = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(e + c.image_off) + v);
  f.byte = e[c.flat_off + b];
  f.word = reinterpret_cast<const uint64_t *>(e)[b / 64];
  f.bit = b & 63;
  return f;
}

// The same for a whole wave whose 64 lanes hold 64 consecutive pieces starting at a multiple of 64 (16
// blocks: one word of the mask, 16 consecutive block bytes): the word and the bytes come through the
// scalar data cache (read only), which keeps them out of the queue of the vector memory pipeline, where
// they would wait behind the row loads of the same compute unit.  e must be 16-byte aligned.
__device__ __forceinline__ void codec_fetch_wave_scalars(const uint8_t *e, const CodecShape &c, uint32_t v_first,
                                                         uint64_t *word, u32x4 *bytes)
{
  const uint64_t pe = (uint64_t)(uintptr_t)e;
  // (the builtin returns a signed int: without the casts the low half would be sign-extended)
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(pe >> 32));
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)pe);
  const uint64_t base = ((uint64_t)hi << 32) | (uint64_t)lo;
  const uint32_t vf = (uint32_t)__builtin_amdgcn_readfirstlane((int)v_first);
  const uint64_t p_word = base + 8ull * (vf >> 8);
  const uint64_t p_bytes = base + c.flat_off + vf / 4;
  uint64_t w;
  u32x4 b;
  asm volatile("s_load_dwordx2 %0, %2, 0x0\n\ts_load_dwordx4 %1, %3, 0x0\n\ts_waitcnt lgkmcnt(0)"
               : "=&s"(w), "=&s"(b)
               : "s"(p_word), "s"(p_bytes)
               : "memory");
  *word = w;
  *bytes = b;
}

// The byte of the block of lane `lane`'s piece out of the 16 bytes fetched above.
__device__ __forceinline__ uint32_t codec_wave_byte(const u32x4 &bytes, uint32_t lane)
{
  const uint32_t i = lane / 4;  // block within the wave
  const uint32_t dw = i < 4 ? bytes.x : i < 8 ? bytes.y : i < 12 ? bytes.z : bytes.w;
  return (dw >> (8 * (i & 3))) & 0xffu;
}

__device__ __forceinline__ u32x4 codec_piece(const CodecFetched &f)
{
  const uint32_t x = f.byte * 0x01010101u;
  return (f.word >> f.bit & 1) ? f.data : u32x4{x, x, x, x};
}

// A learner batch (m <= blockDim) handled by one workgroup: duplicates are resolved in an LDS hash
// table keyed by slot (the highest position wins), so no pass over global memory is needed for
// it, and the old mass is fetched while the table is being filled.
constexpr uint32_t kDedupeSlots = 2048;  // >= 2 * 1024 pairs: linear probing stays short

// Learner-side ComputePriorities (Algorithm 2) fused into the write-back: the new priority of a
// sampled transition is recomputed from the partial return and accumulated discount stored with it
// (Appendix "Implementation", "Adding Data") and the Q-values the learner has just evaluated,
//   | ret + gacc * q_target_next[argmax_a q_online_next[a]] - q_taken |     (Section 3.1 target),
// in the same fp32 order as the actor-side kernel.  q_taken == null: priorities are given.
struct QSource {
  const float *q_taken;        // [m]   q(S_t, A_t) of the online network
  const float *q_online_next;  // [m,A] q(S_{t+n}, .) of the online network
  const float *q_target_next;  // [m,A] q(S_{t+n}, .) of the target network
  uint32_t A;
  const float *ret, *gacc;     // columns of the payload ring
  float *prio_out;             // [m] or null: the priorities that were computed (0 for skipped pairs)
};

__device__ __forceinline__ float td_priority(const QSource &qs, uint32_t i, uint64_t slot)
{
  const float *row = qs.q_online_next + (uint64_t)i * qs.A;
  uint32_t best = 0;
  float vbest = row[0];
  for (uint32_t a = 1; a < qs.A; ++a) {
    const float v = row[a];
    if (v > vbest) {
      vbest = v;
      best = a;
    }
  }
  const float boot = qs.q_target_next[(uint64_t)i * qs.A + best];
  const float target = __builtin_fmaf(qs.gacc[slot], boot, qs.ret[slot]);
  return __builtin_fabsf(target - qs.q_taken[i]);
}

struct UpdateArgs {
  TreeView tv;
  DeviceState *st;
  uint32_t m;
  const uint64_t *key;
  const float *prio;
  QuantParams qp;
  // Set by callers that draw a batch and write its priorities back with nothing touching the tree
  // in between: pair i is known to be valid, to live in slot_hint[i] and to weigh mass_hint[i],
  // which saves the two dependent loads key -> slot -> mass.
  const uint32_t *slot_hint;
  const uint64_t *mass_hint;
  QSource qs;
};

// What one lane holds of its pair between the two halves below.
struct UpdateLane {
  uint64_t key, old;
  uint32_t slot;
  float prio;
  uint64_t head, tail;
};

// First half: only loads, so that a caller can put other memory work behind them.
__device__ __forceinline__ UpdateLane update_batch_load(const UpdateArgs &ua)
{
  UpdateLane u{0, 0, 0, 0.0f, 0, ~0ull};
  const uint32_t i = threadIdx.x;
  if (i < ua.m) {
    if (!ua.qs.q_taken) u.prio = ua.prio[i];
    if (ua.slot_hint) {
      u.slot = ua.slot_hint[i];
      u.old = ua.mass_hint[i];
    } else {
      u.key = ua.key[i];
    }
  }
  if (!ua.slot_hint) {
    u.head = ua.st->head;
    u.tail = ua.st->tail;
  }
  return u;
}

// Second half.  h_slot, h_pos: LDS, kDedupeSlots words each.  Called by every thread of the workgroup.
__device__ __forceinline__ void update_batch_apply(const UpdateArgs &ua, UpdateLane u, uint32_t *h_slot,
                                                   uint32_t *h_pos)
{
  const TreeView &tv = ua.tv;
  const uint32_t i = threadIdx.x;
  for (uint32_t t = i; t < kDedupeSlots; t += blockDim.x) {
    h_slot[t] = 0xffffffffu;  // no slot has this number: max_slots <= 2^31
    h_pos[t] = 0;
  }
  __syncthreads();
  const bool valid = i < ua.m && u.key >= u.head && u.key < u.tail;
  const bool stale = i < ua.m && !valid;
  bool clamped = false;
  uint32_t slot = u.slot, h = 0;
  uint64_t q = 0, old = u.old;
  if (valid) {
    if (!ua.slot_hint) {
      slot = (uint32_t)(u.key % tv.P);
      old = tv.level[0][slot];  // in flight during the dedupe
    }
    h = (slot * 2654435761u) >> 21;  // top 11 bits
    for (;;) {
      const uint32_t prev = atomicCAS(&h_slot[h], 0xffffffffu, slot);
      if (prev == 0xffffffffu || prev == slot) break;
      h = (h + 1) & (kDedupeSlots - 1);
    }
    atomicMax(&h_pos[h], i + 1);
    const float p = ua.qs.q_taken ? td_priority(ua.qs, i, slot) : u.prio;
    q = quantise_priority(p, ua.qp, &clamped);
    if (ua.qs.q_taken && ua.qs.prio_out) ua.qs.prio_out[i] = p;
  }
  if (stale && ua.qs.q_taken && ua.qs.prio_out) ua.qs.prio_out[i] = 0.0f;
  __syncthreads();
  if (valid && h_pos[h] == i + 1) {
    tv.level[0][slot] = q;
    add_to_ancestors(tv, slot, q - old);
  }
  const uint64_t ns = __popcll(__ballot(stale)), nc = __popcll(__ballot(clamped));
  if (lane_id() == 0) {
    if (ns) atomic_add_u64(&ua.st->n_stale, ns);
    if (nc) atomic_add_u64(&ua.st->n_clamped, nc);
  }
}

__device__ __forceinline__ void update_batch_in_block(const UpdateArgs &ua, uint32_t *h_slot, uint32_t *h_pos)
{
  update_batch_apply(ua, update_batch_load(ua), h_slot, h_pos);
}

__global__ __launch_bounds__(1024) void update_small_kernel(UpdateArgs ua)
{
  __shared__ uint32_t h_slot[kDedupeSlots];
  __shared__ uint32_t h_pos[kDedupeSlots];
  update_batch_in_block(ua, h_slot, h_pos);
}

// Importance-sampling weights of one batch of k samples, by one workgroup:
//   (N P_i)^-beta / max_j (N P_j)^-beta  ==  (min_j mass_j / mass_i)^beta,   P_i = mass_i / total.
// `red` is LDS scratch of blockDim/64 words.
struct WeightArgs {
  const uint64_t *mass;  // [nb,k], written by the descent kernel that ran before
  float *weight_out;     // [nb,k]; null: no weights wanted
  uint32_t k;
  float beta;
};

// part, nparts: the workgroup writes the weights of samples [part * k / nparts ...) of batch b only
// (every part still finds the minimum over the whole batch).
__device__ __forceinline__ void batch_weights(const WeightArgs &wa, uint32_t b, uint64_t *red, uint32_t part = 0,
                                              uint32_t nparts = 1)
{
  const uint32_t tid = threadIdx.x, nthr = blockDim.x, nwave = nthr / kWave;
  const uint64_t *bm = wa.mass + (uint64_t)b * wa.k;
  uint64_t mn = ~0ull;
  for (uint32_t i = tid; i < wa.k; i += nthr) mn = bm[i] < mn ? bm[i] : mn;
  mn = wave_min(mn);
  if (lane_id() == 0) red[tid / kWave] = mn;
  __syncthreads();
  for (uint32_t w = 0; w < nwave; ++w) mn = red[w] < mn ? red[w] : mn;
  // fp32 with the library's own power routine (relative error below 1e-6 here): a double-precision
  // pow would cost this kernel 70 registers per lane and half of its occupancy
  const float fmn = (float)mn;
  const uint32_t per = (wa.k + nparts - 1) / nparts;
  const uint32_t lo = min(part * per, wa.k), hi = min(lo + per, wa.k);
  for (uint32_t i = lo + tid; i < hi; i += nthr)
    wa.weight_out[(uint64_t)b * wa.k + i] = pow_fixed_sequence(fmn / (float)bm[i], wa.beta);
}

constexpr int kLongCopyThreads = 1024;  // one workgroup of 16 waves per 28 KB frame stack
constexpr int kLongCopyUnroll = 2;      // 1024 lanes * 2 * 16 B = 32 KB per workgroup

// grid: (batches, parts of a batch)
__global__ __launch_bounds__(256) void batch_weights_kernel(WeightArgs wa)
{
  __shared__ uint64_t red[256 / kWave];
  batch_weights(wa, blockIdx.x, red, blockIdx.y, gridDim.y);
}

// Long rows (frame stacks): a workgroup copies kUnroll * blockDim consecutive vectors of one row,
// all loads issued before the first store so that a whole row can be in flight.
// Some workgroups can take a side job that touches none of the copied bytes (its loads issued
// behind the row loads, its work done once the row has been stored), so that a learner step
// needs no launch of its own for it and the grid stays at one workgroup per row (the chip holds
// exactly 512 workgroups of 1024 lanes at a time, the size of a learner batch):
//   kUpdate = 1  workgroup 0 writes a batch of (key, priority) pairs back into the sum tree;
//   kUpdate = 2  the rows are a freshly drawn batch whose own priorities are written back: the
//                workgroup of row i handles pair i (slot and old mass are known from the draw;
//                it wins unless a later sample drew the same slot), which spreads the atomics
//                over the whole chip;
//   kWeights     the first weight_blocks workgroups (after workgroup 0 if kUpdate = 1) write one
//                batch's importance weights each.
template <typename Vec, int kUnroll, bool kWeights, int kUpdate>
__global__ __launch_bounds__(kLongCopyThreads) void copy_rows_long_kernel(const uint8_t *__restrict__ src, RowMap smap,
                                                                          uint8_t *__restrict__ dst, RowMap dmap,
                                                                          uint32_t vecs_per_row, uint32_t chunks_per_row,
                                                                          uint64_t row_bytes, WeightArgs wa,
                                                                          uint32_t weight_blocks, UpdateArgs ua)
{
  const uint32_t blk = blockIdx.x;
  const uint32_t row = blk / chunks_per_row;
  const uint32_t chunk = blk - row * chunks_per_row;
  const Vec *s = reinterpret_cast<const Vec *>(src + map_row(smap, row) * row_bytes);
  Vec *d = reinterpret_cast<Vec *>(dst + map_row(dmap, row) * row_bytes);
  const uint32_t v0 = chunk * (kUnroll * blockDim.x) + threadIdx.x;
  Vec tmp[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t v = v0 + u * blockDim.x;
    if (v < vecs_per_row) tmp[u] = __builtin_nontemporal_load(s + v);
  }
  // side-job loads go out behind the row loads; the row is stored as soon as it has arrived
  UpdateLane ul{};
  if (kUpdate == 1 && blk == 0) ul = update_batch_load(ua);
  const bool writer = kUpdate == 2 && chunk == 0 && threadIdx.x < kWave;  // first wave of the row's first workgroup
  uint32_t my_slot = 0;
  bool later_dup = false;
  if (writer) {
    my_slot = ua.slot_hint[row];
    for (uint32_t j = row + 1 + threadIdx.x; j < ua.m; j += kWave) later_dup |= ua.slot_hint[j] == my_slot;
    if (threadIdx.x == 0) {
      ul.old = ua.mass_hint[row];
      ul.prio = ua.prio[row];
    }
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t v = v0 + u * blockDim.x;
    if (v < vecs_per_row) __builtin_nontemporal_store(tmp[u], d + v);
  }
  if (kUpdate == 1) {
    __shared__ uint32_t h_slot[kDedupeSlots];
    __shared__ uint32_t h_pos[kDedupeSlots];
    if (blk == 0) update_batch_apply(ua, ul, h_slot, h_pos);
  }
  if (writer) {
    const bool loses = __ballot(later_dup) != 0;  // last occurrence wins, as in a sequential loop
    if (threadIdx.x == 0) {
      bool clamped;
      const uint64_t q = quantise_priority(ul.prio, ua.qp, &clamped);  // counted for losers too
      if (!loses) {
        ua.tv.level[0][my_slot] = q;
        add_to_ancestors(ua.tv, my_slot, q - ul.old);
      }
      if (clamped) atomic_add_u64(&ua.st->n_clamped, 1);
    }
  }
  if (kWeights) {
    __shared__ uint64_t red[kLongCopyThreads / kWave];
    const uint32_t first = kUpdate == 1 ? 1 : 0;
    if (blk >= first && blk < first + weight_blocks) batch_weights(wa, blk - first, red);
  }
}

// Long rows from a dense source into the ring (the payload of an add round: row i of the source is its
// i-th run of row_bytes bytes): the copy is cut into runs of kUnroll * blockDim vectors whatever the row
// boundaries, so that every lane carries a full load (a 28,224-byte row fills only 86 % of a workgroup's
// 2048 vector slots); each vector finds its destination row by one division.  (For gathers, whose source
// rows are looked up per row, one workgroup per row is faster.)
template <typename Vec, int kUnroll>
__global__ __launch_bounds__(kLongCopyThreads) void copy_rows_dense_kernel(const uint8_t *__restrict__ src,
                                                                           uint8_t *__restrict__ dst, RowMap dmap,
                                                                           uint32_t vecs_per_row, uint64_t row_bytes,
                                                                           uint32_t total_vecs)
{
  const uint32_t f0 = blockIdx.x * (kUnroll * blockDim.x) + threadIdx.x;
  const Vec *s = reinterpret_cast<const Vec *>(src);
  Vec tmp[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t f = f0 + u * blockDim.x;
    if (f < total_vecs) tmp[u] = __builtin_nontemporal_load(s + f);
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t f = f0 + u * blockDim.x;
    if (f < total_vecs) {
      const uint32_t row = f / vecs_per_row, v = f - row * vecs_per_row;
      __builtin_nontemporal_store(tmp[u], reinterpret_cast<Vec *>(dst + map_row(dmap, row) * row_bytes) + v);
    }
  }
}

// Long rows looked up through row maps (gathers), packed the same way: a workgroup's run of
// kUnroll * blockDim vectors touches at most kPackedRows rows, whose source and destination offsets its
// first lanes fetch once.  The first weight_blocks workgroups write one batch's importance weights
// each instead of copying.
constexpr uint32_t kPackedRows = 10;  // rows longer than 256 vectors: 2048 / 257 + 2

template <typename Vec, int kUnroll, bool kWeights>
__global__ __launch_bounds__(kLongCopyThreads) void copy_rows_packed_kernel(const uint8_t *__restrict__ src, RowMap smap,
                                                                            uint8_t *__restrict__ dst, RowMap dmap,
                                                                            uint32_t nrows, uint32_t vecs_per_row,
                                                                            uint64_t row_bytes, uint32_t total_vecs,
                                                                            WeightArgs wa, uint32_t weight_blocks)
{
  if (kWeights && blockIdx.x < weight_blocks) {
    __shared__ uint64_t red[kLongCopyThreads / kWave];
    batch_weights(wa, blockIdx.x, red);
    return;
  }
  __shared__ uint64_t src_off[kPackedRows], dst_off[kPackedRows];
  const uint32_t blk = blockIdx.x - (kWeights ? weight_blocks : 0);
  const uint32_t first = blk * (kUnroll * blockDim.x);
  const uint32_t r0 = first / vecs_per_row;
  if (threadIdx.x < kPackedRows && r0 + threadIdx.x < nrows) {
    src_off[threadIdx.x] = map_row(smap, r0 + threadIdx.x) * row_bytes;
    dst_off[threadIdx.x] = map_row(dmap, r0 + threadIdx.x) * row_bytes;
  }
  __syncthreads();
  Vec tmp[kUnroll];
  uint32_t ri[kUnroll], v[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t f = first + threadIdx.x + u * blockDim.x;
    const uint32_t row = f / vecs_per_row;
    ri[u] = row - r0;
    v[u] = f - row * vecs_per_row;
    if (f < total_vecs) tmp[u] = __builtin_nontemporal_load(reinterpret_cast<const Vec *>(src + src_off[ri[u]]) + v[u]);
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t f = first + threadIdx.x + u * blockDim.x;
    if (f < total_vecs) __builtin_nontemporal_store(tmp[u], reinterpret_cast<Vec *>(dst + dst_off[ri[u]]) + v[u]);
  }
}

// Short rows: 2^lanes_log2 lanes per row, several rows per workgroup.
struct ShortCopyArgs {
  const uint8_t *src;
  RowMap smap;
  uint8_t *dst;
  RowMap dmap;
  uint64_t nrows;
  uint32_t vecs_per_row, lanes_log2;
  uint64_t row_bytes;
};

template <typename Vec>
__device__ __forceinline__ void copy_rows_short_block(const ShortCopyArgs &c, uint32_t blk)
{
  const uint32_t rows_per_block = blockDim.x >> c.lanes_log2;
  const uint64_t row = (uint64_t)blk * rows_per_block + (threadIdx.x >> c.lanes_log2);
  const uint32_t v = threadIdx.x & ((1u << c.lanes_log2) - 1);
  if (row >= c.nrows || v >= c.vecs_per_row) return;
  const Vec *s = reinterpret_cast<const Vec *>(c.src + map_row(c.smap, row) * c.row_bytes);
  Vec *d = reinterpret_cast<Vec *>(c.dst + map_row(c.dmap, row) * c.row_bytes);
  d[v] = s[v];
}

template <typename Vec>
__global__ __launch_bounds__(256) void copy_rows_short_kernel(ShortCopyArgs c)
{
  copy_rows_short_block<Vec>(c, blockIdx.x);
}

// All four payload columns of an add round with short observation rows, in one launch: 2^lanes_log2
// lanes per transition copy its observation, its action bytes, and (first lane) its partial
// return and accumulated discount.  act, ret, gacc may be null.
template <typename Vec>
__global__ __launch_bounds__(256) void add_payload_short_kernel(const uint8_t *__restrict__ obs,
                                                                const uint8_t *__restrict__ act,
                                                                const float *__restrict__ ret,
                                                                const float *__restrict__ gacc,
                                                                uint8_t *__restrict__ obs_ring,
                                                                uint8_t *__restrict__ act_ring,
                                                                float *__restrict__ ret_ring,
                                                                float *__restrict__ gacc_ring, RowMap dmap,
                                                                uint64_t nrows, uint32_t vecs_per_row,
                                                                uint32_t lanes_log2, uint64_t obs_bytes,
                                                                uint32_t act_bytes)
{
  const uint32_t rows_per_block = blockDim.x >> lanes_log2, lanes = 1u << lanes_log2;
  const uint64_t row = (uint64_t)blockIdx.x * rows_per_block + (threadIdx.x >> lanes_log2);
  const uint32_t v = threadIdx.x & (lanes - 1);
  if (row >= nrows) return;
  const uint64_t to = map_row(dmap, row);
  if (v < vecs_per_row)
    reinterpret_cast<Vec *>(obs_ring + to * obs_bytes)[v] = reinterpret_cast<const Vec *>(obs + row * obs_bytes)[v];
  if (act)
    for (uint32_t by = v; by < act_bytes; by += lanes) act_ring[to * act_bytes + by] = act[row * act_bytes + by];
  if (v == 0) {
    if (ret) ret_ring[to] = ret[row];
    if (gacc) gacc_ring[to] = gacc[row];
  }
}

// --------------------------------------------------------------------------------------------
// add: masses of the new keys, and their sums into the upper levels
// --------------------------------------------------------------------------------------------
// both: the second copy of the tree (tv2) is in step with the first and is kept so.
struct AddLeavesArgs {
  TreeView tv, tv2;
  bool both;
  DeviceState *st;
  uint64_t count;
  const float *prio;  // [count]
  QuantParams qp;
};

// Workgroup blk of n_wgs.
__device__ __forceinline__ void add_leaves_block(const AddLeavesArgs &a, uint32_t blk, uint32_t n_wgs)
{
  const uint64_t i = (uint64_t)blk * blockDim.x + threadIdx.x;
  const bool active = i < a.count;
  uint64_t slot = 0, q = 0;
  bool clamped = false;
  if (active) {
    slot = (a.st->tail + i) % a.tv.P;
    q = quantise_priority(a.prio[i], a.qp, &clamped);
    a.tv.level[0][slot] = q;  // the slot was empty (mass 0): the ring is never over-filled
    if (a.both) a.tv2.level[0][slot] = q;
  }
  add_to_ancestors_grouped(a.tv, active, slot, q, a.both ? &a.tv2 : nullptr);
  const uint64_t nc = __popcll(__ballot(clamped));
  if (nc && lane_id() == 0) atomic_add_u64(&a.st->n_clamped, nc);
  advance_state_when_all_done(&a.st->ticket_add, &a.st->tail, a.count, n_wgs);
}

__global__ __launch_bounds__(256) void add_leaves_kernel(AddLeavesArgs a) { add_leaves_block(a, blockIdx.x, gridDim.x); }

// A small add round in one launch (Algorithm 1: ComputePriorities, replay.Add): 2^lanes_log2 lanes
// per transition copy its payload row into the ring; the first of them computes the n-step
// priority, stores the partial return and the accumulated discount, and enters the mass into the
// tree; the last workgroup to finish moves the tail on.  act may be null.
// The masses of a workgroup's transitions are collected in LDS and entered into the upper levels by
// whole waves of 64 neighbouring transitions, so that a node receives one atomic per 64 of them.
constexpr int kAddRoundThreads = 1024;

struct AddRoundArgs {
  NstepArgs ns;
  TreeView tv, tv2;
  bool both;  // tv2 receives the same masses
  DeviceState *st;
  QuantParams qp;
  const uint8_t *obs, *act;  // [S*T, obs_bytes], [S*T, act_bytes] (act may be null)
  uint8_t *obs_ring, *act_ring;
  float *ret_ring, *gacc_ring;
  uint32_t vecs_per_row, lanes_log2;
  uint64_t obs_bytes;
  uint32_t act_bytes;
};

// Workgroup blk of n_wgs of such a round; sh_slot, sh_q: blockDim words of LDS each.
template <typename Vec>
__device__ __forceinline__ void add_round_small_block(const AddRoundArgs &a, uint32_t blk, uint32_t n_wgs,
                                                      uint64_t *sh_slot, uint64_t *sh_q)
{
  const uint32_t rows_per_block = blockDim.x >> a.lanes_log2, lanes = 1u << a.lanes_log2;
  const uint32_t r = threadIdx.x >> a.lanes_log2;  // row of this workgroup
  const uint64_t i = (uint64_t)blk * rows_per_block + r;
  const uint32_t v = threadIdx.x & (lanes - 1);
  const uint64_t count = (uint64_t)a.ns.S * a.ns.T;
  const bool in_range = i < count;
  bool clamped = false;
  if (in_range) {
    const uint64_t slot = (a.st->tail + i) % a.tv.P;
    for (uint32_t vv = v; vv < a.vecs_per_row; vv += lanes)
      reinterpret_cast<Vec *>(a.obs_ring + slot * a.obs_bytes)[vv] =
          reinterpret_cast<const Vec *>(a.obs + i * a.obs_bytes)[vv];
    if (a.act)
      for (uint32_t by = v; by < a.act_bytes; by += lanes)
        a.act_ring[slot * a.act_bytes + by] = a.act[i * a.act_bytes + by];
    if (v == 0) {
      const NstepOut o = nstep_one(a.ns, i);
      a.ret_ring[slot] = o.R;
      a.gacc_ring[slot] = o.G;
      const uint64_t q = quantise_priority(o.p, a.qp, &clamped);
      a.tv.level[0][slot] = q;  // the slot was empty (mass 0): the ring is never over-filled
      if (a.both) a.tv2.level[0][slot] = q;
      sh_slot[r] = slot;
      sh_q[r] = q;
    }
  }
  const uint64_t nc = __popcll(__ballot(clamped));
  if (nc && lane_id() == 0) atomic_add_u64(&a.st->n_clamped, nc);
  __syncthreads();
  if (threadIdx.x < ((rows_per_block + kWave - 1) & ~(uint32_t)(kWave - 1))) {  // whole waves
    const uint32_t e = threadIdx.x;
    const bool active = e < rows_per_block && (uint64_t)blk * rows_per_block + e < count;
    add_to_ancestors_grouped(a.tv, active, active ? sh_slot[e] : 0, active ? sh_q[e] : 0, a.both ? &a.tv2 : nullptr);
  }
  advance_state_when_all_done(&a.st->ticket_add, &a.st->tail, count, n_wgs);
}

template <typename Vec>
__global__ __launch_bounds__(kAddRoundThreads) void add_round_small_kernel(AddRoundArgs a)
{
  __shared__ uint64_t sh_slot[kAddRoundThreads], sh_q[kAddRoundThreads];
  add_round_small_block<Vec>(a, blockIdx.x, gridDim.x, sh_slot, sh_q);
}

// evict: zero the masses of the e oldest keys and take them out of the upper levels
__global__ __launch_bounds__(256) void evict_leaves_kernel(TreeView tv, TreeView tv2, bool both,
                                                           DeviceState *__restrict__ st, uint64_t e)
{
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool active = i < e;
  uint64_t slot = 0, old = 0;
  if (active) {
    slot = (st->head + i) % tv.P;
    old = tv.level[0][slot];
    tv.level[0][slot] = 0;
    if (both) tv2.level[0][slot] = 0;
  }
  add_to_ancestors_grouped(tv, active, slot, 0 - old, both ? &tv2 : nullptr);
  advance_state_when_all_done(&st->ticket_evict, &st->head, e);
}

// --------------------------------------------------------------------------------------------
// update: two passes so that, of several pairs naming one key, the last one wins
// --------------------------------------------------------------------------------------------
// pass 1: every valid pair bids its position for the slot (highest position wins)
struct ClaimArgs {
  uint64_t P;
  DeviceState *st;
  uint32_t m;           // 0: nothing to claim
  const uint64_t *key;
  uint32_t *claim;
};

__device__ __forceinline__ void update_claim_block(const ClaimArgs &c, uint32_t blk)
{
  const uint32_t i = blk * blockDim.x + threadIdx.x;
  bool stale = false;
  if (i < c.m) {
    const uint64_t k = c.key[i];
    if (k >= c.st->head && k < c.st->tail)
      __hip_atomic_fetch_max(c.claim + (k % c.P), i + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      stale = true;
  }
  const uint64_t ns = __popcll(__ballot(stale));
  if (ns && lane_id() == 0) atomic_add_u64(&c.st->n_stale, ns);
}

__global__ __launch_bounds__(256) void update_claim_kernel(ClaimArgs c) { update_claim_block(c, blockIdx.x); }

// Everything that only needs the results of a draw of short rows, in one launch: the gather of the rows,
// the importance weights, and the first pass of a priority update of the drawn keys.  Workgroups
// [0, copy_blocks) copy, the next batches * weight_parts write weights, the rest claim.
template <typename Vec>
__global__ __launch_bounds__(256) void finish_short_kernel(ShortCopyArgs c, uint32_t copy_blocks, WeightArgs wa,
                                                           uint32_t batches, uint32_t weight_parts, ClaimArgs cl)
{
  __shared__ uint64_t red[256 / kWave];
  const uint32_t blk = blockIdx.x, weight_blocks = batches * weight_parts;
  if (blk < copy_blocks) {
    copy_rows_short_block<Vec>(c, blk);
  } else if (blk < copy_blocks + weight_blocks) {
    const uint32_t wb = blk - copy_blocks;
    batch_weights(wa, wb / weight_parts, red, wb % weight_parts, weight_parts);
  } else {
    update_claim_block(cl, blk - copy_blocks - weight_blocks);
  }
}

__global__ __launch_bounds__(256) void update_apply_kernel(TreeView tv, DeviceState *__restrict__ st, uint32_t m,
                                                           const uint64_t *__restrict__ key,
                                                           const float *__restrict__ prio, QuantParams qp,
                                                           uint32_t *__restrict__ claim, QSource qs)
{
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  bool clamped = false;
  if (i < m) {
    const uint64_t k = key[i];
    if (k >= st->head && k < st->tail) {
      const uint64_t slot = k % tv.P;
      const float p = qs.q_taken ? td_priority(qs, i, slot) : prio[i];
      if (qs.q_taken && qs.prio_out) qs.prio_out[i] = p;
      const uint64_t q = quantise_priority(p, qp, &clamped);
      if (claim[slot] == i + 1) {
        const uint64_t old = tv.level[0][slot];
        tv.level[0][slot] = q;
        add_to_ancestors(tv, slot, q - old);
        claim[slot] = 0;
      }
    } else if (qs.q_taken && qs.prio_out) {
      qs.prio_out[i] = 0.0f;
    }
  }
  const uint64_t nc = __popcll(__ballot(clamped));
  if (nc && lane_id() == 0) atomic_add_u64(&st->n_clamped, nc);
}

// --------------------------------------------------------------------------------------------
// sample: stratified descent, one wavefront per sample.  The importance weights need the
// smallest mass of a whole batch; they are written by the kernel that runs next (the gather,
// or batch_weights_kernel), so this one needs no fence or counter between workgroups.
// --------------------------------------------------------------------------------------------
struct SampleArgs {
  TreeView tv;
  const DeviceState *st;
  uint32_t k;                // samples per batch
  const uint64_t *k_dev;     // not null: the number of samples is read here, on the device (waves beyond it idle)
  const uint32_t *gen;       // not null: keys are (generation of the slot << 32) | slot instead of ring keys
  const uint64_t *rnd;       // [nb,k]
  uint64_t *key_out;         // [nb,k] or null
  uint32_t *slot_out;        // [nb,k]
  uint64_t *mass;            // [nb,k]: mass of each drawn transition, for the weights
  // small payload columns, gathered here; the observation rows are copied by copy_rows_*
  const uint8_t *act;
  uint32_t act_bytes;
  const float *ret, *gacc;
  uint8_t *act_out;
  float *ret_out, *gacc_out;
  // not null (one batch only): the new priorities of the batch being drawn; their mass differences
};

// Turns pre[0, n_top) (LDS, the top level's masses, complete and visible) into exclusive prefix sums in
// place and returns their total.  wave_total: blockDim/64 words of LDS.  Called by every thread
// of the workgroup; ends with a barrier.
__device__ __forceinline__ uint64_t top_prefix_sums(uint64_t *pre, uint64_t *wave_total, uint32_t n_top)
{
  const uint32_t tid = threadIdx.x, nthr = blockDim.x, nwave = nthr / kWave, wave = tid / kWave;
  const uint32_t per = (n_top + nthr - 1) / nthr;
  const uint32_t lo = min(tid * per, n_top), hi = min(lo + per, n_top);
  uint64_t mine = 0;
  for (uint32_t i = lo; i < hi; ++i) mine += pre[i];
  const uint64_t incl = wave_inclusive_scan(mine);
  if (lane_id() == kWave - 1) wave_total[wave] = incl;
  __syncthreads();
  uint64_t before = 0, total = 0;
  for (uint32_t w = 0; w < nwave; ++w) {
    const uint64_t t = wave_total[w];
    if (w < wave) before += t;
    total += t;
  }
  uint64_t run = before + incl - mine;
  for (uint32_t i = lo; i < hi; ++i) {
    const uint64_t v = pre[i];
    pre[i] = run;
    run += v;
  }
  __syncthreads();
  return total;
}

struct Drawn {
  uint64_t slot, mass;
  uint64_t x;  // where in the slot's interval of cumulative mass the point fell: 0 <= x < mass
};

// Exact floor(n / d) for any n by a multiplication, for a divisor that the host knows at launch time
// (the 64-bit quotient of a sum of masses by the batch size is otherwise a long software division on the
// drawing wave's critical path).  Granlund and Montgomery's unsigned division by an invariant integer:
// L = ceil(log2 d), mul = floor(2^64 (2^L - d) / d) + 1, sh1 = min(L, 1), sh2 = max(L - 1, 0).
struct FastDiv {
  uint64_t mul;
  uint32_t sh1, sh2;
};

__device__ __forceinline__ uint64_t fast_div(uint64_t n, const FastDiv &d)
{
  const uint64_t t = __umul64hi(d.mul, n);
  return (t + ((n - t) >> d.sh1)) >> d.sh2;
}

// Where a walk stands after the top level: node idx of that level, whose interval of cumulative mass
// holds the point; x is the point's offset inside the interval, mass the node's mass.
struct TopHit {
  uint64_t idx, x, mass;
};

// Top level from LDS: `pre` holds its exclusive prefix sums; largest i with pre[i] <= x, by two rounds of
// 64-way comparison.  Called by all 64 lanes.
__device__ __forceinline__ TopHit top_search_lds(const uint64_t *pre, uint32_t n_top, uint64_t total, uint64_t x)
{
  const int lane = lane_id();
  const uint32_t stride = (n_top + kWave - 1) / kWave;
  const uint32_t p0 = lane * stride;
  uint32_t cnt = __popcll(__ballot(p0 < n_top && pre[p0] <= x));
  const uint32_t base = (cnt - 1) * stride;  // pre[0] = 0 <= x, so cnt >= 1
  cnt = 0;
  for (uint32_t off = 0; off < stride; off += kWave) {
    const uint32_t p1 = base + off + lane;
    cnt += __popcll(__ballot(off + lane < stride && p1 < n_top && pre[p1] <= x));
  }
  const uint64_t idx = base + cnt - 1;
  const uint64_t mass = ((idx + 1 < n_top) ? pre[idx + 1] : total) - pre[idx];
  return TopHit{idx, x - pre[idx], mass};
}

// Top level of at most 512 nodes from registers: lane l holds the masses v[0..8) of nodes 8l .. 8l+7 (zero
// beyond the level) and lane_before, the sum of all nodes before them.  The same node as top_search_lds
// finds (the last one whose prefix sum is <= x), without a round trip through LDS: the lane by one
// ballot, the node inside the lane by eight comparisons that every lane makes for itself, the winner's
// values by lane reads.  Called by all 64 lanes.
__device__ __forceinline__ uint32_t read_lane_u32(uint32_t v, uint32_t l)
{
  return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l);
}
__device__ __forceinline__ uint64_t read_lane_u64(uint64_t v, uint32_t l)
{
  return ((uint64_t)read_lane_u32((uint32_t)(v >> 32), l) << 32) | read_lane_u32((uint32_t)v, l);
}
__device__ __forceinline__ TopHit top_search_regs(const uint64_t (&v)[8], uint64_t lane_before, uint64_t x)
{
  const uint32_t l = __popcll(__ballot(lane_before <= x)) - 1;  // lane 0 has lane_before = 0 <= x
  uint64_t p = lane_before, p_hit = lane_before, v_hit = v[0];
  uint32_t t_hit = 0;
#pragma unroll
  for (int t = 1; t < 8; ++t) {
    p += v[t - 1];
    const bool le = p <= x;  // true for the first few t only: the prefix sums do not decrease
    t_hit = le ? t : t_hit;
    p_hit = le ? p : p_hit;
    v_hit = le ? v[t] : v_hit;
  }
  return TopHit{8ull * l + read_lane_u32(t_hit, l), x - read_lane_u64(p_hit, l), read_lane_u64(v_hit, l)};
}

// One wavefront walks from its places in the top level down to the slots whose cumulative-mass intervals
// hold the points: the loads of all samples go out together on every level, so that several draws take
// the time of one.  Called by all 64 lanes.
// between(): called once, when the loads of the first level below the top are on their way (right away if
// the tree has no such level): arithmetic that does not depend on the walk costs nothing there.
template <int kSamples, typename Between>
__device__ __forceinline__ void walk_down(const TreeView &tv, const TopHit (&top)[kSamples], Drawn (&out)[kSamples],
                                          Between between)
{
  const int lane = lane_id();
  // the two lowest levels' addresses are at fixed places of the arguments: fetched with them, not on the way down
  const uint64_t *const low0 = tv.level[0], *const low1 = tv.level[1];
  uint64_t x[kSamples], idx[kSamples], mass[kSamples];
#pragma unroll
  for (int s = 0; s < kSamples; ++s) x[s] = top[s].x, idx[s] = top[s].idx, mass[s] = top[s].mass;
  // 64 children per step, prefix sum across the wave, first child whose running sum exceeds the remainder
  bool called = false;
  for (int l = (int)tv.nlev - 2; l >= 0; --l) {
    const uint64_t *const lv = l == 0 ? low0 : l == 1 ? low1 : tv.level[l];
    uint64_t c[kSamples];
#pragma unroll
    for (int s = 0; s < kSamples; ++s) c[s] = lv[idx[s] * kFanout + lane];
    if (!called) {
      between();
      called = true;
    }
#pragma unroll
    for (int s = 0; s < kSamples; ++s) {
      const uint64_t sc = wave_inclusive_scan(c[s]);
      const uint64_t hit = __ballot(sc > x[s]);
      const int sel = hit ? __ffsll((unsigned long long)hit) - 1 : kWave - 1;
      const uint64_t c_sel = __shfl(c[s], sel, kWave);
      const uint64_t s_sel = __shfl(sc, sel, kWave);
      x[s] -= s_sel - c_sel;
      idx[s] = idx[s] * kFanout + sel;
      mass[s] = c_sel;
    }
  }
  if (!called) between();
#pragma unroll
  for (int s = 0; s < kSamples; ++s) out[s] = Drawn{idx[s], mass[s], x[s]};
}

// The whole descent with the top level in LDS (exclusive prefix sums `pre`).
template <int kSamples, typename Between>
__device__ __forceinline__ void wave_descend(const TreeView &tv, const uint64_t *pre, uint64_t total,
                                             const uint64_t (&x_in)[kSamples], Drawn (&out)[kSamples],
                                             Between between)
{
  TopHit top[kSamples];
#pragma unroll
  for (int s = 0; s < kSamples; ++s) top[s] = top_search_lds(pre, tv.n_top, total, x_in[s]);
  walk_down<kSamples>(tv, top, out, between);
}

template <int kSamples>
__device__ __forceinline__ void wave_descend(const TreeView &tv, const uint64_t *pre, uint64_t total,
                                             const uint64_t (&x_in)[kSamples], Drawn (&out)[kSamples])
{
  wave_descend<kSamples>(tv, pre, total, x_in, out, [] {});
}

// The ring key of a drawn slot: head + its distance from the head's slot around the ring.
// head_slot = head % P.
__device__ __forceinline__ uint64_t ring_key(uint64_t slot, uint64_t head, uint64_t head_slot, uint64_t P)
{
  return head + (slot >= head_slot ? slot - head_slot : slot + P - head_slot);
}

// What a draw writes for sample o (called by all 64 lanes of the wave that drew it).
__device__ __forceinline__ void write_drawn(const SampleArgs &a, uint64_t o, Drawn d, uint64_t head,
                                            uint64_t head_slot)
{
  const TreeView &tv = a.tv;
  const int lane = lane_id();
  const uint64_t slot = d.slot;
  if (lane == 0) {
    a.slot_out[o] = (uint32_t)slot;
    if (a.key_out)
      a.key_out[o] = a.gen ? ((uint64_t)a.gen[slot] << 32) | slot : ring_key(slot, head, head_slot, tv.P);
    a.mass[o] = d.mass;
    if (a.ret_out) a.ret_out[o] = a.ret[slot];
    if (a.gacc_out) a.gacc_out[o] = a.gacc[slot];
  }
  if (a.act_out)
    for (uint32_t by = lane; by < a.act_bytes; by += kWave)
      a.act_out[o * a.act_bytes + by] = a.act[slot * a.act_bytes + by];
}

// Dynamic LDS: n_top uint64 (exclusive prefix sums of the top level) + blockDim/64 words.
__global__ __launch_bounds__(1024) void sample_descent_kernel(SampleArgs a)
{
  extern __shared__ uint64_t lds[];
  const TreeView &tv = a.tv;
  const uint32_t n_top = tv.n_top;
  uint64_t *pre = lds;
  uint64_t *wave_total = lds + n_top;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x, nwave = nthr / kWave;
  const uint32_t wave = tid / kWave;
  const uint32_t b = blockIdx.y;
  const uint32_t j = blockIdx.x * nwave + wave;
  const uint32_t k = a.k_dev ? (uint32_t)*a.k_dev : a.k;
  const uint64_t o = (uint64_t)b * k + j;
  // issued ahead of the LDS work below, which does not depend on them
  const uint64_t u = j < k ? a.rnd[o] : 0;
  const uint64_t head = a.st->head;

  // ---- top level -> LDS, exclusive prefix sums in place
  const uint64_t *top = tv.level[tv.nlev - 1];
  for (uint32_t i = tid; i < n_top; i += nthr) pre[i] = top[i];
  __syncthreads();
  const uint64_t total = top_prefix_sums(pre, wave_total, n_top);

  // ---- one sample per wavefront
  if (j < k) {
    const uint64_t w = total / k;                           // stratum width
    const uint64_t x = (uint64_t)j * w + __umul64hi(u, w);  // point inside stratum j
    const uint64_t xs[1] = {x};
    Drawn drs[1];
    uint64_t head_slot = 0;
    wave_descend<1>(tv, pre, total, xs, drs, [&] { head_slot = head % tv.P; });
    const Drawn dr = drs[0];
    write_drawn(a, o, dr, head, head_slot);
  }
}

// --------------------------------------------------------------------------------------------
// One launch per learner step (Algorithm 2: replay.Sample, replay.SetPriority in strict order):
// the gather of batch i, its importance weights, and the draw of batch i+1 together with the
// write-back of batch i+1's new priorities (which are an argument of the call), so that the next
// launch finds a tree that is up to date.
//
// A draw may not read a tree that other workgroups of the same launch are writing, so the memory
// keeps two copies of the sum tree.  Launch i reads copy R, which holds every write-back up to
// batch i, and writes copy W, which holds those up to batch i-1: workgroup j adds the change of
// pair j of batch i (known from the launch before) and of pair j of batch i+1 (which it has just
// drawn) to W with atomics.  The next launch reads W and writes R: every change is applied twice,
// once to each copy, in consecutive launches.  The first batch of a sequence is drawn by a launch
// of the same kernel that has nothing to gather yet (slot == null, one wave per workgroup), which
// needs both copies equal when it starts.
//
// Within a batch the drawn slots do not decrease (the strata are ordered), so the pairs that
// share a slot are neighbours and the last of them is the one that counts: the wave that draws
// sample j also computes the point of sample j+1 and sees whether it still lies inside the slot's
// interval of cumulative mass.
// --------------------------------------------------------------------------------------------
__device__ __forceinline__ void add_delta(const TreeView &tv, uint32_t slot, uint64_t delta)
{
  if (!delta) return;
  atomic_add_u64(tv.level[0] + slot, delta);
  add_to_ancestors(tv, slot, delta);
}

// Orders the LDS accesses of one wavefront among its lanes (the hardware runs them in order; this
// keeps the compiler from moving them).
__device__ __forceinline__ void wave_lds_sync()
{
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Workgroups of 8 waves, 4 vectors per lane: as fast as 16 waves x 2 when the kernel runs alone, and the
// chip then holds the whole batch in half of its wave slots, which leaves room for the workgroups of
// an add round's payload copy on the other stream (measured: 16.9 instead of 18.4 us per step there).
constexpr int kStepThreads = 512;
constexpr int kStepUnroll = 4;
constexpr uint32_t kStepMaxK = 1024;    // pairs per batch that the fused step handles (size of its scratch rows)

struct StepArgs {
  // gather of batch i: row j of dst = row slot[j] of src; the small columns likewise
  const uint8_t *src;
  uint8_t *dst;
  uint32_t vecs_per_row;  // vectors of sizeof(Vec) bytes
  uint64_t row_bytes;
  const uint8_t *act;
  uint32_t act_bytes;
  const float *ret, *gacc;
  uint8_t *act_out;
  float *ret_out, *gacc_out;
  uint32_t k;             // <= kStepMaxK
  const uint32_t *slot;   // [k] batch i as it was drawn
  const uint64_t *dq;     // [k] its changes: new mass - mass as drawn; null: nothing is written back in this sequence
  TreeView wr;            // the copy that is written
  WeightArgs wa;          // weights of batch i
  SampleArgs next;        // draw of batch i+1 from next.tv, the copy that is read; next.rnd == null: none
  const uint64_t *next_top;  // the top level of next.tv (its address at a fixed place of the arguments)
  FastDiv next_k_div;        // division by next.k
  const float *next_prio; // [k] new priorities of batch i+1 (null: none) ...
  uint64_t *next_dq;      // ... the changes they bring, kept for the next launch
  QuantParams qp;
  DeviceState *st;
  // What the workgroups beyond the first k of the launch carry out (gridDim.x == k: nothing): a small
  // add round (add_round_small_block) or the masses of a round whose payload is in place
  // (add_leaves_block).  Only in a launch that draws nothing: what a round adds to the tree commutes
  // with the write-back of this batch, not with a draw.
  AddRoundArgs add;
  AddLeavesArgs leaves;
  // Rows stored through the block codec (kCodec launches only): row_bytes is then the stride of the
  // encoded rows in src, the rows written to dst are codec.raw_bytes long, and vecs_per_row counts their
  // 16-byte pieces.
  CodecShape codec;
};

enum StepRider { kNoRider = 0, kRoundRides = 1, kLeavesRide = 2 };

typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));

// Waits until every load (and store) that this wave has issued is through.
__device__ __forceinline__ void wait_for_all_loads()
{
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0); the other counters at their maxima (not waited for)
}

// Keeps a wave-uniform value in scalar registers from here on: the compiler would otherwise fetch a
// kernel argument only where it is first used, behind a wait of its own.
template <typename T>
__device__ __forceinline__ void fetch_now(T *p)
{
  asm volatile("" ::"s"(p));
}

// The draw of sample `row` of the next batch by the first wave of a workgroup, with no barrier: the
// top level (eight consecutive nodes per lane and pass of 512, 16-byte loads) into registers, the walk
// down, outputs, and the change that the sample's new priority brings.
// The wave's path through memory is the launch's critical path, so it holds exactly one round trip per
// tree level and as little else as can be:
//  - the top-level loads are the first instructions to go out, the sample's random number, new priority
//    and the ring's head follow them and are used after them (a wave's loads return in the order of issue);
//  - a top level of one pass (kTopChunk == 1: at most 512 nodes) is searched in the registers it was
//    loaded into; larger ones go through LDS as exclusive prefix sums (round_up(n_top, 64) words of 8 bytes);
//  - the stratum width is an exact division by multiplication (StepArgs::next_k_div);
//  - what does not depend on the walk (priority -> mass, head % P, the addresses of everything written at
//    the end) is computed or fetched while the first row of children is on its way.
template <int kTopChunk>
__device__ __forceinline__ void draw_in_first_wave(const StepArgs &a, uint32_t row, uint64_t *pre)
{
  const TreeView &rd = a.next.tv;
  const uint32_t n_top = rd.n_top, lane = lane_id();
  const uint32_t n_top_pad = (n_top + kFanout - 1) & ~(kFanout - 1);  // the level is zero-padded to this in memory
  const bool second = a.next_prio && row + 1 < a.next.k;              // a next sample to compare slots with
  __builtin_amdgcn_s_setprio(2);
  const uint64_t *top = a.next_top;
  constexpr uint32_t kChunkNodes = kTopChunk * 8 * kWave;

  uint64_t v[kTopChunk][8];
  auto issue = [&](uint32_t c0) {
#pragma unroll
    for (int p = 0; p < kTopChunk; ++p) {
      const uint32_t i0 = c0 + p * 8 * kWave + 8 * lane;
#pragma unroll
      for (int t = 0; t < 8; ++t) v[p][t] = 0;
      if (i0 < n_top_pad) {
#pragma unroll
        for (int t = 0; t < 8; t += 2) {
          const u64x2 v2 = *reinterpret_cast<const u64x2 *>(top + i0 + t);
          v[p][t] = v2.x, v[p][t + 1] = v2.y;
        }
      }
    }
  };
  issue(0);
  // no load below is conditional: a branch around a load would make the wave wait for it there
  const uint64_t un0 = a.next.rnd[row], un1 = a.next.rnd[second ? row + 1 : row];
  const float prio_next = *(a.next_prio ? a.next_prio + row : reinterpret_cast<const float *>(a.next.rnd + row));
  const uint64_t head = a.next.st->head;

  // Within a batch the points do not decrease, so the pairs that share a slot are neighbours and the last of
  // them is the one that counts: pair `row` loses to pair row + 1 exactly if the next point still lies in the
  // interval of cumulative mass of the slot drawn here, which needs no second walk: both points are known
  // from the start, and the walk ends with the place of its point inside the slot's interval.
  uint64_t point = 0, next_point = 0;
  TopHit hit[1];
  if constexpr (kTopChunk == 1) {
    // ---- one pass: the level stays in the registers it was loaded into
    uint64_t mine = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) mine += v[0][t];
    const uint64_t incl = wave_inclusive_scan(mine);
    const uint64_t total = read_lane_u64(incl, kWave - 1);
    const uint64_t w = fast_div(total, a.next_k_div);
    point = (uint64_t)row * w + __umul64hi(un0, w), next_point = (uint64_t)(row + 1) * w + __umul64hi(un1, w);
    hit[0] = top_search_regs(v[0], incl - mine, point);
  } else {
    // ---- exclusive prefix sums -> LDS; the loads of kTopChunk passes go out together
    uint64_t carry = 0;
    auto consume = [&](uint32_t c0) {
#pragma unroll
      for (int p = 0; p < kTopChunk; ++p) {
        const uint32_t i0 = c0 + p * 8 * kWave + 8 * lane;
        uint64_t mine = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) mine += v[p][t];
        const uint64_t incl = wave_inclusive_scan(mine);
        uint64_t run = carry + incl - mine;
        if (i0 < n_top_pad) {
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            pre[i0 + t] = run;
            run += v[p][t];
          }
        }
        carry += __shfl(incl, kWave - 1, kWave);
      }
    };
    consume(0);
    for (uint32_t c0 = kChunkNodes; c0 < n_top_pad; c0 += kChunkNodes) {
      issue(c0);
      consume(c0);
    }
    const uint64_t total = carry;
    wave_lds_sync();
    const uint64_t w = fast_div(total, a.next_k_div);
    point = (uint64_t)row * w + __umul64hi(un0, w), next_point = (uint64_t)(row + 1) * w + __umul64hi(un1, w);
    hit[0] = top_search_lds(pre, n_top, total, point);
  }

  bool clamped = false;
  uint64_t q_next = 0, head_slot = 0;
  uint32_t *const slot_out = a.next.slot_out;
  uint64_t *const key_out = a.next.key_out, *const mass_out = a.next.mass, *const dq_out = a.next_dq;
  uint64_t *const wr0 = a.wr.level[0], *const wr1 = a.wr.level[1], *const wr2 = a.wr.level[2];
  const uint32_t wr_nlev = a.wr.nlev;
  auto add_to_written_copy = [&](uint64_t slot, uint64_t delta) {  // one lane
    if (!delta) return;
    atomic_add_u64(wr0 + slot, delta);
    if (wr_nlev > 1) atomic_add_u64(wr1 + (slot >> kFanoutLog2), delta);
    if (wr_nlev > 2) atomic_add_u64(wr2 + (slot >> (2 * kFanoutLog2)), delta);
    uint64_t idx = slot >> (2 * kFanoutLog2);
    for (uint32_t l = 3; l < wr_nlev; ++l) {
      idx >>= kFanoutLog2;
      atomic_add_u64(a.wr.level[l] + idx, delta);
    }
  };
  auto between = [&] {
    fetch_now(slot_out), fetch_now(key_out), fetch_now(mass_out), fetch_now(dq_out);
    fetch_now(wr0), fetch_now(wr1), fetch_now(wr2);
    if (a.next_prio) q_next = quantise_priority(prio_next, a.qp, &clamped);
    head_slot = head % rd.P;
  };
  Drawn dr[1];
  walk_down<1>(rd, hit, dr, between);
  const bool next_has_same_slot = second && next_point - point < dr[0].mass - dr[0].x;
  // Outputs first, atomics last: nothing that the compiler makes wait for an atomic's completion follows them.
  // (The small payload columns of the drawn batch are gathered by the launch that copies its rows.)
  if (lane == 0) {
    const uint64_t slot = dr[0].slot;
    slot_out[row] = (uint32_t)slot;
    if (key_out) key_out[row] = ring_key(slot, head, head_slot, rd.P);
    mass_out[row] = dr[0].mass;
    if (a.next_prio) {
      // the change this pair brings: none if the next pair has the same slot (the later one counts)
      const uint64_t delta = next_has_same_slot ? 0 : q_next - dr[0].mass;
      dq_out[row] = delta;
      add_to_written_copy(slot, delta);
      if (clamped) atomic_add_u64(&a.st->n_clamped, 1);
    }
  }
  __builtin_amdgcn_s_setprio(0);
}

// No barrier anywhere in the first k workgroups (one per row of the batch): their waves run independently.
//   wave 0       draws sample `row` of the next batch and writes its change into the written copy;
//                copies too only when the other waves cannot hold the whole row (its dependent
//                loads would queue behind the row loads)
//   wave 1       lane 0 carries the change of pair `row` of this batch into the written copy;
//                lanes 1, 2 gather ret and gacc of the row
//   wave 2       gathers the action bytes of the row
//   wave 3       in the first ceil(k / 64) workgroups: importance weights of 64 samples
// Dynamic LDS: see draw_in_first_wave.
// kTopChunk: passes of 512 top-level nodes whose loads the drawing wave issues together (1 for tops of at
// most 512 nodes, 2 up to 1024, 4 beyond: more registers, fewer memory round trips).
// kRider: what the workgroups beyond the first k carry (StepArgs::add or ::leaves).
// kCodec: the rows are decoded on their way out (StepArgs::codec; Vec is 16 bytes wide).
template <typename Vec, int kThreads, int kUnroll, int kTopChunk, int kRider, bool kCodec = false>
__global__ __launch_bounds__(kThreads) void learner_step_kernel(StepArgs a)
{
  extern __shared__ uint64_t lds[];
  const uint32_t row = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  if constexpr (kRider == kRoundRides) {
    if (row >= a.k) {
      __shared__ uint64_t sh_slot[kThreads], sh_q[kThreads];
      add_round_small_block<Vec>(a.add, row - a.k, gridDim.x - a.k, sh_slot, sh_q);
      return;
    }
  }
  if constexpr (kRider == kLeavesRide) {
    if (row >= a.k) {
      add_leaves_block(a.leaves, row - a.k, gridDim.x - a.k);
      return;
    }
  }
  const uint32_t wave = tid / kWave, lane = lane_id();
  const bool write_back = a.dq != nullptr, draw = a.next.rnd != nullptr;
  if (!a.slot) {  // the first draw of a sequence (one wave per workgroup): no batch to gather yet
    if (draw && wave == 0) draw_in_first_wave<kTopChunk>(a, row, lds);
    return;
  }
  const uint32_t first = (draw && a.vecs_per_row <= (nthr - kWave) * kUnroll) ? kWave : 0;
  if (draw && wave == 0) {
    draw_in_first_wave<kTopChunk>(a, row, lds);
    if (first) return;
  }
  // The compiler places its waits for memory by counting loads in flight; it can count them only along
  // straight-line code, and where a load sits in a branch, or loads and stores are in flight together, it
  // waits for everything.  As first written this part had the row loads wait for every small load, the
  // weights' eight loads wait for one another, and each of the row's stores wait for the one before it to
  // be acknowledged (read in the kernel's own ISA; the waves with a side job ended 1 - 2 us after the
  // others, and the launch with them).  So: the slot is waited for at once (everything depends on it),
  // no load below sits in a divergent branch (indices are clamped, unused lanes read an address of their
  // own workgroup that is always valid), the row is waited for once, and the side jobs' stores and
  // atomics follow the row's.
  const uint32_t my_slot = a.slot[row];
  wait_for_all_loads();

  // ---- small loads, ahead of the row so that they return ahead of it
  // the change that pair `row` brings (0 if a later pair of the batch has the same slot), carried into the
  // written copy by one lane: behind the row's stores in a launch that draws (its end is set by the drawing
  // wave's own atomics, and ahead of the stores this wave's part of the row would wait for them); as soon as
  // it has arrived in a launch that draws nothing (these atomics are then the last thing to finish)
  const bool carrier = write_back && tid == kWave;
  uint64_t pc_dq = 0;
  if (write_back) pc_dq = a.dq[row];  // by every lane: the same for all, and no address that the whole grid shares
  const bool ret_lane = tid == kWave + 1 && a.ret_out, gacc_lane = tid == kWave + 2 && a.gacc_out;
  const float small = *(ret_lane    ? a.ret + my_slot
                        : gacc_lane ? a.gacc + my_slot
                                    : reinterpret_cast<const float *>(a.slot + row));
  const bool weigher = wave == 3 && a.wa.weight_out && row * kWave < a.k;
  uint8_t act_byte[4] = {0, 0, 0, 0};
  const bool act_early = wave == 2 && a.act_out && a.act_bytes <= 4 * kWave;
  if (act_early) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
      act_byte[t] = a.act[(uint64_t)my_slot * a.act_bytes + min(t * kWave + lane, a.act_bytes - 1)];
  }

  if (!draw) {  // the same for the whole launch: in a launch that draws, nothing here waits for the change
    if (carrier) add_delta(a.wr, my_slot, pc_dq);
  }

  // ---- the row
  const uint32_t copiers = nthr - first;
  const Vec *s = reinterpret_cast<const Vec *>(a.src + (uint64_t)my_slot * a.row_bytes);
  Vec *d = reinterpret_cast<Vec *>(a.dst + (uint64_t)row * (kCodec ? (uint64_t)a.codec.raw_bytes : a.row_bytes));
  const uint32_t v_last = a.vecs_per_row - 1;
  Vec tmp[kUnroll];
  CodecFetched fetched[kCodec ? kUnroll : 1] = {};
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t v = min(tid - first + u * copiers, v_last);
    if constexpr (kCodec) {  // the pieces as the image holds them; mask and block bytes follow below
      fetched[u].data = __builtin_nontemporal_load(
          reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(s) + a.codec.image_off) + v);
    } else {
      tmp[u] = __builtin_nontemporal_load(s + v);
    }
  }
  if constexpr (kCodec) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = tid - first + u * copiers, v_first = v - lane;  // the wave's 64 pieces start at v_first
      if (v_first < a.vecs_per_row) {  // the same for all lanes of the wave
        u32x4 bytes;
        codec_fetch_wave_scalars(reinterpret_cast<const uint8_t *>(s), a.codec, v_first, &fetched[u].word, &bytes);
        fetched[u].byte = codec_wave_byte(bytes, lane);
        fetched[u].bit = (v / 4) & 63;
      }
    }
  }
  // the weights' loads go out behind the row's (ahead of them, the wave's part of the row would leave a
  // round trip or two late): smallest mass of the batch, eight loads per lane in flight
  uint64_t mass_min = ~0ull, mass_mine = 1;
  if (weigher) {
    mass_mine = a.wa.mass[min(row * kWave + lane, a.k - 1)];
    for (uint32_t j0 = 0; j0 < a.k; j0 += 8 * kWave) {
      uint64_t wm[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) wm[t] = a.wa.mass[min(j0 + t * kWave + lane, a.k - 1)];
#pragma unroll
      for (int t = 0; t < 8; ++t) mass_min = wm[t] < mass_min ? wm[t] : mass_min;
    }
  }

  wait_for_all_loads();
  if constexpr (kCodec) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const u32x4 piece = codec_piece(fetched[u]);
      __builtin_memcpy(&tmp[u], &piece, sizeof(Vec));
    }
  }
  // One store at a time per wave (a wave waits for its last store before it issues the next): with a wave's
  // four stores in flight together the launch took 0.3 - 0.8 us longer, and with every piece stored as soon
  // as it had arrived (the row's writes beside the rest of its reads) 0.2 - 0.5 us longer (each measured
  // against this on one box).  Ordinary stores, streaming loads: streaming stores, which such a wave waits
  // for longer, cost 0.4 us per launch; ordinary loads of the rows cost 1.5.
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t v = tid - first + u * copiers;
    if (u > 0 && v - lane < a.vecs_per_row) wait_for_all_loads();  // the same for all lanes of the wave
    if (v < a.vecs_per_row) d[v] = tmp[u];
  }

  // ---- what the side jobs write
  if (carrier && draw) add_delta(a.wr, my_slot, pc_dq);
  if (ret_lane) a.ret_out[row] = small;
  if (gacc_lane) a.gacc_out[row] = small;
  if (act_early) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t by = t * kWave + lane;
      if (by < a.act_bytes) a.act_out[(uint64_t)row * a.act_bytes + by] = act_byte[t];
    }
  }
  if (weigher) {
    const float weight = pow_fixed_sequence((float)wave_min(mass_min) / (float)mass_mine, a.wa.beta);
    if (row * kWave + lane < a.k) a.wa.weight_out[row * kWave + lane] = weight;
  }

  // rows longer than one pass of the workgroup (more than 32 KB, or narrow vectors)
  for (uint32_t base = copiers * kUnroll; base < a.vecs_per_row; base += copiers * kUnroll) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = min(base + tid - first + u * copiers, v_last);
      if constexpr (kCodec) {
        const u32x4 piece = codec_piece(codec_fetch_all(reinterpret_cast<const uint8_t *>(s), a.codec, v));
        __builtin_memcpy(&tmp[u], &piece, sizeof(Vec));
      } else {
        tmp[u] = __builtin_nontemporal_load(s + v);
      }
    }
    wait_for_all_loads();
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t v = base + tid - first + u * copiers;
      if (v < a.vecs_per_row) __builtin_nontemporal_store(tmp[u], d + v);
    }
  }
  if (wave == 2 && a.act_out && !act_early)  // long action rows: after the row, which they would hold up
    for (uint32_t by = lane; by < a.act_bytes; by += kWave)
      a.act_out[(uint64_t)row * a.act_bytes + by] = a.act[(uint64_t)my_slot * a.act_bytes + by];
}

// dst[i] = src[i]: brings the second copy of the tree up to date
__global__ __launch_bounds__(256) void copy_words_kernel(uint64_t *__restrict__ dst, const uint64_t *__restrict__ src,
                                                         uint64_t n)
{
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// zero fill (hipMemset is avoided so that the library's launches stay replayable)
__global__ __launch_bounds__(256) void fill_zero_kernel(uint64_t *p, uint64_t n)
{
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
    p[i] = 0;
}

}  // namespace apex
