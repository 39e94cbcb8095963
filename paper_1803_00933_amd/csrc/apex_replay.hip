// Host side of the C ABI declared in include/apex_replay.h: argument checks, host mirror of
// head/tail, and the kernel launches.  Every entry point only enqueues work on the caller's
// stream; nothing here allocates device memory.
#include "apex_replay.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <new>
#include <vector>

#include "kernels.hpp"

using namespace apex;

// Scratch of apex_replay_sample_noalloc: the masses of the drawn transitions between the descent
// and the weights.  One copy per GPU, held until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress: the device address it yields (static_scratch_ptr) is what goes
// into kernel arguments.
static __device__ __align__(256) uint64_t scratch[APEX_NOALLOC_MAX_SAMPLES];

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_failed(hipError_t e)
{
  if (e == hipSuccess) return false;
  g_last_hip_error = (int)e;
  return true;
}

#define APEX_HIP(call)                         \
  do {                                         \
    if (hip_failed((call))) return APEX_ERR_HIP; \
  } while (0)

// The device address of `scratch` on the GPU that is current in the calling thread: looked up once per
// device (each GPU holds its own copy of the array at its own address) and kept.  Null, with the
// error recorded, if the lookup fails.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint64_t *g_scratch_ptr[kMaxDevices] = {};

uint64_t *static_scratch_ptr()
{
  int dev = -1;
  if (hip_failed(hipGetDevice(&dev)) || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hip_failed(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return nullptr;
    g_scratch_ptr[dev] = static_cast<uint64_t *>(ptr);
  }
  return g_scratch_ptr[dev];
}

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
inline uint32_t blocks_for(uint64_t n, uint32_t per) { return (uint32_t)((n + per - 1) / per); }

uint32_t ceil_log2(uint64_t v)
{
  uint32_t l = 0;
  while ((1ull << l) < v) ++l;
  return l;
}

uint64_t qmax_for(uint64_t max_slots) { return max_slots ? 1ull << (62 - ceil_log2(max_slots)) : 1ull << 62; }

constexpr uint32_t kStepSets = 64;  // buffer sets a sequence of fused steps can cycle through

struct Geometry {
  uint64_t obs_off, act_off, ret_off, gacc_off, storage_bytes;
  uint32_t nlev;
  uint64_t level_off[kMaxLevels], level_size[kMaxLevels], tree_words;
  // scratch: DeviceState | mass | claim | new masses of the batches of fused steps
  uint64_t state_off, mass_off, claim_off, stepq_off, scratch_bytes;
};

int validate(const apex_replay_config_t *c)
{
  if (!c) return APEX_ERR_INVALID_ARG;
  if (c->capacity == 0 || c->max_slots < c->capacity || c->max_slots > (1ull << 31)) return APEX_ERR_INVALID_ARG;
  if (c->obs_bytes == 0 || c->act_bytes == 0 || c->frac_bits > 32 || c->reserved != 0) return APEX_ERR_INVALID_ARG;
  if (!(c->alpha >= -1.0f && c->alpha <= 1.0f) || !(c->eps >= 0.0f) || !(c->eps < 1e30f)) return APEX_ERR_INVALID_ARG;
  return APEX_OK;
}

int geometry(const apex_replay_config_t *c, Geometry *g)
{
  const uint64_t P = c->max_slots;
  g->obs_off = 0;
  g->act_off = g->obs_off + round_up(P * c->obs_bytes, 256);
  g->ret_off = g->act_off + round_up(P * c->act_bytes, 256);
  g->gacc_off = g->ret_off + round_up(P * 4, 256);
  g->storage_bytes = g->gacc_off + round_up(P * 4, 256);

  uint64_t n = P, off = 0;
  uint32_t l = 0;
  for (;;) {
    if (l >= kMaxLevels) return APEX_ERR_INVALID_ARG;
    g->level_off[l] = off;
    g->level_size[l] = n;
    off += round_up(n, kFanout);
    ++l;
    if (n <= kTopMax) break;
    n = (n + kFanout - 1) / kFanout;
  }
  g->nlev = l;
  g->tree_words = off;

  g->state_off = 0;
  g->mass_off = 256;
  g->claim_off = g->mass_off + (uint64_t)APEX_MAX_SAMPLES_PER_CALL * 8;
  g->stepq_off = g->claim_off + round_up(P * 4, 256);
  g->scratch_bytes = g->stepq_off + (uint64_t)kStepSets * kStepMaxK * 8;
  return APEX_OK;
}

}  // namespace

struct apex_replay {
  apex_replay_config_t cfg;
  Geometry geo;
  uint8_t *storage;
  uint64_t *tree;
  uint8_t *scratch;
  uint64_t head, tail;  // host mirror of the device state
  QuantParams qp;
  TreeView tv;
  // Second copy of the tree, behind the first in the tree region: used by sequences of fused learner
  // steps only.  It equals the first while tree_version == second_version; every entry point that
  // changes the first copy moves tree_version on.
  TreeView tv2;
  uint64_t tree_version = 1, second_version = 0;

  DeviceState *state() const { return reinterpret_cast<DeviceState *>(scratch + geo.state_off); }
  uint64_t *mass() const { return reinterpret_cast<uint64_t *>(scratch + geo.mass_off); }
  uint32_t *claim() const { return reinterpret_cast<uint32_t *>(scratch + geo.claim_off); }
  uint64_t *stepq(uint32_t set) const { return reinterpret_cast<uint64_t *>(scratch + geo.stepq_off) + (uint64_t)set * kStepMaxK; }
  uint8_t *obs() const { return storage + geo.obs_off; }
  uint8_t *act() const { return storage + geo.act_off; }
  float *ret() const { return reinterpret_cast<float *>(storage + geo.ret_off); }
  float *gacc() const { return reinterpret_cast<float *>(storage + geo.gacc_off); }
};

namespace {

// Copies nrows rows of row_bytes bytes; picks the widest vector the row size and the base
// addresses allow and the long- or short-row kernel.
// Side jobs a long-row copy can take along in leading workgroups (see copy_rows_long_kernel).
// A field is cleared once a kernel has taken the job on; what is left needs launches of its own.
struct SideJobs {
  WeightArgs wa{nullptr, nullptr, 1, 0.f};  // wa.weight_out != null: importance weights wanted
  UpdateArgs ua{};                          // ua.m != 0: a priority update of at most 1024 pairs
  ClaimArgs claim{};                        // claim.m != 0: first pass of a larger update (short rows only)
};

template <typename Vec>
int launch_copy_t(const uint8_t *src, const RowMap &smap, uint8_t *dst, const RowMap &dmap, uint64_t nrows,
                  uint64_t row_bytes, hipStream_t stream, SideJobs *jobs)
{
  constexpr int kUnroll = kLongCopyUnroll, kThreads = kLongCopyThreads;
  const uint32_t vpr = (uint32_t)(row_bytes / sizeof(Vec));
  if (vpr > 256) {
    const uint32_t cpr = (vpr + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    if (nrows * cpr > 0x7ffffff0ull) return APEX_ERR_TOO_LARGE;
    const uint32_t blocks = (uint32_t)(nrows * cpr);
    bool w = jobs && jobs->wa.weight_out, u = jobs && jobs->ua.m;
    uint32_t nb = w ? (uint32_t)(nrows / jobs->wa.k) : 0;  // one workgroup per batch takes its weights along
    if (blocks < nb + (u ? 1u : 0u)) w = u = false, nb = 0;    // too few workgroups to carry the side jobs
    const WeightArgs wa = w ? jobs->wa : WeightArgs{nullptr, nullptr, 1, 0.f};
    const UpdateArgs ua = u ? jobs->ua : UpdateArgs{};
    const dim3 grid(blocks), block(kThreads);
    if (!jobs && !smap.index && !smap.ring_key && !dmap.index && nrows * vpr < 0xfffff000ull && nrows >= 1024) {
      // dense source, many rows (the payload of an add round): workgroups packed with vectors
      const uint32_t total = (uint32_t)(nrows * vpr);
      copy_rows_dense_kernel<Vec, kUnroll><<<dim3(blocks_for(total, kThreads * kUnroll)), block, 0, stream>>>(
          src, dst, dmap, vpr, row_bytes, total);
      return hip_failed(hipGetLastError()) ? APEX_ERR_HIP : APEX_OK;
    }
    if (!u && vpr <= kThreads * kUnroll / 2 && nrows * vpr < 0xfffff000ull && nrows < 0xffffffffull) {
      // rows that would fill at most half of a workgroup (4 to 16 KB), no write-back riding along:
      // workgroups packed with vectors.  (For longer rows one workgroup per row measured a little faster.)
      const uint32_t total = (uint32_t)(nrows * vpr);
      const dim3 pgrid(blocks_for(total, kThreads * kUnroll) + nb);
      if (w)
        copy_rows_packed_kernel<Vec, kUnroll, true><<<pgrid, block, 0, stream>>>(src, smap, dst, dmap, (uint32_t)nrows, vpr,
                                                                             row_bytes, total, wa, nb);
      else
        copy_rows_packed_kernel<Vec, kUnroll, false><<<pgrid, block, 0, stream>>>(src, smap, dst, dmap, (uint32_t)nrows,
                                                                              vpr, row_bytes, total, wa, 0);
      if (w) jobs->wa.weight_out = nullptr;
      return hip_failed(hipGetLastError()) ? APEX_ERR_HIP : APEX_OK;
    }
    // a same-batch write-back (slot/mass known) has one pair per copied row: spread it over the rows
    const int umode = !u ? 0 : (ua.slot_hint && ua.m == nrows) ? 2 : 1;
#define APEX_LAUNCH_COPY(W, U) \
  copy_rows_long_kernel<Vec, kUnroll, W, U><<<grid, block, 0, stream>>>(src, smap, dst, dmap, vpr, cpr, row_bytes, wa, nb, ua)
    if (w && umode == 2) APEX_LAUNCH_COPY(true, 2);
    else if (w && umode == 1) APEX_LAUNCH_COPY(true, 1);
    else if (w) APEX_LAUNCH_COPY(true, 0);
    else if (umode == 2) APEX_LAUNCH_COPY(false, 2);
    else if (umode == 1) APEX_LAUNCH_COPY(false, 1);
    else APEX_LAUNCH_COPY(false, 0);
#undef APEX_LAUNCH_COPY
    if (w) jobs->wa.weight_out = nullptr;
    if (u) jobs->ua.m = 0;
  } else {
    uint32_t lanes_log2 = 0;
    while ((1u << lanes_log2) < vpr) ++lanes_log2;
    const uint64_t rows_per_block = 256u >> lanes_log2;
    const uint64_t blocks = (nrows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7ffffff0ull) return APEX_ERR_TOO_LARGE;
    const ShortCopyArgs c{src, smap, dst, dmap, nrows, vpr, lanes_log2, row_bytes};
    const bool w = jobs && jobs->wa.weight_out, cl = jobs && jobs->claim.m;
    if (w || cl) {
      // the importance weights and the claim pass of a large update ride along
      const uint32_t batches = w ? (uint32_t)(nrows / jobs->wa.k) : 0, parts = w ? blocks_for(jobs->wa.k, 512) : 0;
      const uint32_t claim_blocks = cl ? blocks_for(jobs->claim.m, 256) : 0;
      finish_short_kernel<Vec><<<dim3((uint32_t)blocks + batches * parts + claim_blocks), dim3(256), 0, stream>>>(
          c, (uint32_t)blocks, w ? jobs->wa : WeightArgs{nullptr, nullptr, 1, 0.f}, batches, parts,
          cl ? jobs->claim : ClaimArgs{});
      if (w) jobs->wa.weight_out = nullptr;
      if (cl) jobs->claim.m = 0;
    } else {
      copy_rows_short_kernel<Vec><<<dim3((uint32_t)blocks), dim3(256), 0, stream>>>(c);
    }
  }
  return hip_failed(hipGetLastError()) ? APEX_ERR_HIP : APEX_OK;
}

int launch_copy(const void *src, const RowMap &smap, void *dst, const RowMap &dmap, uint64_t nrows, uint64_t row_bytes,
                hipStream_t stream, SideJobs *jobs = nullptr)
{
  if (nrows == 0) return APEX_OK;
  const uintptr_t mis = (uintptr_t)src | (uintptr_t)dst | (uintptr_t)row_bytes;
  const uint8_t *s = static_cast<const uint8_t *>(src);
  uint8_t *d = static_cast<uint8_t *>(dst);
  if ((mis & 15) == 0) return launch_copy_t<u32x4>(s, smap, d, dmap, nrows, row_bytes, stream, jobs);
  if ((mis & 3) == 0) return launch_copy_t<uint32_t>(s, smap, d, dmap, nrows, row_bytes, stream, jobs);
  return launch_copy_t<uint8_t>(s, smap, d, dmap, nrows, row_bytes, stream, jobs);
}


// The constants of fast_div for the divisor d >= 1.
FastDiv make_fast_div(uint32_t d)
{
  if (d == 0) d = 1;
  uint32_t L = 0;
  while (L < 32 && (1ull << L) < d) ++L;
  const unsigned __int128 num = ((unsigned __int128)((1ull << L) - d)) << 64;
  return FastDiv{(uint64_t)(num / d) + 1, L < 1 ? L : 1, L > 0 ? L - 1 : 0};
}

// One launch of the fused learner step (see learner_step_kernel) for vectors of sizeof(Vec) bytes.
// Steps whose rows are decoded on their way out (16-byte vectors; riders: none, or the masses of an add round).
void launch_step_codec(const StepArgs &a, uint32_t n_top, uint32_t wgs, uint32_t threads, size_t lds, int rider,
                       hipStream_t stream)
{
  const dim3 grid(wgs), block(threads);
  if (rider == kLeavesRide)
    learner_step_kernel<u32x4, kStepThreads, kStepUnroll, 1, kLeavesRide, true><<<grid, block, lds, stream>>>(a);
  else if (n_top <= 8 * kWave)
    learner_step_kernel<u32x4, kStepThreads, kStepUnroll, 1, kNoRider, true><<<grid, block, lds, stream>>>(a);
  else if (n_top <= 16 * kWave)
    learner_step_kernel<u32x4, kStepThreads, kStepUnroll, 2, kNoRider, true><<<grid, block, lds, stream>>>(a);
  else
    learner_step_kernel<u32x4, kStepThreads, kStepUnroll, 4, kNoRider, true><<<grid, block, lds, stream>>>(a);
}

template <typename Vec>
void launch_step_t(const StepArgs &a, uint32_t n_top, uint32_t wgs, uint32_t threads, size_t lds, int rider,
                   hipStream_t stream)
{
  const dim3 grid(wgs), block(threads);
  if (rider == kRoundRides)  // further workgroups carry part of an add round (such a launch draws nothing)
    learner_step_kernel<Vec, kStepThreads, kStepUnroll, 1, kRoundRides><<<grid, block, lds, stream>>>(a);
  else if (rider == kLeavesRide)
    learner_step_kernel<Vec, kStepThreads, kStepUnroll, 1, kLeavesRide><<<grid, block, lds, stream>>>(a);
  else if (n_top <= 8 * kWave)
    learner_step_kernel<Vec, kStepThreads, kStepUnroll, 1, kNoRider><<<grid, block, lds, stream>>>(a);
  else if (n_top <= 16 * kWave)
    learner_step_kernel<Vec, kStepThreads, kStepUnroll, 2, kNoRider><<<grid, block, lds, stream>>>(a);
  else
    learner_step_kernel<Vec, kStepThreads, kStepUnroll, 4, kNoRider><<<grid, block, lds, stream>>>(a);
}

// A small add round (observations of at most 1 KB per row) as one launch: n-step priorities, payload,
// masses.  Same effect as apex_nstep_priorities + apex_replay_add.

// Arguments of such a round for workgroups of `threads` lanes and vectors of vector_bytes bytes;
// *blocks: the workgroups it takes.
int add_round_args(const apex_replay *r, const NstepArgs &ns, const void *obs, const void *act, uint32_t vector_bytes,
                   uint32_t threads, bool both, AddRoundArgs *out, uint32_t *blocks)
{
  const uint64_t count = (uint64_t)ns.S * ns.T;
  const uint32_t vpr = r->cfg.obs_bytes / vector_bytes;
  uint32_t lanes_log2 = 0;
  while ((1u << lanes_log2) < vpr && lanes_log2 < 6) ++lanes_log2;  // at most one wave per row
  const uint64_t rows_per_block = threads >> lanes_log2;
  const uint64_t nb = (count + rows_per_block - 1) / rows_per_block;
  if (nb > 0x7ffffff0ull) return APEX_ERR_TOO_LARGE;
  *blocks = (uint32_t)nb;
  *out = AddRoundArgs{ns, r->tv, r->tv2, both, r->state(), r->qp, static_cast<const uint8_t *>(obs),
                      static_cast<const uint8_t *>(act), r->obs(), r->act(), r->ret(), r->gacc(), vpr, lanes_log2,
                      r->cfg.obs_bytes, r->cfg.act_bytes};
  return APEX_OK;
}

// Whether a round can go that way, and the widest vector its rows allow (16, 4 or 1 bytes).
bool add_round_small_fits(const apex_replay *r, const NstepArgs &ns, const void *obs, uint32_t *vector_bytes)
{
  if (!obs || r->cfg.obs_bytes > 1024 || (uint64_t)ns.S * ns.T == 0) return false;
  const uintptr_t mis = (uintptr_t)obs | (uintptr_t)r->obs() | (uintptr_t)r->cfg.obs_bytes;
  *vector_bytes = (mis & 15) == 0 ? 16 : (mis & 3) == 0 ? 4 : 1;
  return true;
}

// Host-side bookkeeping of a round that has been enqueued.
void add_round_published(apex_replay *r, uint64_t count, bool both, uint64_t *first_key_out)
{
  ++r->tree_version;
  if (both) r->second_version = r->tree_version;
  if (first_key_out) *first_key_out = r->tail;
  r->tail += count;
}

// APEX_ERR_NOT_READY - with nothing enqueued - when the rows are too long for the single launch.
int add_round_small(apex_replay *r, const NstepArgs &ns, const void *obs, const void *act, uint64_t *first_key_out,
                    hipStream_t stream)
{
  const uint64_t count = (uint64_t)ns.S * ns.T;
  uint32_t vb = 0, blocks = 0;
  if (!add_round_small_fits(r, ns, obs, &vb)) return APEX_ERR_NOT_READY;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  const bool both = r->second_version == r->tree_version;
  AddRoundArgs a;
  const int rc = add_round_args(r, ns, obs, act, vb, kAddRoundThreads, both, &a, &blocks);
  if (rc != APEX_OK) return rc;
  const dim3 grid(blocks), block(kAddRoundThreads);
  if (vb == 16) add_round_small_kernel<u32x4><<<grid, block, 0, stream>>>(a);
  else if (vb == 4) add_round_small_kernel<uint32_t><<<grid, block, 0, stream>>>(a);
  else add_round_small_kernel<uint8_t><<<grid, block, 0, stream>>>(a);
  APEX_HIP(hipGetLastError());
  add_round_published(r, count, both, first_key_out);
  return APEX_OK;
}

// Short observation rows: the whole payload of an add round in one launch.  APEX_ERR_NOT_READY - with
// nothing enqueued - when the rows are long (the column-by-column copies take over).
struct PayloadRing {
  uint8_t *obs, *act;
  float *ret, *gacc;
  uint64_t obs_bytes;
  uint32_t act_bytes;
};

template <typename Vec>
int add_payload_short_t(const PayloadRing &pr, uint64_t count, const void *obs, const void *act, const float *ret,
                        const float *gacc, const RowMap &to, hipStream_t stream)
{
  const uint32_t vpr = (uint32_t)(pr.obs_bytes / sizeof(Vec));
  if (vpr > 256) return APEX_ERR_NOT_READY;
  uint32_t lanes_log2 = 0;
  while ((1u << lanes_log2) < vpr) ++lanes_log2;
  const uint64_t rows_per_block = 256u >> lanes_log2;
  const uint64_t blocks = (count + rows_per_block - 1) / rows_per_block;
  if (blocks > 0x7fffffffull) return APEX_ERR_TOO_LARGE;
  add_payload_short_kernel<Vec><<<dim3((uint32_t)blocks), dim3(256), 0, stream>>>(
      static_cast<const uint8_t *>(obs), static_cast<const uint8_t *>(act), ret, gacc, pr.obs, pr.act, pr.ret, pr.gacc,
      to, count, vpr, lanes_log2, pr.obs_bytes, pr.act_bytes);
  return hip_failed(hipGetLastError()) ? APEX_ERR_HIP : APEX_OK;
}

int add_payload_short(const PayloadRing &pr, uint64_t count, const void *obs, const void *act, const float *ret,
                      const float *gacc, const RowMap &to, hipStream_t stream)
{
  const uintptr_t mis = (uintptr_t)obs | (uintptr_t)pr.obs | (uintptr_t)pr.obs_bytes;
  if ((mis & 15) == 0) return add_payload_short_t<u32x4>(pr, count, obs, act, ret, gacc, to, stream);
  if ((mis & 3) == 0) return add_payload_short_t<uint32_t>(pr, count, obs, act, ret, gacc, to, stream);
  return add_payload_short_t<uint8_t>(pr, count, obs, act, ret, gacc, to, stream);
}

// The three small columns (action bytes, partial return, accumulated discount) in one launch:
// 2^lanes_log2 lanes per transition share the action bytes.
int add_small_columns(const PayloadRing &pr, uint64_t count, const void *act, const float *ret, const float *gacc,
                      const RowMap &to, hipStream_t stream)
{
  uint32_t lanes_log2 = 0;
  while ((4u << lanes_log2) < pr.act_bytes && lanes_log2 < 6) ++lanes_log2;
  const uint64_t rows_per_block = 256u >> lanes_log2;
  const uint64_t blocks = (count + rows_per_block - 1) / rows_per_block;
  if (blocks > 0x7fffffffull) return APEX_ERR_TOO_LARGE;
  add_payload_short_kernel<uint8_t><<<dim3((uint32_t)blocks), dim3(256), 0, stream>>>(
      nullptr, static_cast<const uint8_t *>(act), ret, gacc, pr.obs, pr.act, pr.ret, pr.gacc, to, count,
      /*vecs_per_row=*/0, lanes_log2, pr.obs_bytes, pr.act_bytes);
  return hip_failed(hipGetLastError()) ? APEX_ERR_HIP : APEX_OK;
}

// obs, act, ret, gacc (any may be null) of `count` transitions into the rows that `to` names.
int add_payload_rows(const PayloadRing &pr, uint64_t count, const void *obs, const void *act, const float *ret,
                     const float *gacc, const RowMap &to, hipStream_t stream)
{
  const RowMap ident{nullptr, nullptr, 0};
  int rc;
  if (obs && (rc = add_payload_short(pr, count, obs, act, ret, gacc, to, stream)) != APEX_ERR_NOT_READY) return rc;
  if (obs && (rc = launch_copy(obs, ident, pr.obs, to, count, pr.obs_bytes, stream)) != APEX_OK) return rc;
  if (act || ret || gacc) return add_small_columns(pr, count, act, ret, gacc, to, stream);
  return APEX_OK;
}

}  // namespace

extern "C" {

int apex_last_hip_error(void) { return g_last_hip_error; }

int apex_replay_workspace_bytes(const apex_replay_config_t *cfg, size_t *storage_bytes, size_t *tree_bytes,
                                size_t *scratch_bytes)
{
  int rc = validate(cfg);
  if (rc != APEX_OK) return rc;
  Geometry g;
  rc = geometry(cfg, &g);
  if (rc != APEX_OK) return rc;
  if (storage_bytes) *storage_bytes = g.storage_bytes;
  if (tree_bytes) *tree_bytes = 2 * g.tree_words * 8;  // two copies, see learner_step_kernel
  if (scratch_bytes) *scratch_bytes = g.scratch_bytes;
  return APEX_OK;
}

int apex_replay_create(const apex_replay_config_t *cfg, void *d_storage, void *d_tree, void *d_scratch,
                       apex_replay_t **out)
{
  int rc = validate(cfg);
  if (rc != APEX_OK) return rc;
  if (!d_storage || !d_tree || !d_scratch || !out) return APEX_ERR_INVALID_ARG;
  if (((uintptr_t)d_storage | (uintptr_t)d_tree | (uintptr_t)d_scratch) & 255) return APEX_ERR_INVALID_ARG;
  apex_replay *r = new (std::nothrow) apex_replay();
  if (!r) return APEX_ERR_INVALID_ARG;
  r->cfg = *cfg;
  rc = geometry(cfg, &r->geo);
  if (rc != APEX_OK) {
    delete r;
    return rc;
  }
  r->storage = static_cast<uint8_t *>(d_storage);
  r->tree = static_cast<uint64_t *>(d_tree);
  r->scratch = static_cast<uint8_t *>(d_scratch);
  r->head = r->tail = 0;
  r->qp = QuantParams{cfg->alpha, cfg->eps, cfg->frac_bits, qmax_for(cfg->max_slots)};
  r->tv.nlev = r->geo.nlev;
  r->tv.n_top = (uint32_t)r->geo.level_size[r->geo.nlev - 1];
  r->tv.P = cfg->max_slots;
  for (uint32_t l = 0; l < kMaxLevels; ++l) r->tv.level[l] = l < r->geo.nlev ? r->tree + r->geo.level_off[l] : nullptr;
  r->tv2 = r->tv;
  for (uint32_t l = 0; l < r->geo.nlev; ++l) r->tv2.level[l] = r->tv.level[l] + r->geo.tree_words;

  // set-up for apex_replay_sample_noalloc on this GPU, so that the call itself has nothing left to look up
  if (!static_scratch_ptr()) {
    delete r;
    return APEX_ERR_HIP;
  }
  fill_zero_kernel<<<dim3(1024), dim3(256), 0, nullptr>>>(r->tree, 2 * r->geo.tree_words);
  fill_zero_kernel<<<dim3(1024), dim3(256), 0, nullptr>>>(reinterpret_cast<uint64_t *>(r->scratch),
                                                          r->geo.scratch_bytes / 8);
  if (hip_failed(hipGetLastError()) || hip_failed(hipDeviceSynchronize())) {
    delete r;
    return APEX_ERR_HIP;
  }
  *out = r;
  return APEX_OK;
}

int apex_replay_destroy(apex_replay_t *r)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  delete r;
  return APEX_OK;
}

int apex_replay_layout(const apex_replay_t *r, apex_replay_layout_t *out)
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
  return APEX_OK;
}

int apex_nstep_priorities(uint32_t S, uint32_t T, uint32_t n, uint32_t A, const float *q_online,
                          const float *q_target, const int32_t *action, const float *reward,
                          const float *discount, float alpha, float eps, uint32_t frac_bits,
                          uint64_t max_slots, float *prio, float *ret, float *gacc, uint64_t *prio_fx,
                          void *hip_stream)
{
  if (!S || !T || !n || !A) return APEX_ERR_INVALID_ARG;
  if (!q_online || !q_target || !action || !reward || !discount || !prio || !ret || !gacc) return APEX_ERR_INVALID_ARG;
  if (frac_bits > 32 || !(alpha >= -1.0f && alpha <= 1.0f) || !(eps >= 0.0f) || max_slots > (1ull << 31))
    return APEX_ERR_INVALID_ARG;
  const uint64_t total = (uint64_t)S * T;
  if (total > 0x7fffffffull * 256 || (uint64_t)T + n > 0xffffffffull) return APEX_ERR_TOO_LARGE;
  const QuantParams qp{alpha, eps, frac_bits, qmax_for(max_slots)};
  const NstepArgs ns{S, T, n, A, q_online, q_target, action, reward, discount};
  nstep_kernel<<<dim3(blocks_for(total, 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(ns, qp, prio, ret,
                                                                                                 gacc, prio_fx);
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

int apex_replay_add_payload(apex_replay_t *r, uint64_t count, const void *obs, const void *act, const float *ret,
                            const float *gacc, void *hip_stream)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  if (count == 0) return APEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const RowMap ring{nullptr, &r->state()->tail, r->cfg.max_slots};
  const PayloadRing pr{r->obs(), r->act(), r->ret(), r->gacc(), r->cfg.obs_bytes, r->cfg.act_bytes};
  return add_payload_rows(pr, count, obs, act, ret, gacc, ring, stream);
}

int apex_replay_add_publish(apex_replay_t *r, uint64_t count, const float *prio, uint64_t *first_key_out,
                            void *hip_stream)
{
  if (!r || (count && !prio)) return APEX_ERR_INVALID_ARG;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  if (count) {
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool both = r->second_version == r->tree_version;
    ++r->tree_version;
    if (both) r->second_version = r->tree_version;
    add_leaves_kernel<<<dim3(blocks_for(count, 256)), dim3(256), 0, stream>>>(
        AddLeavesArgs{r->tv, r->tv2, both, r->state(), count, prio, r->qp});
    APEX_HIP(hipGetLastError());
  }
  if (first_key_out) *first_key_out = r->tail;
  r->tail += count;
  return APEX_OK;
}

int apex_replay_add(apex_replay_t *r, uint64_t count, const void *obs, const void *act, const float *ret,
                    const float *gacc, const float *prio, uint64_t *first_key_out, void *hip_stream)
{
  if (!r || (count && !prio)) return APEX_ERR_INVALID_ARG;
  const int rc = apex_replay_add_payload(r, count, obs, act, ret, gacc, hip_stream);
  if (rc != APEX_OK) return rc;
  return apex_replay_add_publish(r, count, prio, first_key_out, hip_stream);
}

namespace {

int sample_begin_impl(apex_replay *r, uint32_t num_batches, uint32_t k, const uint64_t *rnd, uint64_t *key_out,
                      uint32_t *slot_out, uint64_t *mass_out, void *act_out, float *ret_out, float *gacc_out,
                      hipStream_t stream)
{
  if (!r || !num_batches || !k || !rnd || !slot_out || !mass_out) return APEX_ERR_INVALID_ARG;
  if (num_batches > APEX_MAX_BATCHES_PER_CALL || (uint64_t)num_batches * k > APEX_MAX_SAMPLES_PER_CALL)
    return APEX_ERR_TOO_LARGE;
  const uint64_t size = r->tail - r->head;
  if (size < r->cfg.min_size_to_sample) return APEX_ERR_NOT_READY;
  if (size == 0) return APEX_ERR_EMPTY;
  SampleArgs a{};
  a.tv = r->tv;
  a.st = r->state();
  a.k = k;
  a.rnd = rnd;
  a.key_out = key_out;
  a.slot_out = slot_out;
  a.mass = mass_out;
  a.act = r->act();
  a.act_bytes = r->cfg.act_bytes;
  a.ret = r->ret();
  a.gacc = r->gacc();
  a.act_out = static_cast<uint8_t *>(act_out);
  a.ret_out = ret_out;
  a.gacc_out = gacc_out;
  // every workgroup stages the whole top level: with a large top and many samples, larger workgroups
  // (16 samples each) stage it fewer times
  const uint32_t waves = (r->tv.n_top > 1024 && (uint64_t)num_batches * k >= 1024) ? 16 : 4;
  const size_t lds = ((size_t)r->tv.n_top + waves) * sizeof(uint64_t);
  sample_descent_kernel<<<dim3(blocks_for(k, waves), num_batches), dim3(waves * kWave), lds, stream>>>(a);
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

}  // namespace

int apex_replay_sample_begin(apex_replay_t *r, uint32_t num_batches, uint32_t k, const uint64_t *rnd,
                             uint64_t *key_out, uint32_t *slot_out, uint64_t *mass_out, void *act_out, float *ret_out,
                             float *gacc_out, void *hip_stream)
{
  return sample_begin_impl(r, num_batches, k, rnd, key_out, slot_out, mass_out, act_out, ret_out, gacc_out,
                           static_cast<hipStream_t>(hip_stream));
}

namespace {

// claimed: the first pass (update_claim) of a large update has already run.
int launch_update(apex_replay *r, uint64_t m, const uint64_t *key, const float *prio, hipStream_t stream,
                  const QSource &qs = QSource{}, bool claimed = false)
{
  ++r->tree_version;
  if (m <= 1024) {
    const UpdateArgs ua{r->tv, r->state(), (uint32_t)m, key, prio, r->qp, nullptr, nullptr, qs};
    update_small_kernel<<<dim3(1), dim3((uint32_t)round_up(m, kWave)), 0, stream>>>(ua);
  } else {
    const dim3 grid(blocks_for(m, 256)), block(256);
    if (!claimed)
      update_claim_kernel<<<grid, block, 0, stream>>>(ClaimArgs{r->cfg.max_slots, r->state(), (uint32_t)m, key, r->claim()});
    update_apply_kernel<<<grid, block, 0, stream>>>(r->tv, r->state(), (uint32_t)m, key, prio, r->qp, r->claim(), qs);
  }
  return hip_failed(hipGetLastError()) ? APEX_ERR_HIP : APEX_OK;
}

// gather + importance weights (+ a priority update riding along when it fits one workgroup)
// same_batch: the pairs are the batch being finished (key[i] lives in slot[i] and weighs mass[i]) and
// nothing has touched the tree since it was drawn.
int finish_impl(apex_replay *r, uint32_t num_batches, uint32_t k, float beta, const uint32_t *slot,
                const uint64_t *mass, float *weight_out, void *obs_out, uint64_t m, const uint64_t *key,
                const float *prio, hipStream_t stream, bool same_batch = false)
{
  SideJobs jobs;
  jobs.wa = WeightArgs{mass, weight_out, k, beta};
  const bool hint = same_batch && mass && m == (uint64_t)num_batches * k;
  if (m) ++r->tree_version;
  if (m && (m <= 1024 || hint)) {
    jobs.ua = UpdateArgs{r->tv, r->state(), (uint32_t)m, key, prio, r->qp, hint ? slot : nullptr, hint ? mass : nullptr,
                         QSource{}};
  }
  if (m > 1024) jobs.claim = ClaimArgs{r->cfg.max_slots, r->state(), (uint32_t)m, key, r->claim()};
  if (obs_out) {
    const RowMap by_slot{slot, nullptr, 0};
    const RowMap ident{nullptr, nullptr, 0};
    const int rc = launch_copy(r->obs(), by_slot, obs_out, ident, (uint64_t)num_batches * k, r->cfg.obs_bytes, stream, &jobs);
    if (rc != APEX_OK) return rc;
  }
  if (jobs.wa.weight_out) {  // no gather, or short rows: the weights get a small launch of their own
    batch_weights_kernel<<<dim3(num_batches, blocks_for(k, 512)), dim3(256), 0, stream>>>(jobs.wa);
    APEX_HIP(hipGetLastError());
  }
  // whatever of the update no launch above has taken (a claim pass that has run leaves the second pass)
  if (m && (jobs.ua.m || !(m <= 1024 || hint)))
    return launch_update(r, m, key, prio, stream, QSource{}, /*claimed=*/m > 1024 && jobs.claim.m == 0);
  return APEX_OK;
}

// n learner steps of one batch of k each, in strict order (draw i, write-back i, draw i+1, ...), as
// one standalone draw, one launch per step, and one small launch at the end: see
// learner_step_kernel.  Batch i goes to sets[(first_set + i) % depth]; kernel i reads the sets of
// batches i-1 and i and writes that of batch i+1, hence depth >= 3.
// Returns APEX_ERR_NOT_READY - with nothing enqueued - when the shapes do not fit the fused launch.
// The widest vector that the rows of the ring and of the batch buffers allow: 16, 4 or 1 bytes.
uint32_t step_vector_bytes(const apex_replay *r, uint32_t depth, const apex_batch_buffers_t *sets)
{
  uintptr_t mis = (uintptr_t)r->obs() | (uintptr_t)r->cfg.obs_bytes;
  for (uint32_t i = 0; i < depth; ++i) mis |= (uintptr_t)sets[i].obs;
  return (mis & 15) == 0 ? 16 : (mis & 3) == 0 ? 4 : 1;
}

bool fused_steps_fit(const apex_replay *r, uint32_t num_batches, uint32_t k, uint32_t depth,
                     const apex_batch_buffers_t *sets)
{
  if (num_batches != 1 || k > kStepMaxK || depth < 3 || depth > kStepSets) return false;
  for (uint32_t i = 0; i < depth; ++i)
    if ((uintptr_t)sets[i].slot & 15) return false;
  return true;
}

void launch_step(const StepArgs &args, uint32_t vector_bytes, uint32_t n_top, uint32_t wgs, uint32_t threads,
                 size_t lds, hipStream_t stream, int rider = kNoRider)
{
  StepArgs a = args;
  a.next_top = a.next.tv.level[a.next.tv.nlev - 1];
  a.next_k_div = make_fast_div(a.next.k);
  if (a.codec.raw_bytes && a.slot) return launch_step_codec(a, n_top, wgs, threads, lds, rider, stream);
  if (vector_bytes == 16) launch_step_t<u32x4>(a, n_top, wgs, threads, lds, rider, stream);
  else if (vector_bytes == 4) launch_step_t<uint32_t>(a, n_top, wgs, threads, lds, rider, stream);
  else launch_step_t<uint8_t>(a, n_top, wgs, threads, lds, rider, stream);
}

// A step launch that has been prepared but not issued: the last one of a call, held back while a small
// add round is open, because the round can ride in the same launch (see StepArgs::add).
struct HeldStep {
  bool valid = false;
  StepArgs a;
  uint32_t vector_bytes, n_top;
  size_t lds;
};

int issue_held_step(HeldStep *h, hipStream_t stream)
{
  if (!h->valid) return APEX_OK;
  h->valid = false;
  launch_step(h->a, h->vector_bytes, h->n_top, h->a.k, kStepThreads, h->lds, stream);
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

// The held step and a small add round in one launch.  APEX_ERR_NOT_READY - with nothing enqueued - if
// there is no held step or the two do not fit together (the round's rows allow only narrower vectors).
int issue_held_step_with_round(apex_replay *r, HeldStep *h, const NstepArgs &ns, const void *obs, const void *act,
                               uint64_t *first_key_out, hipStream_t stream)
{
  const uint64_t count = (uint64_t)ns.S * ns.T;
  uint32_t vb = 0, blocks = 0;
  if (!h->valid || h->a.codec.raw_bytes || !add_round_small_fits(r, ns, obs, &vb) || vb < h->vector_bytes)
    return APEX_ERR_NOT_READY;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  const bool both = r->second_version == r->tree_version;
  const int rc = add_round_args(r, ns, obs, act, h->vector_bytes, kStepThreads, both, &h->a.add, &blocks);
  if (rc != APEX_OK) return rc;
  h->valid = false;
  launch_step(h->a, h->vector_bytes, h->n_top, h->a.k + blocks, kStepThreads, h->lds, stream, kRoundRides);
  APEX_HIP(hipGetLastError());
  add_round_published(r, count, both, first_key_out);
  return APEX_OK;
}

// The held step and the masses of `count` new keys whose payload is in place (apex_replay_add_publish)
// in one launch.  APEX_ERR_NOT_READY - with nothing enqueued - if there is no held step.
int issue_held_step_with_leaves(apex_replay *r, HeldStep *h, uint64_t count, const float *prio,
                                uint64_t *first_key_out, hipStream_t stream)
{
  if (!h->valid || !count || !prio) return APEX_ERR_NOT_READY;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  const bool both = r->second_version == r->tree_version;
  h->a.leaves = AddLeavesArgs{r->tv, r->tv2, both, r->state(), count, prio, r->qp};
  h->valid = false;
  launch_step(h->a, h->vector_bytes, h->n_top, h->a.k + blocks_for(count, kStepThreads), kStepThreads, h->lds, stream,
              kLeavesRide);
  APEX_HIP(hipGetLastError());
  add_round_published(r, count, both, first_key_out);
  return APEX_OK;
}

int fused_steps(apex_replay *r, uint32_t n, uint32_t k, float beta, const uint64_t *rnd, const float *new_prio,
                const apex_batch_buffers_t *sets, uint32_t depth, uint32_t first_set, HeldStep *hold,
                uint32_t codec_raw_bytes, hipStream_t stream)
{
  // The same gate as apex_replay_sample, from the host mirror and before anything is enqueued: a draw from an
  // empty tree has no defined result (every stratum has width 0), and the learner waits for a minimum fill.
  const uint64_t size = r->tail - r->head;
  if (size < r->cfg.min_size_to_sample) return APEX_ERR_NOT_READY;
  if (size == 0) return APEX_ERR_EMPTY;
  const auto idx = [&](uint32_t i) { return (first_set + i) % depth; };
  const auto set = [&](uint32_t i) -> const apex_batch_buffers_t & { return sets[idx(i)]; };
  const apex_batch_buffers_t &b0 = set(0);
  const size_t lds = round_up(r->tv.n_top, kFanout) * 8;
  const uint32_t vb = step_vector_bytes(r, depth, sets);
  if (new_prio) {
    // Launch i reads one copy of the tree and writes the other; the first draw is launch "-1" of that
    // scheme (it reads the first copy and writes the first batch's changes into the second), so both
    // copies have to be equal before it.
    if (r->second_version != r->tree_version)
      copy_words_kernel<<<dim3(2048), dim3(256), 0, stream>>>(r->tv2.level[0], r->tv.level[0], r->geo.tree_words);
    StepArgs a{};
    a.k = k;
    a.qp = r->qp;
    a.st = r->state();
    a.wr = r->tv2;
    a.next.tv = r->tv;
    a.next.st = r->state();
    a.next.k = k;
    a.next.rnd = rnd;
    a.next.key_out = b0.key;
    a.next.slot_out = b0.slot;
    a.next.mass = b0.mass;
    a.next_prio = new_prio;
    a.next_dq = r->stepq(idx(0));
    launch_step(a, vb, r->tv.n_top, k, kWave, lds, stream);
    APEX_HIP(hipGetLastError());
  } else {
    const int rc = sample_begin_impl(r, 1, k, rnd, b0.key, b0.slot, b0.mass, nullptr, nullptr, nullptr, stream);
    if (rc != APEX_OK) return rc;
  }
  for (uint32_t i = 0; i < n; ++i) {
    const apex_batch_buffers_t &b = set(i);
    const TreeView &rd = (new_prio && !(i & 1)) ? r->tv2 : r->tv;
    const TreeView &wr = (new_prio && !(i & 1)) ? r->tv : r->tv2;
    StepArgs a{};
    a.src = r->obs();
    a.dst = static_cast<uint8_t *>(b.obs);
    a.row_bytes = r->cfg.obs_bytes;
    a.vecs_per_row = (uint32_t)(a.row_bytes / vb);
    if (codec_raw_bytes) {  // rows decoded on their way out: the set's obs buffer is [k, raw bytes]
      a.codec = codec_shape(codec_raw_bytes);
      a.vecs_per_row = codec_raw_bytes / 16;
    }
    a.act = r->act();
    a.act_bytes = r->cfg.act_bytes;
    a.ret = r->ret();
    a.gacc = r->gacc();
    a.act_out = static_cast<uint8_t *>(b.act);
    a.ret_out = b.ret;
    a.gacc_out = b.gacc;
    a.k = k;
    a.slot = b.slot;
    a.dq = new_prio ? r->stepq(idx(i)) : nullptr;
    a.qp = r->qp;
    a.wr = wr;
    a.st = r->state();
    a.wa = WeightArgs{b.mass, b.weight, k, beta};
    a.next.tv = rd;
    a.next.st = r->state();
    a.next.k = k;
    if (i + 1 < n) {
      const apex_batch_buffers_t &nb = set(i + 1);
      a.next.rnd = rnd + (uint64_t)(i + 1) * k;
      a.next.key_out = nb.key;
      a.next.slot_out = nb.slot;
      a.next.mass = nb.mass;
      // the small columns of batch i+1 are gathered by the launch that copies its rows
      if (new_prio) {
        a.next_prio = new_prio + (uint64_t)(i + 1) * k;
        a.next_dq = r->stepq(idx(i + 1));
      }
    }
    if (hold && i + 1 == n) {  // issued by the caller's next call, perhaps together with an add round
      hold->valid = true;
      hold->a = a;
      hold->vector_bytes = vb;
      hold->n_top = r->tv.n_top;
      hold->lds = lds;
    } else {
      launch_step(a, vb, r->tv.n_top, k, kStepThreads, lds, stream);
    }
  }
  // (every change has now been applied to both copies)
  if (new_prio) r->second_version = ++r->tree_version;
  APEX_HIP(hipGetLastError());
  return APEX_OK;
}

int check_finish_args(const apex_replay *r, uint32_t num_batches, uint32_t k, float beta, const uint32_t *slot,
                      const uint64_t *mass, const float *weight_out)
{
  if (!r || !num_batches || !k || !slot || !(beta >= 0.0f) || !(beta <= 1.0f)) return APEX_ERR_INVALID_ARG;
  if (weight_out && !mass) return APEX_ERR_INVALID_ARG;
  if (num_batches > APEX_MAX_BATCHES_PER_CALL || (uint64_t)num_batches * k > APEX_MAX_SAMPLES_PER_CALL)
    return APEX_ERR_TOO_LARGE;
  return APEX_OK;
}

}  // namespace

int apex_replay_sample_finish(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint32_t *slot,
                              const uint64_t *mass, float *weight_out, void *obs_out, void *hip_stream)
{
  const int rc = check_finish_args(r, num_batches, k, beta, slot, mass, weight_out);
  if (rc != APEX_OK) return rc;
  return finish_impl(r, num_batches, k, beta, slot, mass, weight_out, obs_out, 0, nullptr, nullptr,
                     static_cast<hipStream_t>(hip_stream));
}

int apex_replay_sample_finish_update(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta,
                                     const uint32_t *slot, const uint64_t *mass, float *weight_out, void *obs_out,
                                     uint64_t m, const uint64_t *key, const float *prio, void *hip_stream)
{
  const int rc = check_finish_args(r, num_batches, k, beta, slot, mass, weight_out);
  if (rc != APEX_OK) return rc;
  if (m && !prio) return APEX_ERR_INVALID_ARG;
  if (m >= 0xffffffffull) return APEX_ERR_TOO_LARGE;
  if (m && !key) return APEX_ERR_INVALID_ARG;
  return finish_impl(r, num_batches, k, beta, slot, mass, weight_out, obs_out, m, key, prio,
                     static_cast<hipStream_t>(hip_stream));
}

int apex_replay_sample_finish_writeback(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta,
                                        const uint64_t *key, const uint32_t *slot, const uint64_t *mass,
                                        float *weight_out, void *obs_out, const float *prio, void *hip_stream)
{
  const int rc = check_finish_args(r, num_batches, k, beta, slot, mass, weight_out);
  if (rc != APEX_OK) return rc;
  if (!key || !mass || !prio) return APEX_ERR_INVALID_ARG;
  return finish_impl(r, num_batches, k, beta, slot, mass, weight_out, obs_out, (uint64_t)num_batches * k, key, prio,
                     static_cast<hipStream_t>(hip_stream), /*same_batch=*/true);
}

int apex_replay_sample(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                       uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                       float *ret_out, float *gacc_out, void *hip_stream)
{
  if (!r || !(beta >= 0.0f) || !(beta <= 1.0f)) return APEX_ERR_INVALID_ARG;
  const int rc = apex_replay_sample_begin(r, num_batches, k, rnd, key_out, slot_out, r->mass(), act_out, ret_out,
                                          gacc_out, hip_stream);
  if (rc != APEX_OK) return rc;
  if (!weight_out && !obs_out) return APEX_OK;
  return apex_replay_sample_finish(r, num_batches, k, beta, slot_out, r->mass(), weight_out, obs_out, hip_stream);
}

int apex_replay_sample_noalloc(apex_replay_t *r, uint32_t num_batches, uint32_t k, float beta, const uint64_t *rnd,
                               uint64_t *key_out, uint32_t *slot_out, float *weight_out, void *obs_out, void *act_out,
                               float *ret_out, float *gacc_out, void *hip_stream)
{
  if (!r || !(beta >= 0.0f) || !(beta <= 1.0f)) return APEX_ERR_INVALID_ARG;
  if (num_batches && k && (uint64_t)num_batches * k > APEX_NOALLOC_MAX_SAMPLES) return APEX_ERR_TOO_LARGE;
  uint64_t *const mass = static_scratch_ptr();  // this GPU's copy; every entry the weights read is written by the draw
  if (!mass) return APEX_ERR_HIP;
  const int rc = apex_replay_sample_begin(r, num_batches, k, rnd, key_out, slot_out, mass, act_out, ret_out, gacc_out,
                                          hip_stream);
  if (rc != APEX_OK) return rc;
  if (!weight_out && !obs_out) return APEX_OK;
  return apex_replay_sample_finish(r, num_batches, k, beta, slot_out, mass, weight_out, obs_out, hip_stream);
}

int apex_replay_gather(apex_replay_t *r, uint64_t count, const uint32_t *slot, void *obs_out, void *act_out,
                       float *ret_out, float *gacc_out, void *hip_stream)
{
  if (!r || (count && !slot)) return APEX_ERR_INVALID_ARG;
  if (count > APEX_MAX_SAMPLES_PER_CALL) return APEX_ERR_TOO_LARGE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const RowMap by_slot{slot, nullptr, 0};
  const RowMap ident{nullptr, nullptr, 0};
  int rc;
  if (obs_out && (rc = launch_copy(r->obs(), by_slot, obs_out, ident, count, r->cfg.obs_bytes, stream)) != APEX_OK) return rc;
  if (act_out && (rc = launch_copy(r->act(), by_slot, act_out, ident, count, r->cfg.act_bytes, stream)) != APEX_OK) return rc;
  if (ret_out && (rc = launch_copy(r->ret(), by_slot, ret_out, ident, count, 4, stream)) != APEX_OK) return rc;
  if (gacc_out && (rc = launch_copy(r->gacc(), by_slot, gacc_out, ident, count, 4, stream)) != APEX_OK) return rc;
  return APEX_OK;
}

int apex_replay_update_priorities(apex_replay_t *r, uint64_t m, const uint64_t *key, const float *prio,
                                  void *hip_stream)
{
  if (!r || (m && (!key || !prio))) return APEX_ERR_INVALID_ARG;
  if (m >= 0xffffffffull) return APEX_ERR_TOO_LARGE;
  if (m == 0) return APEX_OK;
  return launch_update(r, m, key, prio, static_cast<hipStream_t>(hip_stream));
}

int apex_replay_update_from_q(apex_replay_t *r, uint64_t m, const uint64_t *key, uint32_t A, const float *q_taken,
                              const float *q_online_next, const float *q_target_next, float *prio_out,
                              void *hip_stream)
{
  if (!r || !A || (m && (!key || !q_taken || !q_online_next || !q_target_next))) return APEX_ERR_INVALID_ARG;
  if (m >= 0xffffffffull) return APEX_ERR_TOO_LARGE;
  if (m == 0) return APEX_OK;
  const QSource qs{q_taken, q_online_next, q_target_next, A, r->ret(), r->gacc(), prio_out};
  return launch_update(r, m, key, nullptr, static_cast<hipStream_t>(hip_stream), qs);
}

int apex_replay_evict(apex_replay_t *r, uint64_t *evicted_out, void *hip_stream)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  const uint64_t size = r->tail - r->head;
  const uint64_t e = size > r->cfg.capacity ? size - r->cfg.capacity : 0;
  if (evicted_out) *evicted_out = e;
  if (e == 0) return APEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const bool both = r->second_version == r->tree_version;
  ++r->tree_version;
  if (both) r->second_version = r->tree_version;
  evict_leaves_kernel<<<dim3(blocks_for(e, 256)), dim3(256), 0, stream>>>(r->tv, r->tv2, both, r->state(), e);
  APEX_HIP(hipGetLastError());
  r->head += e;
  return APEX_OK;
}

int apex_replay_resync(apex_replay_t *r, void *hip_stream)
{
  if (!r) return APEX_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceState st;
  APEX_HIP(hipMemcpyAsync(&st, r->state(), sizeof st, hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipStreamSynchronize(stream));
  r->head = st.head;
  r->tail = st.tail;
  return APEX_OK;
}

int apex_replay_stats(apex_replay_t *r, apex_replay_stats_t *out, void *hip_stream)
{
  if (!r || !out) return APEX_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  DeviceState st;
  APEX_HIP(hipMemcpyAsync(&st, r->state(), sizeof st, hipMemcpyDeviceToHost, stream));
  // root = sum of the top level (at most kTopMax words)
  static thread_local uint64_t top[kTopMax];
  APEX_HIP(hipMemcpyAsync(top, r->tv.level[r->tv.nlev - 1], (size_t)r->tv.n_top * 8, hipMemcpyDeviceToHost, stream));
  APEX_HIP(hipStreamSynchronize(stream));
  uint64_t root = 0;
  for (uint32_t i = 0; i < r->tv.n_top; ++i) root += top[i];
  out->size = st.tail - st.head;
  out->head = st.head;
  out->tail = st.tail;
  out->root = root;
  out->n_stale_dropped = st.n_stale;
  out->n_clamped = st.n_clamped;
  return APEX_OK;
}

}  // extern "C"

#include "pipeline.inc.hpp"
#include "evict_prio.inc.hpp"
#include "codec.inc.hpp"
