// Lossless block codec of stored observations (Section 4.1: observations are kept compressed in the
// replay memory and decompressed as batches are fetched): encode on the way into the ring, decode on
// the way out.  Included by apex_replay.hip (one translation unit), after the plain entry points.
//
// A row of raw_bytes = 64 * nb bytes is cut into nb blocks of 64 bytes.  A block whose bytes are all
// equal is kept as that byte, any other block as it is.  Encoded row, little-endian:
//   0            u32 n_raw (blocks kept as they are), 12 zero bytes
//   16           mask, bit b set iff block b is kept as it is: ceil(nb/64) u64 words, zero-padded to 16 bytes
//   16 + M       the byte of every other block, in block order (room for nb, rounded up to 16)
//   16 + M + V   the blocks kept as they are, in block order, 64 bytes each
// The stride of the store (obs_bytes of the memory) must be at least 16 + M + V + 64 * nb.

namespace apex {

constexpr uint32_t kCodecThreads = 512;
constexpr uint32_t kCodecMaxBlocks = 4096;  // 256 KB of raw row; one LDS word per block

// Blocks kept as they are before block b (mask words in LDS).
__device__ __forceinline__ uint32_t codec_rank(const uint64_t *mask, uint32_t b)
{
  uint32_t r = 0;
  for (uint32_t w = 0; w < b / 64; ++w) r += __popcll(mask[w]);
  return r + __popcll(mask[b / 64] & ((1ull << (b % 64)) - 1));
}

// One workgroup per row: row i of the dense source into the ring row that `to` names.  A thread looks
// at a whole block (four 16-byte loads), the wave's ballot is a word of the mask, and once the
// workgroup's mask is complete every thread knows where its block goes.
__global__ __launch_bounds__(kCodecThreads) void codec_encode_rows_kernel(const uint8_t *__restrict__ src,
                                                                         uint8_t *__restrict__ ring, RowMap to,
                                                                         uint64_t ring_stride, CodecShape c)
{
  __shared__ uint64_t mask[kCodecMaxBlocks / 64];
  const uint64_t i = blockIdx.x;
  const u32x4 *s = reinterpret_cast<const u32x4 *>(src + i * c.raw_bytes);
  uint8_t *d = ring + map_row(to, i) * ring_stride;
  const uint32_t tid = threadIdx.x;
  const uint32_t chunks = (c.nb + kCodecThreads - 1) / kCodecThreads;

  u32x4 v[4];
  bool flat = true;  // of this thread's block in the chunk at hand
  for (uint32_t ch = 0; ch < chunks; ++ch) {
    const uint32_t b = ch * kCodecThreads + tid;
    flat = true;
    if (b < c.nb) {
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = s[4 * b + q];
      const uint32_t first = v[0].x;
      flat = first == (first & 0xffu) * 0x01010101u;
#pragma unroll
      for (int q = 0; q < 4; ++q) flat = flat && v[q].x == first && v[q].y == first && v[q].z == first && v[q].w == first;
    }
    const uint64_t word = __ballot(!flat);
    if (lane_id() == 0 && b / 64 < c.mask_words) mask[b / 64] = word;
  }
  __syncthreads();

  if (tid == 0) {
    uint32_t n_raw = 0;
    for (uint32_t w = 0; w < c.mask_words; ++w) n_raw += __popcll(mask[w]);
    *reinterpret_cast<u32x4 *>(d) = u32x4{n_raw, 0, 0, 0};
  }
  for (uint32_t w = tid; w < (c.flat_off - 16) / 8; w += kCodecThreads)  // the mask and its padding
    reinterpret_cast<uint64_t *>(d + 16)[w] = w < c.mask_words ? mask[w] : 0;

  for (uint32_t ch = 0; ch < chunks; ++ch) {
    const uint32_t b = ch * kCodecThreads + tid;
    if (b >= c.nb) break;
    if (chunks > 1) {  // the registers hold the last chunk only
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = s[4 * b + q];
    }
    const bool kept = mask[b / 64] >> (b % 64) & 1;
    const uint32_t rank = codec_rank(mask, b);
    if (kept) {
      u32x4 *o = reinterpret_cast<u32x4 *>(d + c.raw_off + 64ull * rank);
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q] = v[q];
    } else {
      d[c.flat_off + (b - rank)] = (uint8_t)v[0].x;
    }
  }
}

// The same for rows of at most 512 blocks (32 KB raw) with every load and store 16 bytes per lane in row
// order: four neighbouring lanes hold a block, agree on whether it is flat with two exchanges, and the first
// of them enters the block's bit into the mask in LDS; after one barrier every lane knows where its 16 bytes go.
__global__ __launch_bounds__(kCodecThreads) void codec_encode_rows_direct_kernel(const uint8_t *__restrict__ src,
                                                                                uint8_t *__restrict__ ring, RowMap to,
                                                                                uint64_t ring_stride, CodecShape c)
{
  __shared__ uint64_t mask[8];  // 512 blocks
  uint32_t *mask32 = reinterpret_cast<uint32_t *>(mask);
  const uint64_t i = blockIdx.x;
  const u32x4 *s = reinterpret_cast<const u32x4 *>(src + i * c.raw_bytes);
  uint8_t *d = ring + map_row(to, i) * ring_stride;
  const uint32_t tid = threadIdx.x, nvec = c.raw_bytes / 16;
  if (tid < 16) mask32[tid] = 0;
  u32x4 t[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint32_t v = u * kCodecThreads + tid;
    t[u] = v < nvec ? __builtin_nontemporal_load(s + v) : u32x4{0, 0, 0, 0};
  }
  __syncthreads();  // the mask is cleared
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint32_t v = u * kCodecThreads + tid, b = v / 4;
    const uint32_t x = t[u].x;
    bool flat = x == (x & 0xffu) * 0x01010101u && t[u].y == x && t[u].z == x && t[u].w == x;
    // the four lanes of a block: all flat, with the same byte
    flat = flat && __shfl_xor(x, 1, kWave) == x;
    flat = __shfl_xor((int)flat, 1, kWave) && flat;
    flat = flat && __shfl_xor(x, 2, kWave) == x;
    flat = __shfl_xor((int)flat, 2, kWave) && flat;
    if (v < nvec && (v & 3) == 0 && !flat) atomicOr(&mask32[b / 32], 1u << (b % 32));
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t n_raw = 0;
    for (uint32_t w = 0; w < 16; ++w) n_raw += __popc(mask32[w]);
    *reinterpret_cast<u32x4 *>(d) = u32x4{n_raw, 0, 0, 0};
  }
  if (tid < (c.flat_off - 16) / 8) reinterpret_cast<uint64_t *>(d + 16)[tid] = tid < c.mask_words ? mask[tid] : 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint32_t v = u * kCodecThreads + tid, b = v / 4;
    if (v >= nvec) break;
    const bool kept = mask[b / 64] >> (b % 64) & 1;
    const uint32_t rank = codec_rank(mask, b);
    if (kept)
      __builtin_nontemporal_store(t[u], reinterpret_cast<u32x4 *>(d + c.raw_off + 64ull * rank) + (v & 3));
    else if ((v & 3) == 0)
      d[c.flat_off + (b - rank)] = (uint8_t)t[u].x;
  }
}

// One workgroup per output row: the mask into LDS, one LDS word per block saying where its bytes come
// from, then the row is written 16 bytes per lane, in order, as a plain gather writes it.
__global__ __launch_bounds__(kCodecThreads) void codec_decode_rows_kernel(const uint8_t *__restrict__ ring,
                                                                         const uint32_t *__restrict__ slot,
                                                                         uint64_t ring_stride,
                                                                         uint8_t *__restrict__ out, CodecShape c)
{
  __shared__ uint64_t mask[kCodecMaxBlocks / 64];
  __shared__ uint32_t from[kCodecMaxBlocks];  // offset of a kept block in the encoded row, or 0x80000000 | byte
  const uint64_t i = blockIdx.x;
  const uint8_t *e = ring + (uint64_t)slot[i] * ring_stride;
  const uint32_t tid = threadIdx.x;
  for (uint32_t w = tid; w < c.mask_words; w += kCodecThreads) mask[w] = reinterpret_cast<const uint64_t *>(e + 16)[w];
  __syncthreads();
  for (uint32_t b = tid; b < c.nb; b += kCodecThreads) {
    const uint32_t rank = codec_rank(mask, b);
    const bool kept = mask[b / 64] >> (b % 64) & 1;
    from[b] = kept ? c.raw_off + 64 * rank : 0x80000000u | e[c.flat_off + (b - rank)];
  }
  __syncthreads();
  u32x4 *o = reinterpret_cast<u32x4 *>(out + i * c.raw_bytes);
  const uint32_t nvec = c.raw_bytes / 16;
  for (uint32_t v0 = 0; v0 < nvec; v0 += 4 * kCodecThreads) {
    u32x4 t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid;
      if (v < nvec) {
        const uint32_t f = from[v / 4];
        if (f & 0x80000000u) {
          const uint32_t x = (f & 0xffu) * 0x01010101u;
          t[u] = u32x4{x, x, x, x};
        } else {
          t[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(e + f) + (v & 3));
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid;
      if (v < nvec) __builtin_nontemporal_store(t[u], o + v);
    }
  }
}

// The same for rows of at most 512 blocks (32 KB raw), without LDS and without a barrier: the mask is at most
// eight words, which every wave holds in scalar registers; the 64 lanes of a wave work on 16 consecutive
// blocks, all within one word of the mask, so where a block's bytes come from is a few popcounts.
__global__ __launch_bounds__(kCodecThreads) void codec_decode_rows_direct_kernel(const uint8_t *__restrict__ ring,
                                                                                const uint32_t *__restrict__ slot,
                                                                                uint64_t ring_stride,
                                                                                uint8_t *__restrict__ out, CodecShape c)
{
  const uint64_t i = blockIdx.x;
  const CodecRow enc = codec_open_row(ring + (uint64_t)slot[i] * ring_stride, c);
  const uint32_t tid = threadIdx.x, nvec = c.raw_bytes / 16;
  u32x4 *o = reinterpret_cast<u32x4 *>(out + i * c.raw_bytes);
  CodecFetched f[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) f[u] = codec_fetch(enc, c, u * kCodecThreads + tid);
  u32x4 t[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) t[u] = codec_piece(f[u]);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint32_t v = u * kCodecThreads + tid;
    if (v < nvec) __builtin_nontemporal_store(t[u], o + v);
  }
}

}  // namespace apex

extern "C" {

size_t apex_codec_row_bytes(uint32_t raw_bytes)
{
  if (raw_bytes == 0 || raw_bytes % 64 || raw_bytes / 64 > kCodecMaxBlocks) return 0;
  return (size_t)codec_shape(raw_bytes).stride;
}

int apex_replay_add_payload_encoded(apex_replay_t *r, uint64_t count, const void *raw_obs, uint32_t raw_bytes,
                                    const void *act, const float *ret, const float *gacc, void *hip_stream)
{
  if (!r || (count && !raw_obs)) return APEX_ERR_INVALID_ARG;
  const size_t stride = apex_codec_row_bytes(raw_bytes);
  if (!stride || ((uintptr_t)raw_obs & 15) || (r->cfg.obs_bytes & 15)) return APEX_ERR_INVALID_ARG;
  if (stride > r->cfg.obs_bytes) return APEX_ERR_TOO_LARGE;
  if ((r->tail - r->head) + count > r->cfg.max_slots) return APEX_ERR_FULL;
  if (count == 0) return APEX_OK;
  if (count > 0x7ffffff0ull) return APEX_ERR_TOO_LARGE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const RowMap ring{nullptr, &r->state()->tail, r->cfg.max_slots};
  const CodecShape c = codec_shape(raw_bytes);
  if (c.nb <= kCodecThreads)
    codec_encode_rows_direct_kernel<<<dim3((uint32_t)count), dim3(kCodecThreads), 0, stream>>>(
        static_cast<const uint8_t *>(raw_obs), r->obs(), ring, r->cfg.obs_bytes, c);
  else
    codec_encode_rows_kernel<<<dim3((uint32_t)count), dim3(kCodecThreads), 0, stream>>>(
        static_cast<const uint8_t *>(raw_obs), r->obs(), ring, r->cfg.obs_bytes, c);
  APEX_HIP(hipGetLastError());
  if (act || ret || gacc) {
    const PayloadRing pr{r->obs(), r->act(), r->ret(), r->gacc(), r->cfg.obs_bytes, r->cfg.act_bytes};
    return add_small_columns(pr, count, act, ret, gacc, ring, stream);
  }
  return APEX_OK;
}

int apex_replay_gather_decoded(apex_replay_t *r, uint64_t count, const uint32_t *slot, uint32_t raw_bytes,
                               void *obs_out, void *act_out, float *ret_out, float *gacc_out, void *hip_stream)
{
  if (!r || (count && !slot)) return APEX_ERR_INVALID_ARG;
  const size_t stride = apex_codec_row_bytes(raw_bytes);
  if (!stride || ((uintptr_t)obs_out & 15) || (r->cfg.obs_bytes & 15)) return APEX_ERR_INVALID_ARG;
  if (stride > r->cfg.obs_bytes || count > APEX_MAX_SAMPLES_PER_CALL) return APEX_ERR_TOO_LARGE;
  if (count == 0) return APEX_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (obs_out) {
    const CodecShape c = codec_shape(raw_bytes);
    if (c.nb <= kCodecThreads)
      codec_decode_rows_direct_kernel<<<dim3((uint32_t)count), dim3(kCodecThreads), 0, stream>>>(
          r->obs(), slot, r->cfg.obs_bytes, static_cast<uint8_t *>(obs_out), c);
    else
      codec_decode_rows_kernel<<<dim3((uint32_t)count), dim3(kCodecThreads), 0, stream>>>(
          r->obs(), slot, r->cfg.obs_bytes, static_cast<uint8_t *>(obs_out), c);
    APEX_HIP(hipGetLastError());
  }
  return apex_replay_gather(r, count, slot, nullptr, act_out, ret_out, gacc_out, hip_stream);
}

}  // extern "C"
