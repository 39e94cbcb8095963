// Lossless block codec of stored observations (Section 4.1: observations are kept compressed in the
// replay memory and decompressed as batches are fetched): encode on the way into the ring, decode on
// the way out.  Included by apex_replay.hip (one translation unit), after the plain entry points.
//
// A row of raw_bytes = 64 * nb bytes is cut into nb blocks of 64 bytes.  A block whose bytes are all
// equal is kept as that byte, any other block as it is, and every part has a fixed place, so that
// nothing has to be looked up before it can be fetched.  Encoded row, little-endian:
//   0        mask, bit b set iff block b is kept as it is: ceil(nb/64) u64 words, zero-padded to 16 bytes (M)
//   M        one byte per block: the byte of block b if it is not kept as it is (else unspecified); nb bytes,
//            rounded up to a multiple of 16 (V)
//   M + V    the image of the row: bytes [64 b, 64 b + 64) hold block b if it is kept as it is (else unspecified)
// The stride of the store (obs_bytes of the memory) must be at least M + V + 64 * nb.  An encoder writes,
// and a decoder that looks at the mask first reads, only the parts that carry data.

namespace apex {

constexpr uint32_t kCodecThreads = 512;
constexpr uint32_t kCodecUnroll = 4;

// One workgroup per row, a lane per 16-byte piece, in row order (loads and stores as a plain copy makes them):
// the four lanes of a block agree on whether it is flat with two exchanges; a wave's ballot, every fourth
// bit of it, is 16 bits of the mask.  No LDS, no barrier.
__global__ __launch_bounds__(kCodecThreads) void codec_encode_rows_kernel(const uint8_t *__restrict__ src,
                                                                         uint8_t *__restrict__ ring, RowMap to,
                                                                         uint64_t ring_stride, CodecShape c)
{
  const uint64_t i = blockIdx.x;
  const u32x4 *s = reinterpret_cast<const u32x4 *>(src + i * c.raw_bytes);
  uint8_t *d = ring + map_row(to, i) * ring_stride;
  const uint32_t tid = threadIdx.x, nvec = c.raw_bytes / 16;
  const uint32_t groups = (c.nb + 15) / 16;  // 16-bit pieces of the mask that hold blocks
  for (uint32_t g = groups + tid; g < c.flat_off / 2; g += kCodecThreads) reinterpret_cast<uint16_t *>(d)[g] = 0;
  for (uint32_t v0 = 0; v0 < nvec; v0 += kCodecUnroll * kCodecThreads) {
    u32x4 t[kCodecUnroll];
#pragma unroll
    for (int u = 0; u < (int)kCodecUnroll; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid;
      t[u] = v < nvec ? __builtin_nontemporal_load(s + v) : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < (int)kCodecUnroll; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid, b = v / 4;
      const uint32_t x = t[u].x;
      bool flat = x == (x & 0xffu) * 0x01010101u && t[u].y == x && t[u].z == x && t[u].w == x;
      // the four lanes of a block: all flat, with the same byte
      flat = flat && __shfl_xor(x, 1, kWave) == x;
      flat = __shfl_xor((int)flat, 1, kWave) && flat;
      flat = flat && __shfl_xor(x, 2, kWave) == x;
      flat = __shfl_xor((int)flat, 2, kWave) && flat;
      const bool kept = v < nvec && !flat;
      uint64_t bits = __ballot(kept) & 0x1111111111111111ull;  // one bit per block, at every fourth place
      bits = (bits | bits >> 3) & 0x0303030303030303ull;
      bits = (bits | bits >> 6) & 0x000f000f000f000full;
      bits = (bits | bits >> 12) & 0x000000ff000000ffull;
      bits = (bits | bits >> 24) & 0xffffull;
      const uint32_t first_v = v0 + u * kCodecThreads + (tid & ~(kWave - 1));  // of this wave
      if (lane_id() == 0 && first_v < nvec) reinterpret_cast<uint16_t *>(d)[first_v / 64] = (uint16_t)bits;
      if (kept)
        __builtin_nontemporal_store(t[u], reinterpret_cast<u32x4 *>(d + c.image_off) + v);
      else if (v < nvec && (v & 3) == 0)
        d[c.flat_off + b] = (uint8_t)x;
    }
  }
}

// One workgroup per output row, a lane per 16-byte piece, in row order.  The word of the mask first (the 64
// lanes of a wave share it), then only what carries data is read: the piece, or its block's byte.
__global__ __launch_bounds__(kCodecThreads) void codec_decode_rows_kernel(const uint8_t *__restrict__ ring,
                                                                         const uint32_t *__restrict__ slot,
                                                                         uint64_t ring_stride,
                                                                         uint8_t *__restrict__ out, CodecShape c)
{
  const uint64_t i = blockIdx.x;
  const uint8_t *e = ring + (uint64_t)slot[i] * ring_stride;
  const uint64_t *mask = reinterpret_cast<const uint64_t *>(e);
  u32x4 *o = reinterpret_cast<u32x4 *>(out + i * c.raw_bytes);
  const uint32_t tid = threadIdx.x, nvec = c.raw_bytes / 16;
  for (uint32_t v0 = 0; v0 < nvec; v0 += kCodecUnroll * kCodecThreads) {
    uint64_t word[kCodecUnroll];
#pragma unroll
    for (int u = 0; u < (int)kCodecUnroll; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid;
      word[u] = v < nvec ? mask[v >> 8] : 0;
    }
    u32x4 t[kCodecUnroll];
    uint32_t byte[kCodecUnroll];
#pragma unroll
    for (int u = 0; u < (int)kCodecUnroll; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid, b = v / 4;
      t[u] = u32x4{0, 0, 0, 0};
      byte[u] = 0;
      if (v < nvec) {
        if (word[u] >> (b & 63) & 1)
          t[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(e + c.image_off) + v);
        else
          byte[u] = e[c.flat_off + b];
      }
    }
#pragma unroll
    for (int u = 0; u < (int)kCodecUnroll; ++u) {
      const uint32_t v = v0 + u * kCodecThreads + tid, b = v / 4;
      if (v < nvec) {
        const uint32_t x = byte[u] * 0x01010101u;
        __builtin_nontemporal_store((word[u] >> (b & 63) & 1) ? t[u] : u32x4{x, x, x, x}, o + v);
      }
    }
  }
}

}  // namespace apex

extern "C" {

size_t apex_codec_row_bytes(uint32_t raw_bytes)
{
  if (raw_bytes == 0 || raw_bytes % 64) return 0;
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
  codec_encode_rows_kernel<<<dim3((uint32_t)count), dim3(kCodecThreads), 0, stream>>>(
      static_cast<const uint8_t *>(raw_obs), r->obs(), ring, r->cfg.obs_bytes, codec_shape(raw_bytes));
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
    codec_decode_rows_kernel<<<dim3((uint32_t)count), dim3(kCodecThreads), 0, stream>>>(
        r->obs(), slot, r->cfg.obs_bytes, static_cast<uint8_t *>(obs_out), codec_shape(raw_bytes));
    APEX_HIP(hipGetLastError());
  }
  return apex_replay_gather(r, count, slot, nullptr, act_out, ret_out, gacc_out, hip_stream);
}

}  // extern "C"
