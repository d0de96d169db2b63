// Streaming copy of one piece of a chunk by one wavefront (device code only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ckpt {

constexpr int MOVE_UNROLL = 16;  // 16 KiB piece = 16 x (64 lanes x 16 B), all loads issued before the stores

// Non-temporal 16-byte global accesses: staged data is touched once per pass,
// and on MI355X a copy with nt loads and nt stores measured 5.9 TB/s (read +
// write) against 5.3 TB/s with plain accesses.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const u32x4 __attribute__((address_space(1))) *global_load_ptr;
typedef u32x4 __attribute__((address_space(1))) *global_store_ptr;
__device__ __forceinline__ uint4 stream_load16(const uint8_t *p) {
  const u32x4 v = __builtin_nontemporal_load((global_load_ptr)(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store16(uint8_t *p, uint4 v) {
  const u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, (global_store_ptr)(p));
}

__device__ __forceinline__ uint4 load_partial16(const uint8_t *src, uint32_t valid) {
  // bytes [0, valid) from src, zeros above; valid in 1..15
  uint32_t w[4] = {0, 0, 0, 0};
  for (uint32_t b = 0; b < valid; ++b) w[b >> 2] |= (uint32_t)src[b] << (8 * (b & 3));
  return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ void store_partial16(uint8_t *dst, uint4 v, uint32_t valid) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  for (uint32_t b = 0; b < valid; ++b) dst[b] = (uint8_t)(w[b >> 2] >> (8 * (b & 3)));
}

// Copies bytes [lo, hi) of a chunk of length len from src to dst and touches
// nothing outside that range; lo, hi are multiples of 16 (hi at most pad16(len)).  The piece that straddles
// len is assembled bytewise: ZERO_PAD writes it as a full 16 bytes with zeros
// above len (staging), otherwise exactly the valid bytes are written.
template <bool ZERO_PAD>
__device__ __forceinline__ void move_piece(const uint8_t *src, uint8_t *dst, uint32_t lo, uint32_t hi,
                                           uint32_t len, uint32_t lane) {
  for (uint32_t base = lo + lane * 16; base < hi; base += 64 * 16 * MOVE_UNROLL) {
    uint4 v[MOVE_UNROLL];
#pragma unroll
    for (int u = 0; u < MOVE_UNROLL; ++u) {
      const uint32_t o = base + u * 64 * 16;
      if (o >= hi) continue;                 // the piece may end before the chunk does
      if (o + 16 <= len)
        v[u] = stream_load16(src + o);
      else if (o < len)
        v[u] = load_partial16(src + o, len - o);
    }
#pragma unroll
    for (int u = 0; u < MOVE_UNROLL; ++u) {
      const uint32_t o = base + u * 64 * 16;
      if (o >= hi) continue;
      if (o + 16 <= len) {
        stream_store16(dst + o, v[u]);
      } else if (o < len) {
        if (ZERO_PAD)
          stream_store16(dst + o, v[u]);                     // zero padded by load_partial16
        else
          store_partial16(dst + o, v[u], len - o);
      }
    }
  }
}

}  // namespace ckpt
