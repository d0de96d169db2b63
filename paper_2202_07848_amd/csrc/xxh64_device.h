// XXH64 building blocks for gfx950 (device code only).
//
// XXH64 of a message of >= 32 bytes runs four independent accumulators; each
// one consumes the t-th 8-byte little-endian word of every 32-byte stripe:
//     acc <- rotl64(acc + word * PRIME2, 31) * PRIME1
// The rotate makes the recurrence non-associative, so the only parallelism
// inside one message is these four chains.  Everything else (merging the four
// accumulators, the < 32-byte tail, the avalanche) happens once per message.
#pragma once

#include <stdint.h>

namespace ckpt {
namespace xxh {

constexpr uint64_t PRIME1 = 0x9E3779B185EBCA87ull;
constexpr uint64_t PRIME2 = 0xC2B2AE3D27D4EB4Full;
constexpr uint64_t PRIME3 = 0x165667B19E3779F9ull;
constexpr uint64_t PRIME4 = 0x85EBCA77C2B2AE63ull;
constexpr uint64_t PRIME5 = 0x27D4EB2F165667C5ull;

__device__ __forceinline__ uint64_t rotl(uint64_t x, int r) { return (x << r) | (x >> (64 - r)); }

// rotl(x, 31) as two funnel shifts over the register pair (v_alignbit_b32).
__device__ __forceinline__ uint64_t rotl31(uint64_t x) {
  const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
  const uint32_t rlo = __builtin_amdgcn_alignbit(lo, hi, 1);   // lo << 31 | hi >> 1
  const uint32_t rhi = __builtin_amdgcn_alignbit(hi, lo, 1);   // hi << 31 | lo >> 1
  return ((uint64_t)rhi << 32) | rlo;
}

__device__ __forceinline__ uint64_t round(uint64_t acc, uint64_t word) {
  acc += word * PRIME2;
  acc = rotl31(acc);
  return acc * PRIME1;
}

// Initial value of accumulator t (0..3) for seed 0.
__device__ __forceinline__ uint64_t acc_init(int t) {
  return t == 0 ? PRIME1 + PRIME2 : t == 1 ? PRIME2 : t == 2 ? 0ull : 0ull - PRIME1;
}

__device__ __forceinline__ uint64_t merge_acc(uint64_t h, uint64_t acc) {
  h ^= round(0, acc);
  return h * PRIME1 + PRIME4;
}

// Converge the four accumulators of a message that had at least one stripe.
__device__ __forceinline__ uint64_t converge(uint64_t v1, uint64_t v2, uint64_t v3, uint64_t v4) {
  uint64_t h = rotl(v1, 1) + rotl(v2, 7) + rotl(v3, 12) + rotl(v4, 18);
  h = merge_acc(h, v1);
  h = merge_acc(h, v2);
  h = merge_acc(h, v3);
  h = merge_acc(h, v4);
  return h;
}

__device__ __forceinline__ uint64_t tail8(uint64_t h, uint64_t word) {
  h ^= round(0, word);
  return rotl(h, 27) * PRIME1 + PRIME4;
}

__device__ __forceinline__ uint64_t tail4(uint64_t h, uint32_t word) {
  h ^= (uint64_t)word * PRIME1;
  return rotl(h, 23) * PRIME2 + PRIME3;
}

__device__ __forceinline__ uint64_t tail1(uint64_t h, uint8_t byte) {
  h ^= (uint64_t)byte * PRIME5;
  return rotl(h, 11) * PRIME1;
}

__device__ __forceinline__ uint64_t avalanche(uint64_t h) {
  h ^= h >> 33;
  h *= PRIME2;
  h ^= h >> 29;
  h *= PRIME3;
  h ^= h >> 32;
  return h;
}

}  // namespace xxh
}  // namespace ckpt
