// Pieces of the tile walk shared by the sparse kernels: the TileOffsets window and the slow path
// for tiles denser than the register ring stages.  gfx950 only.
#pragma once
#include "fls_device.h"

namespace fls {

// TileOffsets of 64 consecutive tiles, one per lane of a VGPR, picked with v_readlane: stepping
// to the next tile then costs no memory access (a load per tile, scalar or vector, would put its
// latency on the critical path of every tile).
struct OffsetWindow {
  const uint32_t* offs;
  uint32_t T;       // index of the last entry that differs from its successor (offs[T] = total words)
  uint32_t total;   // words in NonZeros: no offset is taken to lie beyond (a damaged blob must not send loads elsewhere)
  uint32_t base;    // tile whose offset lane 0 holds
  uint32_t window;  // this lane's offset
  int lane;

  // The two halves of a reload; between them the caller may do work that does not need the offsets.
  __device__ __forceinline__ void request(uint32_t t) {
    base = t;
    const uint32_t idx = t + (uint32_t)lane;
    const uint32_t v = offs[idx < T ? idx : T];
    window = v < total ? v : total;
  }
  __device__ __forceinline__ void arrive() {
    // Wait for the value here, inside the (rare) reload path: if its arrival were first needed
    // after the paths join, every tile would pay a full "wait for all loads".
    asm volatile("" : "+v"(window));
  }
  __device__ __forceinline__ void load(uint32_t t) {
    request(t);
    arrive();
  }
  // offsets of tiles t and t + 1; reloads the window when t or t + 1 falls outside it - t may lie
  // before the window: the load side looks a few tiles past the end of a piece, which can move the
  // window beyond the tile the next piece starts with
  __device__ __forceinline__ void get(uint32_t t, uint32_t& begin, uint32_t& end) {
    if (t - base > 62u) load(t);
    begin = (uint32_t)__builtin_amdgcn_readlane((int)window, (int)(t - base));
    end = (uint32_t)__builtin_amdgcn_readlane((int)window, (int)(t + 1 - base));
    if (end < begin) end = begin;  // offsets that do not ascend: an empty run
  }
};

// Words of a tile beyond the R*256 that the register ring stages (a tile denser than the kernel
// variant was picked for): loaded and extracted on the spot.  Slow, rare, and out of line.
static __device__ __noinline__ void extract_overflow(const uint32_t* words, uint32_t begin, uint32_t end, unsigned char* tile) {
  const int lane = threadIdx.x & 63;
  for (uint32_t i = begin + lane * 4; i < end; i += 256) {
    const u32x4 w = *(const u32x4*)(words + i);
#pragma unroll
    for (int j = 0; j < 4; ++j) *(uint16_t*)(tile + ((w[j] & 0xffffu) << 1)) = (uint16_t)(w[j] >> 16);
  }
}

// ---- format version 2: groups of four entries in three words (two of values, one of locations)

typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
constexpr uint32_t kGroupWords = 3;  // words of a group
constexpr uint32_t kRoundWords2 = 64 * kGroupWords;  // words one round of 64 lanes stages (256 entries)

// Format version 2: the four entries of one group (value0 | value1 << 16, value2 | value3 << 16, loc0 | dist1 << 12 |
// dist2 << 18 | dist3 << 24).  The values go to their locations in the LDS tile at byte address `base` (or of the
// padding slot, for a lane past the end of the run, whose loads returned 0); returns the four byte addresses,
// which is all the later re-zeroing needs.  A group decodes by itself: three additions, nothing from other lanes.
__device__ __forceinline__ u32x4 extract_group(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t base, bool store = true) {
  typedef __attribute__((address_space(3))) uint16_t* lds_u16_ptr;
  const uint32_t a0 = base + 2u * (w2 & 0xfffu);
  const uint32_t a1 = a0 + 2u * ((w2 >> 12) & 0x3fu);
  const uint32_t a2 = a1 + 2u * ((w2 >> 18) & 0x3fu);
  const uint32_t a3 = a2 + 2u * ((w2 >> 24) & 0x3fu);
  if (store) {  // (false in the latency-breakdown builds that erase the extraction)
    *(lds_u16_ptr)(uintptr_t)a0 = (uint16_t)w0;
    *(lds_u16_ptr)(uintptr_t)a1 = (uint16_t)(w0 >> 16);
    *(lds_u16_ptr)(uintptr_t)a2 = (uint16_t)w1;
    *(lds_u16_ptr)(uintptr_t)a3 = (uint16_t)(w1 >> 16);
  }
  return u32x4{a0, a1, a2, a3};
}

// Groups of a tile beyond the R rounds that the register ring stages (a tile denser than the kernel
// variant was picked for): loaded and extracted on the spot.  Slow, rare, and out of line.
static __device__ __noinline__ void extract_overflow_v2(const uint32_t* words, uint32_t begin, uint32_t end, unsigned char* tile) {
  const int lane = threadIdx.x & 63;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)tile;
  for (uint32_t w = begin + (uint32_t)lane * kGroupWords; w < end; w += kRoundWords2)
    extract_group(words[w], words[w + 1], words[w + 2], tile_addr);
}

}  // namespace fls
