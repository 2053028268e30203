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
  uint32_t base;    // tile whose offset lane 0 holds
  uint32_t window;  // this lane's offset
  int lane;

  // The two halves of a reload; between them the caller may do work that does not need the offsets.
  __device__ __forceinline__ void request(uint32_t t) {
    base = t;
    const uint32_t idx = t + (uint32_t)lane;
    window = offs[idx < T ? idx : T];
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

}  // namespace fls
