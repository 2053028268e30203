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

// ---- format version 2: groups of four entries in three words (two of values, one of 8-bit distances)

typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
constexpr uint32_t kGroupWords = 3;  // words of a group
constexpr uint32_t kRoundWords2 = 64 * kGroupWords;  // words one round of 64 lanes stages (256 entries)

// Inclusive prefix sum over the 64 lanes: four steps inside the rows of 16 lanes (DPP row shifts),
// then the totals of the rows before are added through scalar registers.
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t v, int lane) {
#define FLS_ROW_SHR(n) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x110 + (n), 0xf, 0xf, true)
  FLS_ROW_SHR(1);
  FLS_ROW_SHR(2);
  FLS_ROW_SHR(4);
  FLS_ROW_SHR(8);
#undef FLS_ROW_SHR
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
  const uint32_t r1 = r0 + (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
  const uint32_t r2 = r1 + (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
  const uint32_t row = (uint32_t)lane >> 4;
  return v + (row == 0 ? 0u : row == 1 ? r0 : row == 2 ? r1 : r2);
}

// The four entries of one group: their values go to the locations that the running counter reaches.
// `counter` = the location counter in front of this lane's group; `base` = LDS byte address of the tile
// (or of the padding slot, with counter 0, for a lane past the end of the run, whose loads returned 0).
__device__ __forceinline__ void extract_group(const u32x3& g, uint32_t counter, uint32_t base) {
  typedef __attribute__((address_space(3))) uint16_t* lds_u16_ptr;
  const uint32_t l0 = counter + (g[2] & 0xffu);
  const uint32_t l1 = l0 + ((g[2] >> 8) & 0xffu);
  const uint32_t l2 = l1 + ((g[2] >> 16) & 0xffu);
  const uint32_t l3 = l2 + (g[2] >> 24);
  *(lds_u16_ptr)(uintptr_t)(base + 2u * l0) = (uint16_t)g[0];
  *(lds_u16_ptr)(uintptr_t)(base + 2u * l1) = (uint16_t)(g[0] >> 16);
  *(lds_u16_ptr)(uintptr_t)(base + 2u * l2) = (uint16_t)g[1];
  *(lds_u16_ptr)(uintptr_t)(base + 2u * l3) = (uint16_t)(g[1] >> 16);
}

// Groups of a tile beyond the R rounds that the register ring stages (a tile denser than the kernel
// variant was picked for): loaded and extracted on the spot.  `counter` = the location counter
// behind the staged groups.  Slow, rare, and out of line.
static __device__ __noinline__ void extract_overflow_v2(const uint32_t* words, uint32_t begin, uint32_t end, uint32_t counter,
                                                        unsigned char* tile) {
  const int lane = threadIdx.x & 63;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)tile;
  for (uint32_t i = begin; i < end; i += kRoundWords2) {
    const uint32_t w = i + (uint32_t)lane * kGroupWords;
    u32x3 g = {0u, 0u, 0u};
    if (w < end) g = u32x3{words[w], words[w + 1], words[w + 2]};
    const uint32_t sum = __builtin_amdgcn_sad_u8(g[2], 0u, 0u);
    const uint32_t incl = wave_prefix_sum(sum, lane);
    // lanes past the end hold zeros: they would write a zero where the counter stands, so they get the padding slot
    extract_group(g, w < end ? counter + incl - sum : 0u, w < end ? tile_addr : tile_addr + (uint32_t)kTileBytes);
    counter += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
  }
}

}  // namespace fls
