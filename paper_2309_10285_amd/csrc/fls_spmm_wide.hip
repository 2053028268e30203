// fls_spmm for more than 32 columns: 64 columns per pass (Flash-LLM's kernel for its widest batch
// sizes, re-cut for gfx950).
//
// A workgroup has four waves, one per SIMD with the whole register file (128 accumulator
// registers, a deep ring of tiles in flight), and takes four row bands (one per wave) x one K slice:
// the four waves walk the same K tiles side by side, so the X rows of a tile are fetched once per
// workgroup - straight from the caller's X into LDS, a loop body (4 or 8 tiles) ahead, by all four
// waves together - and every wave reads its B fragments from there.  With 64 columns a tile needs
// 4 KB of X against some 1.6 - 5 KB of compressed W, and fragments fetched from L2 by every wave
// for itself cost more vector-memory time than the stream of words.  The waves meet at one barrier
// per loop body (after storing their part of the next X chunk, before reading from it); everything
// else of the tile loop is private to a wave.
//
// Work is cut as (group of four bands) x (K slice), S slices per group so that the grid fills the
// CUs.  With S = 1 a wave's sum is its band's result and goes to C directly, otherwise to a
// partial-sum area [band][column group][slice] that a second, small kernel adds up in slice order and converts
// (no flags, no waiting between workgroups, deterministic).
//
// Inside a wave the stages are those of the narrow kernel - register ring of tiles, extraction by
// 2 B LDS stores, 16 B fragment reads - software-pipelined by hand, since no second wave shares the
// SIMD: the MFMAs of a tile are asm statements in a fixed order with the step's other work (re-zero
// the tile, extract the next one, read its fragments, refill the ring, X chunk traffic) dealt out
// between them, and they work on fragments that were read during the step before.  The shape is
// v_mfma_f32_32x32x16_f16 (16 per tile).
#include <atomic>
#include <type_traits>

#include "fls_device.h"
#include "fls_launch.h"
#include "fls_tile.h"

// Latency-breakdown builds (see fls_spmm.hip): 2 no MFMA, 4 no extract, 8 no re-zeroing, 16 no LDS
// fragment reads, 32 no global loads of the words, 256 no X traffic (loads, LDS stores, B fragment
// reads).  0 in the library.
#ifndef FLS_ABLATE
#define FLS_ABLATE 0
#endif

namespace fls {

constexpr int kWideWaves = 4;                   // four bands, one wave each
constexpr int kWideNB = 4;                      // 16-column blocks per pass
constexpr int kWideTileLds = kTileBytes + 16;   // a wave's tile + the slot padding words land in

// X in MFMA fragment order, for the dense 64-column pass: block (K tile kt, column block nb) holds,
// for lane l = 16 g + c, the 8 halves X[32 kt + 8 g .. +7][16 nb + c] (zeros for columns past N).
// One wave per pair of K tiles and column block, so that it uses the whole 128 B line of each of
// its 16 columns; loads are quad-contiguous (lane j reads column j >> 2, chunk j & 3), stores go to
// the fragment position.
__global__ __launch_bounds__(256) void xpack_kernel(const _Float16* X, _Float16* Xp, uint32_t K, uint32_t N, uint32_t units,
                                                    uint32_t blocks) {
  const uint32_t u = blockIdx.x * 4 + (threadIdx.x >> 6);  // (pair of K tiles, column block)
  if (u >= units) return;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t pair = u / blocks, nb = u - pair * blocks;
  const uint32_t c = lane >> 2, g = lane & 3u;
  const uint32_t col = nb * 16u + c;
  const uint32_t KT = K / kTileK;
#pragma unroll
  for (uint32_t h = 0; h < 2; ++h) {
    const uint32_t kt = 2u * pair + h;
    if (kt < KT) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (col < N) v = *(const u32x4*)(X + (size_t)col * K + kt * kTileK + g * 8u);
      *(u32x4*)(Xp + (((size_t)kt * blocks + nb) * 64u + g * 16u + c) * 8u) = v;
    }
  }
}

// Compile-time loop: f(integral_constant<int, I>) for I in [B, E).
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

// acc += a . b with the accumulator kept where it is (sixteen AGPRs): as an asm statement, so that
// the instruction keeps its place between the memory operations around it.
//
// The 64-column pass multiplies with v_mfma_f32_32x32x16_f16 rather than 16x16x32: half as many
// instructions for the same work, each leaving eight issue slots in its shadow.  Operand layouts
// of the 32x32x16 shape, lane l = 32 h + c:
//   A: row c of the 32-row block, the 8 k of chunk h of the 16-k step;  B: column c, the same 8 k;
//   C/D: column c, rows 8 q + 4 h + (0..3) in registers 4 q .. 4 q + 3, q = 0..3.
// A and B hold the same thing in the same lanes, so either operand can be the W block.  The pass
// computes the transposed product, X block (A) times W block (B): the chip's clock under this
// kernel is set by power, the matrix cores draw less when the operand that is mostly zeros is B,
// and the call is 3 % faster for it (measured; with X all zeros instead of random values the same
// instruction stream runs 15 - 18 % faster still, with W's values all equal 2 %).  An accumulator block
// is therefore 32 columns of X (its rows) by 32 rows of W (its columns).
typedef float float16v __attribute__((ext_vector_type(16)));
__device__ __forceinline__ void mfma_in_place(float16v& acc, const half8& a, const half8& b) {
  asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
constexpr int kRowBlocks32 = kTileM / 32;  // 32-row blocks of a tile
constexpr int kColBlocks32 = 2;            // 32-column blocks of a group of 64 columns
constexpr int kSteps16 = kTileK / 16;      // 16-k steps of a tile

// Converts a wave's 128 x 64 accumulators (32x32 layout, transposed: see above) to fp16 and stores them
// to column-major C: register 4 q + r of block (rb, cb) is row 32 rb + c of the band, column
// 32 cb + 8 q + 4 h + r of the group - 64 contiguous bytes of C per store and half wave.
template <int CB>
__device__ __forceinline__ void store_band32(_Float16* C, uint32_t M, uint32_t N, uint32_t n0,
                                             const float16v (&acc)[kRowBlocks32][CB], uint32_t band, int lane) {
  const uint32_t c = lane & 31, h = lane >> 5;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t n = n0 + cb * 32 + q * 8 + h * 4 + r;
        if (n < N) {
#pragma unroll
          for (int rb = 0; rb < kRowBlocks32; ++rb)
            C[(size_t)n * M + band * kTileM + rb * 32 + c] = (_Float16)acc[rb][cb][4 * q + r];
        }
      }
}

// LDS of a workgroup: two X chunks (a chunk = the NS K tiles of a loop body x 64 columns, 4 KB per
// tile), then the four waves' tiles.  The chunks come first so that the two lie 2^k apart and a
// body switches between them by flipping one address bit.
template <int NS>
constexpr int wide_lds_bytes() { return 2 * NS * 4096 + kWideWaves * kWideTileLds; }

// FMT = format version of the blob (see fls_spmm.hip): a stage register holds a round's four words
// (version 1) or a group's three (version 2) and, once extracted, the four LDS addresses they went to.
// CB = 32-column blocks that are multiplied: 2, or 1 for a call of at most 32 columns that takes this
// pass for the sake of sharing X between four bands (the X chunk keeps its 64-column shape; the
// columns past N cost no memory traffic, and nothing of the second block is read, multiplied or stored).
template <int R, int NS, int FMT, int CB>
__global__ __launch_bounds__(kWideWaves * 64) void spmm_wide_kernel(WideParams p) {
  constexpr int NB = kWideNB;
  constexpr uint32_t kRoundWords = FMT == 2 ? kRoundWords2 : 256u;  // words one round of 64 lanes stages
  static_assert(NS == 4 || NS == 8, "a body is 4 or 8 tiles");
  // X loads of a chunk that this wave issues.  With one column block and eight-tile bodies a wave has a tile pair to
  // itself and its loads e >= 4 are columns 32 - 63: never issued.  (With four-tile bodies two waves share a pair and
  // the odd one's loads are those columns; they are issued and leave the buffer: zeros, no memory traffic.)
  constexpr int kXLoads = CB == 1 && NS == 8 ? 4 : NS;
  constexpr uint32_t kChunkBytes = NS * 4096u;
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // The workgroup: four row bands (one per wave) x one K slice, which all four waves walk together,
  // x one group of 64 columns.  A call of more than 64 columns is one launch over all its column
  // groups (with G groups the chip is filled by G times fewer K slices, so G times fewer partial
  // sums per column go through memory than with a launch per group).  The G workgroups that stream
  // the same words get workgroup ids 8 apart: consecutive ids go to the chip's eight XCDs in turn,
  // so those G land on one XCD, one after the other, and all but the first find the words in its L2.
  const uint32_t pairs = ((p.bands + 3u) / 4u) * p.S;  // (group of bands, slice) pairs
  const uint32_t cg = (blockIdx.x >> 3) % p.G, pair = ((blockIdx.x >> 3) / p.G) * 8u + (blockIdx.x & 7u);
  if (pair >= pairs) return;  // the grid is rounded up to a multiple of eight pairs
  const uint32_t quad = pair / p.S, slice = pair - quad * p.S;
  const uint32_t n0 = p.n0 + cg * 64u;
  const uint32_t band = quad * 4 + wave;
  const bool active = band < p.bands;  // a wave past the last band loads no words but shares the X work
  const uint32_t KT = p.KT, T = p.bands * KT;
  // the slice: whole bodies of NS tiles, cut evenly; the K tiles that fill no body go to the last slice
  const uint32_t bodies_all = KT / NS;
  const uint32_t b0 = (uint32_t)((uint64_t)slice * bodies_all / p.S), b1 = (uint32_t)((uint64_t)(slice + 1) * bodies_all / p.S);
  const uint32_t bodies = b1 - b0;
  const uint32_t k0 = b0 * NS, k1 = k0 + bodies * NS;          // tiles of the pipelined loop
  const uint32_t ktail = slice + 1 == p.S ? KT : k1;           // ... and of the plain loop behind it
  const uint32_t t0 = active ? band * KT + k0 : T;
  const uint32_t ntiles = active ? bodies * NS : 0;            // tiles this wave loads words for

  unsigned char* tile = lds + 2 * kChunkBytes + wave * kWideTileLds;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;

  float16v acc[kRowBlocks32][CB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks32; ++rb)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;

  // ---- X, from the caller's layout into LDS, once per workgroup and K tile.
  // A load instruction takes 8 columns x 64 k (two K tiles): lane l reads the 16 B of column
  // l >> 3, k chunk l & 7, so eight neighbouring lanes read one whole 128 B line.  The chunk's
  // 4 NS such loads are split evenly over the four waves (NS each).  The descriptor ends after column N - 1
  // (the column is in the per-lane offset, which is what the bounds check of a raw buffer looks
  // at), so columns that pad the pass up to 64 read as zero.
  // In LDS a K tile is four 1 KB blocks, one per (32-column block cb, 16-k step ks), of 64 slots of
  // 16 B: the B fragment of MFMA lane 32 h + c sits in slot 32 h + (c ^ (4 ks + 2 h + 8 tp)), tp = the
  // tile's parity.  The MFMA read (16 neighbouring lanes: 16 neighbouring slots in some order) and
  // the store of a loaded register (the 8 k chunks of a column: 8 different 16 B bank groups) are both
  // free of bank conflicts.
  const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)p.X, 0, (int)(p.N * p.K * 2u), kBufferFlags);
  const uint32_t c8 = (uint32_t)lane >> 3, ch = (uint32_t)lane & 7u;
  const uint32_t colgrp_bytes = 16u * p.K;  // eight columns further
  // This wave's loads of a chunk are q = wave * NS + e, e < NS: tile pair q >> 3, column group q & 7;
  // NS is 4 or 8, so the pair and the group's upper part are the wave's (folded into the per-lane
  // offsets below) and e only adds to the group.  Everything that may leave the buffer - the column and,
  // for the chunk requested past the end of K, the k offset - is in the per-lane offset.
  const uint32_t pair_w = (wave * NS) >> 3, grp_w = (wave * NS) & 7u;
  const uint32_t xg_lane = ((n0 + 8u * grp_w + c8) * p.K + pair_w * 64u + ch * 8u) * 2u;  // + e column groups + the chunk's k
  // LDS byte address of this lane's store of load e, by e & 3 (the column group inside its 32-column
  // block), in the chunk to fill: k chunk ch of the tile pair = tile parity ch >> 2, step (ch >> 1) & 1,
  // lane half ch & 1
  uint32_t xw_addr[4];
#pragma unroll
  for (int e3 = 0; e3 < 4; ++e3)
    xw_addr[e3] = (uint32_t)(uintptr_t)lds + kChunkBytes + pair_w * 8192u + (grp_w >> 2) * 2048u + (ch >> 2) * 4096u +
                  ((ch >> 1) & 1u) * 1024u + (32u * (ch & 1u) + ((8u * e3 + c8) ^ (2u * ch))) * 16u;
  // LDS byte address of this lane's fragment read by tile parity and 16-k step, in the chunk in use and in the other one
  uint32_t xr_addr[2][kSteps16], xr_other[2][kSteps16];
  {
    const uint32_t c = (uint32_t)lane & 31u, h = (uint32_t)lane >> 5;
#pragma unroll
    for (int tp = 0; tp < 2; ++tp)
#pragma unroll
      for (int ks = 0; ks < kSteps16; ++ks) {
        xr_addr[tp][ks] = (uint32_t)(uintptr_t)lds + ks * 1024u + (32u * h + (c ^ (4u * ks + 2u * h + 8u * tp))) * 16u;
        xr_other[tp][ks] = xr_addr[tp][ks] + kChunkBytes;
      }
  }
  typedef __attribute__((address_space(3))) u32x4* lds_v4_ptr;
  typedef __attribute__((address_space(3))) const half8* lds_h8_ptr;
  // loads e0, e0 + 1 of this wave's share of the chunk that starts at K tile kt
  auto xload2 = [&](u32x4(&xs)[NS], int e0, uint32_t kt) {
#pragma unroll
    for (int e = e0; e < e0 + 2; ++e)
      xs[e] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, xg_lane + (uint32_t)e * colgrp_bytes + kt * 64u, 0, 0);
  };
  // ... and their stores into the chunk to fill
  auto xstore2 = [&](const u32x4(&xs)[NS], int e0) {
#pragma unroll
    for (int e = e0; e < e0 + 2; ++e) *(lds_v4_ptr)(uintptr_t)(xw_addr[e & 3] + (uint32_t)(e >> 2) * 2048u) = xs[e];
  };
  // B fragment (column block cb, step ks) of tile `it` (0 .. NS - 1) of the chunk in use (`other`: of the
  // other chunk, the next body's)
  auto xfrag = [&](int it, int cb, int ks, bool other) {
    const uint32_t base = other ? xr_other[it & 1][ks] : xr_addr[it & 1][ks];
    return *(lds_h8_ptr)(uintptr_t)(base + (uint32_t)it * 4096u + (uint32_t)cb * 2048u);
  };
  // all four waves have stored their part of the next chunk and are done reading the present one
  auto chunk_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
  auto flip_chunks = [&]() {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      xw_addr[j] ^= kChunkBytes;
      xr_addr[j >> 1][j & 1] ^= kChunkBytes;
      xr_other[j >> 1][j & 1] ^= kChunkBytes;
    }
  };

  // ---- W
  // TileOffsets: a window of 64 entries in a VGPR (lane i = entry first + i), replaced once per
  // body by the window that was requested a body earlier - an unconditional load per NS tiles, so
  // stepping from tile to tile costs v_readlane (with a constant lane) and no wait.
  const uint32_t* offs = p.offs;
  auto window_at = [&](uint32_t first) {
    const uint32_t idx = first + (uint32_t)lane;
    return offs[idx < T ? idx : T];
  };
  uint32_t window = window_at(t0);
  // Request of the tile whose offsets are lanes i, i + 1 of the window, and which is tile `rel` of
  // the run: n = words staged (0 past the run: nothing loaded, nothing extracted).
  auto issue = [&](u32x4(&s)[R], uint32_t& n, int i, uint32_t rel) {
    const uint32_t begin = (uint32_t)__builtin_amdgcn_readlane((int)window, i);
    const uint32_t end = (uint32_t)__builtin_amdgcn_readlane((int)window, i + 1);
    n = end - begin;
    if (n > R * kRoundWords) n = R * kRoundWords;
    if (rel >= ntiles) n = 0;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(p.words + begin), 0, (int)(n * 4u), kBufferFlags);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if constexpr (FMT == 2) {
        u32x3 g = {(uint32_t)lane, 1u, 0x01041000u};
        if (!(FLS_ABLATE & 32)) g = __builtin_amdgcn_raw_buffer_load_b96(rsrc, (r * 64 + lane) * 12, 0, kAuxNonTemporal);
        s[r] = u32x4{g[0], g[1], g[2], 0u};
      } else {
        if (FLS_ABLATE & 32) s[r] = u32x4{(uint32_t)lane, 1u, 2u, 3u};
        else s[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (r * 64 + lane) * 16, 0, kAuxNonTemporal);
      }
    }
  };

  // extract (Alg. 2), branch-free so that a step is one basic block: lanes past the end of the
  // run (their loads returned 0: location 0, value 0) get the slot that padding words go to as
  // their base.  The words are then replaced by the LDS addresses they went to, which is all the
  // later re-zeroing needs.  (No tile has more than R * 256 words here: see `densest` below.)
  typedef __attribute__((address_space(3))) uint16_t* lds_u16_ptr;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)tile;  // LDS addresses are the low 32 bits
  auto extract = [&](u32x4(&s)[R], uint32_t n) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if constexpr (FMT == 2) {
        const uint32_t base = (r * 64 + lane) * kGroupWords < n ? tile_addr : tile_addr + (uint32_t)kTileBytes;
        s[r] = extract_group(s[r][0], s[r][1], s[r][2], base, !(FLS_ABLATE & 4));
      } else {
        const uint32_t base = (r * 64 + lane) * 4u < n ? tile_addr : tile_addr + (uint32_t)kTileBytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t w = s[r][j];
          const uint32_t addr = scatter_addr(w, base);
          if (FLS_ABLATE & 4) asm volatile("" ::"v"(w));
          else *(lds_u16_ptr)(uintptr_t)addr = (uint16_t)(w >> 16);
          s[r][j] = addr;
        }
      }
    }
  };

  // A fragment (32-row block rb, 16-k step ks): row 32 rb + (lane & 31), k chunk 2 ks + (lane >> 5) of the
  // [k chunk][row][8] tile
  const unsigned char* frag = tile + ((lane >> 5) * kTileM + (lane & 31)) * 16;
  auto afrag = [&](int rb, int ks) { return *(const half8*)(frag + ks * 4096 + rb * 512); };

  // rst_smem.  Sparse tiles (R <= 4: at most 1024 words) are re-zeroed by storing zeros where
  // their words went - as many 2 B stores as the extraction - instead of clearing all 8 KB.
  constexpr bool kUnscatter = R <= 4;

  // One step = one tile t, tile `it` of its body.  On entry the tile's A fragments are in `fa` and its B
  // fragments in `fb` (both read from LDS during the step before), its words - LDS addresses by now -
  // in stage `cur`.  The 16 MFMAs of tile t are issued one by one with the step's other work dealt
  // out between them in a fixed order (a wave alone on its SIMD issues in order: what stands between
  // two MFMAs runs in the shadow of the first): this wave's part of the X chunk of the next body (loads
  // in the first half of a body, stores into LDS in the second), re-zero tile t, extract tile t + 1
  // (stage `nxt`), read its fragments into `fan` / `fbn`, refill stage `cur`.  LDS executes a wave's
  // operations in order, so no wait separates re-zeroing, extraction and the fragment reads; the
  // MFMAs never wait for anything issued in their own step.  The last step of a body meets the other
  // waves before it reads B fragments from the chunk they filled together.
  constexpr int kFragsA = kSteps16 * kRowBlocks32, kFragsB = kSteps16 * CB;
  auto step = [&](auto it_, u32x4(&cur)[R], uint32_t& cn, uint32_t rel, u32x4(&nxt)[R], uint32_t nn, u32x4(&xs)[NS],
                  uint32_t kt_next, const half8(&fa)[kFragsA], const half8(&fb)[kFragsB], half8(&fan)[kFragsA],
                  half8(&fbn)[kFragsB]) {
    constexpr int it = decltype(it_)::value;
    constexpr int kZ = kUnscatter ? 4 * R : kTileBytes / 1024;  // re-zeroing operations
    constexpr int kE = 5 * R;                                   // extraction: per round a base select and four words
    constexpr int kOps = 1 + kZ + kE + 1 + kFragsA + kFragsB + 1;
    constexpr int kMfmas = kSteps16 * kRowBlocks32 * CB;
    uint32_t ebase = 0, eaddr = 0, ekeep = 0;
    auto other = [&](auto o_) {
      constexpr int o = decltype(o_)::value;
      if constexpr (o == 0) {
        // (with one column block only the chunk's first four column groups hold columns of the call: the
        // wave's loads e >= 4 would fetch nothing but zeros)
        if (FLS_ABLATE & 256) {
        } else if constexpr (it < NS / 2) {
          if constexpr (2 * it < kXLoads) xload2(xs, 2 * it, kt_next);
        } else {
          if constexpr (2 * (it - NS / 2) < kXLoads) xstore2(xs, 2 * (it - NS / 2));
        }
      } else if constexpr (o < 1 + kZ) {
        constexpr int z = o - 1;
        if (FLS_ABLATE & 8) {
        } else if constexpr (kUnscatter) {
          *(lds_u16_ptr)(uintptr_t)cur[z / 4][z % 4] = (uint16_t)0;
        } else {
          *(u32x4*)(tile + z * 1024 + lane * 16) = zero4;
        }
      } else if constexpr (o < 1 + kZ + kE) {
        constexpr int r = (o - 1 - kZ) / 5, j = (o - 1 - kZ) % 5 - 1;
        if constexpr (j < 0) {
          ebase = (r * 64 + lane) * (FMT == 2 ? kGroupWords : 4u) < nn ? tile_addr : tile_addr + (uint32_t)kTileBytes;
        } else if constexpr (FMT == 2) {
          // entry j of the lane's group: its address is the one before plus a 6-bit distance (the first: the
          // group's 12-bit location); the words make room for the addresses as they are used up
          const uint32_t w2 = nxt[r][2];
          if constexpr (j == 0) eaddr = ebase + 2u * (w2 & 0xfffu);
          else eaddr = eaddr + 2u * ((w2 >> (6 + 6 * j)) & 0x3fu);
          const uint32_t v = nxt[r][j >> 1];
          if (FLS_ABLATE & 4) asm volatile("" ::"v"(v));
          else *(lds_u16_ptr)(uintptr_t)eaddr = (j & 1) ? (uint16_t)(v >> 16) : (uint16_t)v;
          if constexpr (j == 0) nxt[r][3] = eaddr;
          else if constexpr (j == 1) nxt[r][0] = eaddr;
          else if constexpr (j == 2) ekeep = eaddr;
          else {
            nxt[r][1] = ekeep;
            nxt[r][2] = eaddr;
          }
        } else {
          const uint32_t w = nxt[r][j];
          const uint32_t addr = scatter_addr(w, ebase);
          if (FLS_ABLATE & 4) asm volatile("" ::"v"(w));
          else *(lds_u16_ptr)(uintptr_t)addr = (uint16_t)(w >> 16);
          nxt[r][j] = addr;
        }
      } else if constexpr (o == 1 + kZ + kE) {
        if constexpr (it == NS - 1) chunk_barrier();
      } else if constexpr (o < 2 + kZ + kE + kFragsA) {
        constexpr int j = o - 2 - kZ - kE;  // step-major: the fragments of the first 16 k come first
        if (FLS_ABLATE & 16) fan[j] = fb[j % kFragsB];
        else fan[j] = afrag(j % kRowBlocks32, j / kRowBlocks32);
      } else if constexpr (o < 2 + kZ + kE + kFragsA + kFragsB) {
        constexpr int j = o - 2 - kZ - kE - kFragsA;
        if (FLS_ABLATE & 256) fbn[j] = fb[j];
        else fbn[j] = xfrag((it + 1) % NS, j % CB, j / CB, it == NS - 1);
      } else {
        issue(cur, cn, it, rel);
      }
    };
    // MFMA s: 16-k step s / 8, row block (s % 8) / 2, column block s % 2 - the two MFMAs of an
    // accumulator lie eight apart
    static_for<0, kMfmas>([&](auto s_) {
      constexpr int s = decltype(s_)::value;
      constexpr int ks = s / (kRowBlocks32 * CB), rb = (s / CB) % kRowBlocks32, cb = s % CB;
      if (FLS_ABLATE & 2) acc[rb][cb][0] += (float)fa[ks * kRowBlocks32 + rb][0] * (float)fb[ks * CB + cb][0];
      else mfma_in_place(acc[rb][cb], fb[ks * CB + cb], fa[ks * kRowBlocks32 + rb]);
      static_for<s * kOps / kMfmas, (s + 1) * kOps / kMfmas>(other);
    });
  };

  // B fragments straight from the caller's X, for the plain loop: lane 32 h + c takes column c of a
  // 32-column block, k chunk h of a 16-k step
  const uint32_t xd_lane = ((n0 + ((uint32_t)lane & 31u)) * p.K + ((uint32_t)lane >> 5) * 8u) * 2u;
  // One tile the plain way: words straight from memory into LDS, fragments, re-zero, MFMAs.
  auto plain_tile = [&](uint32_t t, uint32_t kt) {
    const uint32_t begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)offs[t]);
    const uint32_t end = (uint32_t)__builtin_amdgcn_readfirstlane((int)offs[t + 1]);
    if constexpr (FMT == 2) {
      for (uint32_t i = begin + (uint32_t)lane * kGroupWords; i < end; i += kRoundWords2)
        extract_group(p.words[i], p.words[i + 1], p.words[i + 2], tile_addr);
    } else {
      for (uint32_t i = begin + (uint32_t)lane * 4u; i < end; i += 256u) {
        const u32x4 w = *(const u32x4*)(p.words + i);
#pragma unroll
        for (int j = 0; j < 4; ++j) *(uint16_t*)(tile + ((w[j] & 0xffffu) << 1)) = (uint16_t)(w[j] >> 16);
      }
    }
    half8 fa[kFragsA], fb[kFragsB];
#pragma unroll
    for (int j = 0; j < kFragsB; ++j)
      fb[j] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(
                                            xrsrc, xd_lane + (j % CB) * 4u * colgrp_bytes + kt * 64u + (j / CB) * 32u, 0, 0));
#pragma unroll
    for (int j = 0; j < kFragsA; ++j) fa[j] = afrag(j % kRowBlocks32, j / kRowBlocks32);
#pragma unroll
    for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
#pragma unroll
    for (int ks = 0; ks < kSteps16; ++ks)
#pragma unroll
      for (int rb = 0; rb < kRowBlocks32; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
          acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[ks * CB + cb], fa[ks * kRowBlocks32 + rb], acc[rb][cb], 0, 0, 0);
  };

  // The launcher picks R from the header the host remembers for this blob address.  If the memory
  // holds a denser blob by now (one written there without the library's knowing), the ring cannot
  // stage its tiles: the whole grid then takes the plain loop for all its tiles, which is slow and right.
  const uint32_t densest = offs[kHeaderMaxTileWords - kHeaderWords];
  uint32_t kplain = k0;  // first K tile of the plain loop
  if (densest <= R * kRoundWords && bodies > 0) {
    kplain = k1;
    // Prologue: the first chunk of X into LDS, the ring of words filled, the first tile in LDS and
    // its fragments in registers.  (The next window of offsets is requested before the ring's loads,
    // as in the loop: the wait for a window then never covers the ring loads issued after it.)
    u32x4 s[NS][R];
    uint32_t sn[NS];
    u32x4 xs[NS];
    uint32_t next_window = window_at(t0 + NS);
#pragma unroll
    for (int e = 0; e < kXLoads; e += 2) xload2(xs, e, k0);
#pragma unroll
    for (int i = 0; i < NS; ++i) issue(s[i], sn[i], i, (uint32_t)i);
    flip_chunks();  // the stores below fill the chunk the loop starts with
#pragma unroll
    for (int e = 0; e < kXLoads; e += 2) xstore2(xs, e);
    flip_chunks();
    extract(s[0], sn[0]);
    chunk_barrier();
    half8 fa0[kFragsA], fa1[kFragsA], fb0[kFragsB], fb1[kFragsB];
#pragma unroll
    for (int j = 0; j < kFragsA; ++j) fa0[j] = afrag(j % kRowBlocks32, j / kRowBlocks32);
#pragma unroll
    for (int j = 0; j < kFragsB; ++j) fb0[j] = xfrag(0, j % CB, j / CB, false);
    uint32_t rel = NS;       // first tile the body's refills ask for
    uint32_t kt_next = k0;   // first K tile of the chunk the body loads
    for (uint32_t body = 0; body < bodies; ++body) {
      // refills of this body ask for tiles rel ... rel + NS - 1 of the run: lanes 0 ... NS of the window
      // that starts at tile t0 + rel
      window = next_window;
      next_window = window_at(t0 + rel + NS);
      kt_next += NS;
      static_for<0, NS / 2>([&](auto h_) {
        constexpr int i = 2 * decltype(h_)::value, i1 = i + 1, i2 = (i + 2) % NS;
        step(std::integral_constant<int, i>{}, s[i], sn[i], rel + i, s[i1], sn[i1], xs, kt_next, fa0, fb0, fa1, fb1);
        step(std::integral_constant<int, i1>{}, s[i1], sn[i1], rel + i1, s[i2], sn[i2], xs, kt_next, fa1, fb1, fa0, fb0);
      });
      rel += NS;
      flip_chunks();
    }
    // the last MFMAs' results are read by ordinary instructions next: the accumulators are asm
    // operands, so the wait states between the two are given here by hand
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  }
  // K tiles that fill no body (and everything, for a blob denser than the ring was picked for)
  if (active)
    for (uint32_t kt = kplain; kt < ktail; ++kt) plain_tile(band * KT + kt, kt);
  if (!active) return;

  // The band's result for the slice: to C directly when the slice is all of K, else to the
  // partial-sum area [band][slice] that a second, small kernel adds up in slice order.
  if (p.S == 1) {
    store_band32<CB>(p.C, p.M, p.N, n0, acc, band, lane);
  } else {
    // [band][column group][slice][column block][row block][q][lane] float4: row (lane & 31) of the row block,
    // columns 8 q + 4 (lane >> 5) + (0..3) of the column block
    float4v* dst = (float4v*)p.parts + ((size_t)((band * p.G + cg) * p.S + slice) * (NB * kRowBlocks)) * 64 + lane;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int rb = 0; rb < kRowBlocks32; ++rb)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          dst[((cb * kRowBlocks32 + rb) * 4 + q) * 64] =
              float4v{acc[rb][cb][4 * q], acc[rb][cb][4 * q + 1], acc[rb][cb][4 * q + 2], acc[rb][cb][4 * q + 3]};
  }
}

// Adds the S partial results of every band in slice order, converts, writes C.  One wave per 1 KB
// unit of a band's partial result (32 units; 16 when the pass multiplied one column block): S loads of 16 B per lane, all issued before the first is
// used.  A unit is (column block of 16, row block of 16) in the 16x16 accumulator layout of the dense
// pass, (column block of 32, row block of 32, q) in the 32x32 layout of the sparse pass (LAYOUT32).
template <bool LAYOUT32>
__global__ __launch_bounds__(256) void wide_reduce_kernel(WideParams p) {
  const uint32_t per_band = LAYOUT32 ? p.cb * 16u : (uint32_t)(kWideNB * kRowBlocks);  // units of a band and column group that hold sums
  const uint32_t unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= p.bands * p.G * per_band) return;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t bg = unit / per_band, sub = unit - bg * per_band;  // (band, column group), block
  const uint32_t band = bg / p.G, n0 = p.n0 + (bg - band * p.G) * 64u;
  const float4v* src = (const float4v*)p.parts + ((size_t)bg * p.S * (kWideNB * kRowBlocks) + sub) * 64 + lane;
  float4v sum = {0.f, 0.f, 0.f, 0.f};
  for (uint32_t s0 = 0; s0 < p.S; s0 += 8) {
    float4v v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t s = s0 + j < p.S ? s0 + j : s0;
      v[j] = src[(size_t)s * (kWideNB * kRowBlocks) * 64];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < p.S) sum += v[j];
  }
  if (LAYOUT32) {
    // four columns of one row per lane: 64 contiguous bytes of C per store and half wave
    const uint32_t n = n0 + (sub / 16u) * 32u + (sub % 4u) * 8u + (lane >> 5) * 4u;
    const uint32_t row = ((sub / 4u) % 4u) * 32u + (lane & 31u);
#pragma unroll
    for (uint32_t r = 0; r < 4; ++r)
      if (n + r < p.N) p.C[(size_t)(n + r) * p.M + band * kTileM + row] = (_Float16)sum[r];
  } else {
    const uint32_t n = n0 + (sub / kRowBlocks) * 16u + (lane & 15u);
    const uint32_t row = (sub % kRowBlocks) * 16u + (lane >> 4) * 4u;
    if (n < p.N) {
      half4 h;
#pragma unroll
      for (int r = 0; r < 4; ++r) h[r] = (_Float16)sum[r];
      *(half4*)(p.C + (size_t)n * p.M + band * kTileM + row) = h;
    }
  }
}

template <int R, int NS, int FMT, int CB = 2>
static hipError_t launch_wide_variant(WideParams p, int cus, hipStream_t stream) {
  static std::atomic<bool> attr_done{false};  // per kernel variant; setting the attribute twice from two threads is harmless
  constexpr int kLds = wide_lds_bytes<NS>();
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)spmm_wide_kernel<R, NS, FMT, CB>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  const uint32_t quads = (p.bands + 3u) / 4u;
  p.S = wide_quad_slices(p.bands, p.G, p.KT, cus, NS);
  const uint32_t grid = (quads * p.S + 7u) / 8u * 8u * p.G;  // (group of bands, slice) pairs rounded up to eight, x column groups
  p.cb = CB;
  hipLaunchKernelGGL((spmm_wide_kernel<R, NS, FMT, CB>), dim3(grid), dim3(kWideWaves * 64), kLds, stream, p);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && p.S > 1) e = launch_wide_reduce(p, true, stream);
  return e;
}

// X (all N columns of the call) into fragment order, once per call of the dense 64-column pass.
hipError_t launch_xpack(const _Float16* X, _Float16* xpack, uint32_t K, uint32_t N, hipStream_t stream) {
  const uint32_t blocks = (N + 15u) / 16u, units = ((K / kTileK + 1u) / 2u) * blocks;
  hipLaunchKernelGGL(xpack_kernel, dim3((units + 3) / 4), dim3(256), 0, stream, X, xpack, K, N, units, blocks);
  return hipGetLastError();
}

hipError_t launch_wide_reduce(const WideParams& p, bool layout32, hipStream_t stream) {
  const uint32_t units = p.bands * p.G * (layout32 ? p.cb * 16u : (uint32_t)(kWideNB * kRowBlocks));
  if (layout32) hipLaunchKernelGGL(wide_reduce_kernel<true>, dim3((units + 3) / 4), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(wide_reduce_kernel<false>, dim3((units + 3) / 4), dim3(256), 0, stream, p);
  return hipGetLastError();
}

// `groups` groups of 64 columns starting at column n0, in one launch (the last group may reach past N).
hipError_t launch_spmm_wide(const SpmmLaunch& a, uint32_t n0, uint32_t groups, hipStream_t stream) {
  WideParams p;
  p.offs = a.offs;
  p.words = a.words;
  p.W = nullptr;
  p.X = a.X;
  p.Xp = nullptr;
  p.C = a.C;
  p.parts = a.parts;
  p.M = a.M;
  p.K = a.K;
  p.N = a.N;
  p.n0 = n0;
  p.G = groups;
  p.KT = a.K / kTileK;
  p.bands = a.M / kTileM;
  p.S = 1;
  // Variants by rounds staged per tile (256 words in version 1, 64 groups = 192 words in version 2); the ring is
  // 8 tiles deep while the registers allow.
  // At most 32 columns in all: only the first 32-column block is multiplied (the variants that wide32_pays can
  // ask for; anything else - a header that is out of date - falls through to the two-block variants, which are right
  // for any N).
  if (groups == 1 && a.N - n0 <= 32u) {
    const uint32_t round = a.version == 2 ? kRoundWords2 : 256u;
    if (a.version == 2) {
      if (a.max_tile_words <= 2 * round) return launch_wide_variant<2, 8, 2, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 3 * round) return launch_wide_variant<3, 8, 2, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 4 * round) return launch_wide_variant<4, 8, 2, 1>(p, a.num_cus, stream);
    } else {
      if (a.max_tile_words <= 2 * round) return launch_wide_variant<2, 8, 1, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 3 * round) return launch_wide_variant<3, 8, 1, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 4 * round) return launch_wide_variant<4, 8, 1, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 6 * round) return launch_wide_variant<6, 4, 1, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 8 * round) return launch_wide_variant<8, 4, 1, 1>(p, a.num_cus, stream);
      if (a.max_tile_words <= 10 * round) return launch_wide_variant<10, 4, 1, 1>(p, a.num_cus, stream);
    }
  }
  if (a.version == 2) {
    const uint32_t round = kRoundWords2;
    if (a.max_tile_words <= 2 * round) return launch_wide_variant<2, 8, 2>(p, a.num_cus, stream);
    if (a.max_tile_words <= 3 * round) return launch_wide_variant<3, 8, 2>(p, a.num_cus, stream);
    if (a.max_tile_words <= 4 * round) return launch_wide_variant<4, 8, 2>(p, a.num_cus, stream);
    if (a.max_tile_words <= 6 * round) return launch_wide_variant<6, 4, 2>(p, a.num_cus, stream);
    if (a.max_tile_words <= 8 * round) return launch_wide_variant<8, 4, 2>(p, a.num_cus, stream);
    return launch_wide_variant<10, 4, 2>(p, a.num_cus, stream);
  }
  if (a.max_tile_words <= 2 * 256) return launch_wide_variant<2, 8, 1>(p, a.num_cus, stream);
  if (a.max_tile_words <= 3 * 256) return launch_wide_variant<3, 8, 1>(p, a.num_cus, stream);
  if (a.max_tile_words <= 4 * 256) return launch_wide_variant<4, 8, 1>(p, a.num_cus, stream);
  if (a.max_tile_words <= 6 * 256) return launch_wide_variant<6, 4, 1>(p, a.num_cus, stream);
  if (a.max_tile_words <= 8 * 256) return launch_wide_variant<8, 4, 1>(p, a.num_cus, stream);
  return launch_wide_variant<10, 4, 1>(p, a.num_cus, stream);
}

}  // namespace fls
