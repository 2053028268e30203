// fls_spmm for more than 32 columns: 64 columns per pass (Flash-LLM's kernel for its widest batch
// sizes, re-cut for gfx950).
//
// A workgroup has four waves, one per SIMD with the whole register file (128 accumulator
// registers, a deep ring of tiles in flight), each with a tile run of its own; in the tile loop
// the waves share nothing but the CU: no barrier, no waiting.  With 64 columns a tile needs 4 KB of X against some
// 1.6 - 5 KB of compressed W, so how X reaches the MFMAs matters as much as W: a first kernel
// repacks X once per call into MFMA fragment order, after which a wave's four B fragments of a K
// tile are four fully coalesced 1 KB loads from L2, kept a few tiles ahead in a register ring of
// their own.  (Fragments loaded from X as the caller lays it out touch sixteen cache lines per
// load and bound the kernel; X shared between the four waves through LDS - double-buffered
// chunks, one barrier per four tiles - costs LDS bandwidth and lockstep, and measured 6 - 10 %
// slower for sparse tiles.)
//
// Work is cut as (pair of bands) x (K slice), S slices per pair so that the grid fills the CUs;
// inside a workgroup each band has two waves, one per half of the slice, whose accumulators meet
// in LDS when both are done (the one barrier of the kernel).  The sum is the band's partial
// result for the slice: with S = 1 it is stored to C directly, otherwise to a partial-sum area
// [band][slice] that a second, small kernel adds up in slice order and converts (no flags, no
// waiting between workgroups).  Two waves per band halve the partial sums that go through memory
// against one wave per band and slice.
//
// Inside a wave the stages are those of the narrow kernel - register ring of tiles, extraction by
// 2 B LDS stores, 16 B fragment reads, v_mfma_f32_16x16x32_f16 - software-pipelined, since no
// second wave shares the SIMD: a step reads the fragments of its tile, extracts the next tile
// behind those reads, and runs its MFMAs spread between the extraction's instructions.
#include "fls_device.h"
#include "fls_launch.h"

// Latency-breakdown builds (see fls_spmm.hip): 2 no MFMA, 4 no extract, 8 no re-zeroing, 16 no LDS
// fragment reads, 32 no global loads of the words, 256 no loads of X.  0 in the library.
#ifndef FLS_ABLATE
#define FLS_ABLATE 0
#endif

namespace fls {

constexpr int kWideWaves = 4;                   // two bands x two halves of the K slice
constexpr int kWideNB = 4;                      // column blocks per pass
constexpr int kWideTileLds = kTileBytes + 16;   // a wave's tile + the slot padding words land in
constexpr int kWideLdsBytes = kWideWaves * kWideTileLds + 2 * kWideNB * kRowBlocks * 64 * 16;  // tiles + two bands' accumulators

// X in MFMA fragment order: block (K tile kt, column block nb) holds, for lane l = 16 g + c, the 8
// halves X[32 kt + 8 g .. +7][16 nb + c] (zeros for columns past N).  One wave per pair of K tiles
// and column block, so that it uses the whole 128 B line of each of its 16 columns; loads are
// quad-contiguous (lane j reads column j >> 2, chunk j & 3), stores go to the fragment position.
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

template <int R, int NS, int XS>
__global__ __launch_bounds__(kWideWaves * 64) void spmm_wide_kernel(WideParams p) {
  constexpr int NB = kWideNB;
  static_assert(NS % XS == 0, "the unrolled ring must hold whole turns of the X ring");
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // the workgroup: two row bands x the two halves of its K slice
  const uint32_t pair = blockIdx.x / p.S, slice = blockIdx.x - pair * p.S;
  const uint32_t band = pair * 2 + (wave & 1u), half = wave >> 1;
  const bool active = band < p.bands;  // a wave past the last band walks an empty run and meets the barrier
  const uint32_t KT = p.KT, T = p.bands * KT;
  const uint32_t ka = (uint32_t)((uint64_t)slice * KT / p.S), kb = (uint32_t)((uint64_t)(slice + 1) * KT / p.S);
  const uint32_t km = ka + (kb - ka + 1) / 2;
  const uint32_t k0 = half ? km : ka, k1 = active ? (half ? kb : km) : k0;
  const uint32_t t0 = active ? band * KT + k0 : T, t1 = active ? band * KT + k1 : T;
  const uint32_t bodies = (k1 - k0 + NS - 1) / NS;  // of NS steps each

  unsigned char* tile = lds + wave * kWideTileLds;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;

  float4v acc[kRowBlocks][NB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

  // X: tile kt holds blocks of all columns of the call; this pass takes four from block n0 / 16 on.
  const uint32_t xblocks = (p.N + 15u) / 16u;
  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.Xp, 0, (int)(KT * xblocks * 1024u), kBufferFlags);
  const uint32_t xlane = (p.n0 / 16u) * 1024u + (uint32_t)lane * 16u;
  // the last pass of a call may have fewer than four column blocks left: the others read as zero
  const uint32_t xvalid = xblocks - p.n0 / 16u;
  // One tile's four blocks into a stage of the X ring.  Tiles past the slice (the padding of the
  // last body) must contribute nothing even if X holds Inf or NaN further along K: their X reads
  // as zero.  (Everything that may leave the buffer is in the per-lane offset: that is the part
  // the bounds check of a raw buffer looks at.)
  uint32_t xti = k0;
  auto xissue = [&](u32x4(&xq)[NB]) {
    const uint32_t base = xti * xblocks * 1024u + xlane;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const bool wanted = xti < k1 && (uint32_t)nb < xvalid;
      if (FLS_ABLATE & 256) xq[nb] = u32x4{base, 1u, 2u, 3u};
      else xq[nb] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, wanted ? base + nb * 1024u : 0xffffff00u, 0, 0);  // else: 0
    }
    ++xti;
  };

  // TileOffsets: a window of 64 entries in a VGPR (lane i = entry base + i), replaced once per
  // body by the window that was requested a body earlier - an unconditional load per NS tiles, so
  // stepping from tile to tile costs v_readlane and no wait.
  const uint32_t* offs = p.offs;
  auto window_at = [&](uint32_t first) {
    const uint32_t idx = first + (uint32_t)lane;
    return offs[idx < T ? idx : T];
  };
  uint32_t wbase = t0, window = window_at(t0);
  uint32_t ti = t0;  // next tile to request
  auto issue = [&](u32x4(&s)[R], uint32_t& begin, uint32_t& end) {
    begin = (uint32_t)__builtin_amdgcn_readlane((int)window, (int)(ti - wbase));
    end = (uint32_t)__builtin_amdgcn_readlane((int)window, (int)(ti + 1 - wbase));
    uint32_t n = end - begin;
    if (n > R * 256u) n = R * 256u;
    if (ti >= t1) {  // past the run: nothing to load, nothing to extract
      n = 0;
      end = begin;
    }
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(p.words + begin), 0, (int)(n * 4u), kBufferFlags);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (FLS_ABLATE & 32) s[r] = u32x4{(uint32_t)lane, 1u, 2u, 3u};
      else s[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (r * 64 + lane) * 16, 0, kAuxNonTemporal);
    }
    ++ti;
  };

  // extract (Alg. 2), branch-free so that a step is one basic block: lanes past the end of the
  // run (their loads returned 0: location 0, value 0) get the slot that padding words go to as
  // their base.  The words are then replaced by the LDS addresses they went to, which is all the
  // later re-zeroing needs.  (No tile has more than R * 256 words here: see `densest` below.)
  typedef __attribute__((address_space(3))) uint16_t* lds_u16_ptr;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)tile;  // LDS addresses are the low 32 bits
  auto extract = [&](u32x4(&s)[R], uint32_t begin, uint32_t end) {
    const uint32_t n = end - begin;
#pragma unroll
    for (int r = 0; r < R; ++r) {
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
  };

  const unsigned char* frag = tile + ((lane >> 4) * kTileM + (lane & 15)) * 16;

  // rst_smem.  Sparse tiles (R <= 4: at most 1024 words) are re-zeroed by storing zeros where
  // their words went - as many 2 B stores as the extraction - instead of clearing all 8 KB.
  constexpr bool kUnscatter = R <= 4;
  auto unscatter = [&](const u32x4(&s)[R]) {
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) *(lds_u16_ptr)(uintptr_t)s[r][j] = (uint16_t)0;
  };

  // One tile, whose words stage `cur` still holds (as LDS addresses by now) and which the step
  // before extracted into LDS: the X stage that step used is refilled, the tile's A fragments are
  // read, the tile is re-zeroed behind the reads, stage `cur` is refilled, the next tile (stage
  // `nxt`) is extracted, and the MFMAs run spread between those instructions.
  auto step = [&](u32x4(&cur)[R], uint32_t& cb, uint32_t& ce, u32x4(&nxt)[R], uint32_t nb_, uint32_t ne_,
                  u32x4(&xfill)[NB], const u32x4(&xuse)[NB]) {
    half8 fa[kRowBlocks], fb[NB];
    xissue(xfill);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) fb[nb] = __builtin_bit_cast(half8, xuse[nb]);
#pragma unroll
    for (int j = 0; j < kRowBlocks; ++j) {
      if (FLS_ABLATE & 16) fa[j] = fb[j % NB];
      else fa[j] = *(const half8*)(frag + j * 256);
    }
    if (FLS_ABLATE & 8) {
    } else if constexpr (kUnscatter) {
      unscatter(cur);
    } else {
#pragma unroll
      for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
    }
    issue(cur, cb, ce);
    extract(nxt, nb_, ne_);
#pragma unroll
    for (int j = 0; j < kRowBlocks; ++j)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        if (FLS_ABLATE & 2) acc[j][nb][0] += (float)fa[j][0] * (float)fb[nb][0];
        else acc[j][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[j], fb[nb], acc[j][nb], 0, 0, 0);
      }
    // asks the scheduler for: one MFMA, then up to three instructions of the other kinds
#pragma unroll
    for (int i = 0; i < kRowBlocks * NB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002 | 0x004 | 0x010 | 0x080, 3, 0);
    }
  };

  // The launcher picks R from the header the host remembers for this blob address.  If the memory
  // holds a denser blob by now (one written there without the library's knowing), the ring cannot
  // stage its tiles: the whole grid then takes a plain path - tile by tile, words straight from
  // memory into LDS, X fragments from the packed copy - which is slow and right.
  const uint32_t densest = offs[kHeaderMaxTileWords - kHeaderWords];
  if (densest > R * 256u) {
    for (uint32_t t = t0; t < t1; ++t) {
      const uint32_t begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)offs[t]);
      const uint32_t end = (uint32_t)__builtin_amdgcn_readfirstlane((int)offs[t + 1]);
      for (uint32_t i = begin + (uint32_t)lane * 4u; i < end; i += 256u) {
        const u32x4 w = *(const u32x4*)(p.words + i);
#pragma unroll
        for (int j = 0; j < 4; ++j) *(uint16_t*)(tile + ((w[j] & 0xffffu) << 1)) = (uint16_t)(w[j] >> 16);
      }
      const uint32_t kt = k0 + (t - t0);
      half8 fa[kRowBlocks], fb[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(
            xrsrc, (uint32_t)nb < xvalid ? kt * xblocks * 1024u + xlane + nb * 1024u : 0xffffff00u, 0, 0);
        fb[nb] = __builtin_bit_cast(half8, v);
      }
#pragma unroll
      for (int j = 0; j < kRowBlocks; ++j) fa[j] = *(const half8*)(frag + j * 256);
#pragma unroll
      for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
#pragma unroll
      for (int j = 0; j < kRowBlocks; ++j)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[j][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[j], fb[nb], acc[j][nb], 0, 0, 0);
    }
  } else {
    // Rings: NS tiles of W words in flight; X fragments XS - 1 tiles ahead (they come from L2 and
    // ride behind the words in the same in-order load queue).  Prologue: both rings filled, first
    // tile in LDS.
    u32x4 s[NS][R];
    uint32_t sb[NS], se[NS];
    u32x4 xq[XS][NB];
#pragma unroll
    for (int i = 0; i < XS - 1; ++i) xissue(xq[i]);
#pragma unroll
    for (int i = 0; i < NS; ++i) issue(s[i], sb[i], se[i]);
    uint32_t next_window = window_at(t0 + NS);
    extract(s[0], sb[0], se[0]);
    for (uint32_t body = 0; body < bodies; ++body) {
      // refills of this body ask for tiles t0 + NS * body + NS ... + 2 NS - 1: inside the window
      // that starts at t0 + NS * (body + 1)
      window = next_window;
      wbase = t0 + NS * (body + 1);
      next_window = window_at(t0 + NS * (body + 2));
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int i1 = (i + 1) % NS;  // stage of the next tile
        step(s[i], sb[i], se[i], s[i1], sb[i1], se[i1], xq[(i + XS - 1) % XS], xq[i % XS]);
      }
    }
  }

  // The two halves of the K slice meet in LDS: the waves of the second half leave their
  // accumulators there, the waves of the first half add them to their own and write the band's
  // result for the slice - half as many partial sums in memory as waves.
  float4v* meet = (float4v*)(lds + kWideWaves * kWideTileLds) + (wave & 1u) * (NB * kRowBlocks * 64) + lane;
  if (half == 1) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb) meet[(nb * kRowBlocks + rb) * 64] = acc[rb][nb];
  }
  __syncthreads();
  if (half == 1 || !active) return;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb) acc[rb][nb] += meet[(nb * kRowBlocks + rb) * 64];
  if (p.S == 1) {
    OutParams o;
    o.C = p.C;
    o.M = p.M;
    o.N = p.N;
    o.n0 = p.n0;
    store_band<NB>(o, acc, band, lane);
  } else {
    float4v* dst = (float4v*)p.parts + ((size_t)(band * p.S + slice) * (NB * kRowBlocks)) * 64 + lane;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb) dst[(nb * kRowBlocks + rb) * 64] = acc[rb][nb];
  }
}

// Adds the S partial results of every band in slice order, converts, writes C.  One wave per
// (band, column block, row block): S loads of 16 B per lane, all issued before the first is used.
__global__ __launch_bounds__(256) void wide_reduce_kernel(WideParams p) {
  const uint32_t unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= p.bands * (kWideNB * kRowBlocks)) return;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t band = unit / (kWideNB * kRowBlocks), sub = unit - band * (kWideNB * kRowBlocks);
  const uint32_t nb = sub / kRowBlocks, rb = sub - nb * kRowBlocks;
  const float4v* src = (const float4v*)p.parts + ((size_t)band * p.S * (kWideNB * kRowBlocks) + sub) * 64 + lane;
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
  const uint32_t n = p.n0 + nb * 16 + (lane & 15u);
  if (n < p.N) {
    half4 h;
#pragma unroll
    for (int r = 0; r < 4; ++r) h[r] = (_Float16)sum[r];
    *(half4*)(p.C + (size_t)n * p.M + band * kTileM + rb * 16 + (lane >> 4) * 4) = h;
  }
}

template <int R, int NS, int XS>
static hipError_t launch_wide_variant(const WideParams& p, int grid, hipStream_t stream) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)spmm_wide_kernel<R, NS, XS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kWideLdsBytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL((spmm_wide_kernel<R, NS, XS>), dim3(grid), dim3(kWideWaves * 64), kWideLdsBytes, stream, p);
  return hipGetLastError();
}

// X (all N columns of the call) into fragment order, once per call.
hipError_t launch_xpack(const _Float16* X, _Float16* xpack, uint32_t K, uint32_t N, hipStream_t stream) {
  const uint32_t blocks = (N + 15u) / 16u, units = ((K / kTileK + 1u) / 2u) * blocks;
  hipLaunchKernelGGL(xpack_kernel, dim3((units + 3) / 4), dim3(256), 0, stream, X, xpack, K, N, units, blocks);
  return hipGetLastError();
}

hipError_t launch_wide_reduce(const WideParams& p, hipStream_t stream) {
  const uint32_t units = p.bands * (kWideNB * kRowBlocks);
  hipLaunchKernelGGL(wide_reduce_kernel, dim3((units + 3) / 4), dim3(256), 0, stream, p);
  return hipGetLastError();
}

// One 64-column pass starting at column n0; `xpack` holds all N columns in fragment order.
hipError_t launch_spmm_wide(const SpmmLaunch& a, uint32_t n0, hipStream_t stream) {
  WideParams p;
  p.offs = a.offs;
  p.words = a.words;
  p.W = nullptr;
  p.Xp = a.xpack;
  p.C = a.C;
  p.parts = a.parts;
  p.M = a.M;
  p.K = a.K;
  p.N = a.N;
  p.n0 = n0;
  p.KT = a.K / kTileK;
  p.bands = a.M / kTileM;
  const uint32_t pairs = (p.bands + 1u) / 2u;
  p.S = wide_pair_slices(p.bands, p.KT, a.num_cus);
  const int grid = (int)(pairs * p.S);
  hipError_t e;
  // rounds of 256 words staged per tile; the ring is 8 tiles deep while the registers allow; X fragments 3 tiles ahead
  if (a.max_tile_words <= 2 * 256) e = launch_wide_variant<2, 8, 4>(p, grid, stream);
  else if (a.max_tile_words <= 3 * 256) e = launch_wide_variant<3, 8, 4>(p, grid, stream);
  else if (a.max_tile_words <= 4 * 256) e = launch_wide_variant<4, 8, 4>(p, grid, stream);
  else if (a.max_tile_words <= 6 * 256) e = launch_wide_variant<6, 4, 4>(p, grid, stream);
  else if (a.max_tile_words <= 8 * 256) e = launch_wide_variant<8, 4, 4>(p, grid, stream);
  else e = launch_wide_variant<10, 4, 4>(p, grid, stream);
  if (e != hipSuccess) return e;
  if (p.S > 1) e = launch_wide_reduce(p, stream);
  return e;
}

}  // namespace fls
