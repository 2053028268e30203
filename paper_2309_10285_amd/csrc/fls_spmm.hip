// fls_spmm, passes of up to 32 columns: Load-as-Sparse / Compute-as-Dense SpMM for gfx950
// (Flash-LLM, Alg. 1 re-designed for wave64 / MFMA / 160 KB LDS).
//
// One persistent workgroup per CU; every wave owns a contiguous run of Tiled-CSL tiles, which it
// walks piece by piece (a piece = its tiles of one row band), and a private 8 KB LDS tile, so the
// stages of Alg. 1 run per wave with no workgroup barrier:
//   gmem2reg : the tile's words stream from HBM into VGPRs with 16 B non-temporal loads,
//              a few tiles ahead of their use (register ring)
//   extract  : each word's fp16 value is stored at its location in the zero-filled LDS tile
//              (Alg. 2); the location field already is the position in the MFMA operand layout
//   smem2tc  : A fragments are 16 B LDS reads; B fragments (X) come from L2 as 16 B loads in the
//              ring and pass through a 1 KB LDS stage that puts them into MFMA order;
//              v_mfma_f32_16x16x32_f16 accumulates in fp32
//   rst_smem : right behind the fragment reads (LDS operations of a wave execute in order, so no
//              wait separates the stages) the tile is made zero again: sparse tiles by storing
//              zeros where their words went, dense ones by clearing all 8 KB
// Split-K: the tile sequence (band-major) is cut evenly over all waves of the grid; partial
// bands are summed in LDS inside a workgroup and through fp32 slots in HBM between workgroups.
// More than 32 columns: fls_spmm_wide.hip.
#include <atomic>
#include <type_traits>

#include "fls_device.h"
#include "fls_launch.h"
#include "fls_tile.h"

// Latency-breakdown builds (the paper's Fig. 11 method: erase the other operations and time what is
// left).  FLS_ABLATE is a bit mask, 0 in the library: 1 no split-K hand-over, 2 no MFMA, 4 no extract,
// 8 no re-zeroing, 16 no LDS fragment reads, 32 no global loads of the words, 64 no hand-over
// between workgroups, 128 no reduction inside the workgroup.  Results are wrong by design.
#ifndef FLS_ABLATE
#define FLS_ABLATE 0
#endif

namespace fls {

// LDS of one wave: its tile, the 16 B slot that padding words land in, the X stage (1 KB per column block)
constexpr int wave_lds(int NB) { return kTileBytes + 16 + NB * 1024; }

struct SpmmParams {
  const uint32_t* offs;   // TileOffsets
  const uint32_t* words;  // NonZeros
  const _Float16* X;
  uint32_t K;
  OutParams out;
};

// FMT = format version of the blob: 1 = 32-bit words (value, location), R rounds of 256 words staged
// per tile; 2 = groups of four entries in three words (the first location in full, three 6-bit
// distances), R rounds of 64 groups (256 entries, 192 words) staged per tile.  A stage register holds
// four words either way: what a lane loads per round (three of them in version 2), then the four LDS
// addresses its entries went to.
template <int NB, int WAVES, int R, int NS, int FMT>
__global__ __launch_bounds__(WAVES * 64) void spmm_kernel(SpmmParams p) {
  typedef u32x4 stage_t;
  constexpr uint32_t kRoundWords = FMT == 2 ? kRoundWords2 : 256u;
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t g = blockIdx.x * WAVES + wave, G = gridDim.x * WAVES;
  const uint32_t T = p.out.T, KT = p.out.KT;
  const uint32_t t0 = (uint32_t)((uint64_t)g * T / G), t1 = (uint32_t)((uint64_t)(g + 1) * T / G);
  const uint32_t share0 = share_begin(blockIdx.x, T, gridDim.x), share1 = share_begin(blockIdx.x + 1, T, gridDim.x);
  constexpr int kWaveLds = wave_lds(NB);
  // the first offsets are on their way while LDS is set up
  OffsetWindow win;
  win.offs = p.offs;
  win.T = T;
  win.total = p.offs[kHeaderTotalWords - kHeaderWords];  // from the blob's own header, like every length
  win.lane = lane;
  win.request(t0 < T ? t0 : T);
  WgReduceLds<NB>* red = (WgReduceLds<NB>*)(lds + WAVES * kWaveLds);
  wg_reduce_init<NB>(red, threadIdx.x, WAVES * 64);
  __syncthreads();  // the only barrier: from here on the waves run independently
  if (t0 >= t1) return;

  unsigned char* tile = lds + wave * kWaveLds;
  unsigned char* xs = tile + kTileBytes + 16;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;

  float4v acc[kRowBlocks][NB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

  XFrags xf;
  xf.init(p.X, p.K, p.out.N, p.out.n0, lane);
  win.arrive();
  const unsigned char* frag = tile + ((lane >> 4) * kTileM + (lane & 15)) * 16;

  // A wave's run [t0, t1) is walked piece by piece, a piece being its tiles of one row band
  // [tc, pend).  Load side: tile ti is the next to be requested; consume side: tile tc is the
  // next to be used.
  uint32_t tc = t0, ktc = t0 % KT, bandc = t0 / KT;
  uint32_t ti = tc, kti = ktc, pend = tc;

  // gmem2reg.  No branch may enclose the ring's loads (the compiler's vmcnt bookkeeping would fall
  // back to "wait for everything" and the ring would be lost), so a lane past the end of the
  // run, or a tile past the end of the wave's tiles, is turned away by the bounds check of the
  // buffer descriptor instead: it returns 0 and moves no data.  Nothing is requested past the
  // end of the piece either: the ring runs empty there, so that the hand-over that follows has
  // the registers to itself (no value of the ring is live across it).
  auto issue = [&](stage_t(&s)[R], u32x4(&x)[NB], uint32_t& begin, uint32_t& end) {
    win.get(ti, begin, end);
    uint32_t n = end - begin;
    if (n > R * kRoundWords) n = R * kRoundWords;
    if (ti >= pend) {
      n = 0;
      end = begin;  // nothing to extract either
    }
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
    xf.template load<NB>(x, kti);
    ++ti;
    if (++kti == KT) kti = 0;
  };

  // extract (Alg. 2): value = high half of the word, byte address = 2 * location.  Where the tile
  // is re-zeroed by un-scatter, a word is replaced by the LDS address it went to, which is all
  // that step needs.
  typedef __attribute__((address_space(3))) uint16_t* lds_u16_ptr;
  const uint32_t tile_addr = (uint32_t)(uintptr_t)tile;  // LDS addresses are the low 32 bits
  auto extract = [&](stage_t(&s)[R], uint32_t begin, uint32_t end) {
    const uint32_t n = end - begin;
    if constexpr (FMT == 2) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        // no branch: a lane past the end of the run (its loads returned 0) writes zeros to the padding slot
        const uint32_t base = (r * 64 + lane) * kGroupWords < n ? tile_addr : tile_addr + (uint32_t)kTileBytes;
        s[r] = extract_group(s[r][0], s[r][1], s[r][2], base, !(FLS_ABLATE & 4));
      }
      if (n > R * kRoundWords) extract_overflow_v2(p.words, begin + R * kRoundWords, end, tile);
      return;
    } else {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      // no branch: a lane past the end of the run (its loads returned 0: location 0, value 0) gets
      // the slot that padding words go to as its base
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
    if (n > R * 256u) extract_overflow(p.words, begin + R * 256u, end, tile);
    }
  };

  // rst_smem for sparse tiles: instead of zeroing all 8 KB (eight 16 B stores per lane, 64 LDS
  // clocks), store a zero at the places the tile's words went to - the same count of 2 B stores
  // as the extraction, which is less LDS time as long as a tile has at most about 1000 words.
  constexpr bool kUnscatter = R <= 4;
  auto unscatter = [&](const stage_t(&s)[R], uint32_t begin, uint32_t end) {
    const uint32_t n = end - begin;
    if (n > R * kRoundWords) {  // the overflow path wrote words this wave no longer holds
#pragma unroll
      for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) *(lds_u16_ptr)(uintptr_t)s[r][j] = (uint16_t)0;
    }
  };
  auto read_frags = [&](half8(&a)[kRowBlocks]) {
#pragma unroll
    for (int j = 0; j < kRowBlocks; ++j) {
      if (FLS_ABLATE & 16) a[j] = half8{1, 1, 1, 1, 1, 1, 1, 1};
      else a[j] = *(const half8*)(frag + j * 256);
    }
  };
  auto mfma = [&](const half8(&a)[kRowBlocks], const half8(&b)[NB]) {
#pragma unroll
    for (int j = 0; j < kRowBlocks; ++j) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        if (FLS_ABLATE & 2) acc[j][nb][0] += (float)a[j][0] * (float)b[nb][0];
        else acc[j][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[j], b[nb], acc[j][nb], 0, 0, 0);
      }
    }
  };
  auto compute = [&]() {
    half8 x[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) x[nb] = xf.frag(xs, nb);
    // fragments of H row blocks at a time (all eight when the accumulators leave the registers for it)
    constexpr int H = NB == 1 ? 8 : 4;
#pragma unroll
    for (int h = 0; h < kRowBlocks; h += H) {
      half8 a[H];
#pragma unroll
      for (int j = 0; j < H; ++j) {
        if (FLS_ABLATE & 16) a[j] = x[0];
        else a[j] = *(const half8*)(frag + (h + j) * 256);
      }
      if (h + H == kRowBlocks && !(FLS_ABLATE & 8)) {
#pragma unroll
        for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
      }
#pragma unroll
      for (int j = 0; j < H; ++j) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          if (FLS_ABLATE & 2) acc[h + j][nb][0] += (float)a[j][0] * (float)x[nb][0];
          else acc[h + j][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[j], x[nb], acc[h + j][nb], 0, 0, 0);
        }
      }
    }
  };

  // Hand-over of the piece of `tiles` tiles that just ended in `band`.
  HandoverState hs;
  auto hand_over = [&](uint32_t band, uint32_t tiles) {
    if (FLS_ABLATE & 1) {
      float sum = 0.f;  // keeps every accumulator alive
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sum += acc[rb][nb][0] + acc[rb][nb][1] + acc[rb][nb][2] + acc[rb][nb][3];
      if (sum == 1234.5f) p.out.C[lane] = (_Float16)1;
    } else if (FLS_ABLATE & 128) {
      store_band<NB>(p.out, acc, band, lane);
    } else {
      hand_over_piece<NB>(p.out, red, acc, hs, band, tiles, share0, share1, blockIdx.x, lane, (FLS_ABLATE & 64) != 0, true);
    }
    if (FLS_ABLATE & (1 | 128)) {
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
    }
  };

  // Register ring of NS tiles in flight.  A stage is refilled as soon as its words are in LDS,
  // before the MFMA work of its tile, so loads lead their use by NS - 1 tiles of work.  The loop
  // is straight-line in the ring's loads - every step issues the same number, none under a
  // condition - which lets the compiler wait for exactly the stage it needs
  // (s_waitcnt vmcnt(n), n = loads issued since).
  stage_t s[NS][R];
  u32x4 x[NS][NB];
  uint32_t sb[NS], se[NS];  // word range of the tile each stage holds

  auto step = [&](stage_t(&ss)[R], u32x4(&sx)[NB], uint32_t& b, uint32_t& e) {
    // Two waves share a SIMD and, at equal priority, the older one wins every issue slot both
    // want (LDS and memory instructions compete CU-wide), so it would finish its run microseconds
    // ahead of the younger, which then runs the tail alone.  The younger waves sit at priority 1;
    // the older ones alternate between 0 and 2 from tile to tile, so each side wins half the time.
    if (WAVES > 4 && wave < WAVES / 2) {
      if (tc & 1u) __builtin_amdgcn_s_setprio(2);
      else __builtin_amdgcn_s_setprio(0);
    }
    extract(ss, b, e);
    xf.template stage<NB>(xs, sx);
    if constexpr (kUnscatter) {
      half8 fa[kRowBlocks], fb[NB];
      read_frags(fa);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) fb[nb] = xf.frag(xs, nb);
      if (!(FLS_ABLATE & 8)) unscatter(ss, b, e);  // behind the reads: LDS keeps a wave's operations in order
      issue(ss, sx, b, e);
      mfma(fa, fb);
    } else {
      issue(ss, sx, b, e);
      compute();
    }
    ++tc;
  };

  // When the workgroup's share lies inside one band (with a tile for every wave), every wave has one
  // piece, all of the same band, and when its run is over none has anything else left to do: they
  // meet at a barrier and share the sum.  Every wave leaves its accumulators of one column block in
  // its tile buffer (8 KB, free by then), and wave w adds the eight buffers' row block w in wave
  // order - a fixed order.  What happens to those 16 rows depends on the share's place in the band:
  //  - the whole band (the band-aligned grid; the last thing the whole chip waits for): converted and
  //    stored to C by the wave that summed them;
  //  - the band's beginning: this workgroup is the band's owner; the row blocks go through an LDS slot
  //    into wave 0's registers, which finishes the band after the loop, once the other workgroups'
  //    sums are there;
  //  - else: stored to the workgroup's partial-sum slot by the wave that summed them; wave 0 starts
  //    the release once all eight parts have reached the L2, and publishes the slot after the loop.
  // (A build that erases the hand-over erases it in every workgroup: were this path left in, its owners would wait
  // out their bounded spin for partial sums that the erased path never publishes.)
  const bool one_band = !(FLS_ABLATE & (1 | 128)) && share0 / KT == (share1 - 1) / KT && share1 - share0 >= (uint32_t)WAVES;
  auto one_band_sum = [&](uint32_t band) {
    static_assert(WAVES == kRowBlocks, "one row block per wave");
    const bool from_start = share0 % KT == 0, to_end = share1 % KT == 0;
    const bool whole = (from_start && to_end) || (FLS_ABLATE & 64);
    const uint32_t col = lane & 15, rsub = (lane >> 4) * 4;
    const __amdgpu_buffer_rsrc_t mine = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.out.parts + (size_t)blockIdx.x * (NB * kAccPerBlock)), 0, NB * kAccPerBlock * 4, kBufferFlags);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      if (nb > 0) __syncthreads();  // every wave is done reading the buffers of the column block before
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb) *(float4v*)(tile + rb * 1024 + lane * 16) = acc[rb][nb];
      __syncthreads();
      float4v sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < WAVES; ++w) sum += *(const float4v*)(lds + w * kWaveLds + wave * 1024 + lane * 16);
      if (whole) {
        const uint32_t n = p.out.n0 + nb * 16 + col;
        if (n < p.out.N) {
          half4 h;
#pragma unroll
          for (int r = 0; r < 4; ++r) h[r] = (_Float16)sum[r];
          *(half4*)(p.out.C + (size_t)n * p.out.M + band * kTileM + wave * 16 + rsub) = h;
        }
      } else if (from_start) {
        red->slot[0][(nb * kRowBlocks + wave) * 64 + lane] = sum;
      } else {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, sum), mine, ((nb * kRowBlocks + wave) * 64 + lane) * 16,
                                               0, kAuxCoherent);
      }
    }
    if (whole) return;
    if (from_start) {
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int rb = 0; rb < kRowBlocks; ++rb) acc[rb][nb] = red->slot[0][(nb * kRowBlocks + rb) * 64 + lane];
        hs.own = true;
        hs.own_band = band;
      }
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's part of the partial sum has reached the L2
      __syncthreads();
      if (wave == 0) {
        release_begin();
        hs.released = true;
        hs.publish = true;
      }
    }
  };

  if (WAVES > 4 && wave >= WAVES / 2) __builtin_amdgcn_s_setprio(1);
  while (tc < t1) {
    const uint32_t piece0 = tc;
    pend = tc + (KT - ktc) < t1 ? tc + (KT - ktc) : t1;
    ti = tc;
    kti = ktc;
#pragma unroll
    for (int i = 0; i < NS; ++i) issue(s[i], x[i], sb[i], se[i]);
    while (tc + NS <= pend) {
#pragma unroll
      for (int i = 0; i < NS; ++i) step(s[i], x[i], sb[i], se[i]);
    }
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
      if (tc < pend) step(s[i], x[i], sb[i], se[i]);
    if (one_band) one_band_sum(bandc);
    else hand_over(bandc, pend - piece0);
    ktc += pend - piece0;
    if (ktc == KT) {
      ktc = 0;
      ++bandc;
    }
  }
  hand_over_finish<NB>(p.out, acc, hs, blockIdx.x, gridDim.x, lane);
}

// ---------------------------------------------------------------- host launcher


// Tiles in flight per wave: set by measurement.  Two tiles ahead (about 8 KB per wave, 64 KB per CU
// in flight at 1024 words per tile) everywhere but one column block per wave with tiles of more
// than 1024 words, where three were 1 % faster; deeper rings measured slower (C2 with two / three /
// four tiles: 33.7 / 35.5 / 35.8 us; 28672 x 7168 at 90 %, 32 columns, two / four: 30.3 / 31.3 us).
// A stage costs 4 R + 4 NB registers, the accumulators 32 NB, and a wave has 256 registers.
constexpr int ring_depth(int NB, int WAVES, int R) {
  return NB == 1 && R > 4 ? 3 : 2;
}

template <int NB, int WAVES, int R, int FMT>
static hipError_t launch_variant(const SpmmParams& p, int grid, hipStream_t stream) {
  constexpr int NS = ring_depth(NB, WAVES, R);
  static std::atomic<bool> attr_done{false};  // per kernel variant; setting the attribute twice from two threads is harmless
  const int lds_bytes = WAVES * wave_lds(NB) + (int)sizeof(WgReduceLds<NB>);
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)spmm_kernel<NB, WAVES, R, NS, FMT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       lds_bytes);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((spmm_kernel<NB, WAVES, R, NS, FMT>), dim3(grid), dim3(WAVES * 64), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int NB, int WAVES, int FMT>
static hipError_t launch_r(int R, const SpmmParams& p, int grid, hipStream_t stream) {
  switch (R) {
    case 2: return launch_variant<NB, WAVES, 2, FMT>(p, grid, stream);
    case 3: return launch_variant<NB, WAVES, 3, FMT>(p, grid, stream);
    case 4: return launch_variant<NB, WAVES, 4, FMT>(p, grid, stream);
    case 6: return launch_variant<NB, WAVES, 6, FMT>(p, grid, stream);
    default: return launch_variant<NB, WAVES, 8, FMT>(p, grid, stream);
  }
}

hipError_t launch_spmm(const SpmmLaunch& a, hipStream_t stream) {
  SpmmParams p;
  p.offs = a.offs;
  p.words = a.words;
  p.X = a.X;
  p.K = a.K;
  p.out.T = (a.M / kTileM) * (a.K / kTileK);
  p.out.C = a.C;
  p.out.parts = a.parts;
  p.out.flags = a.flags;
  p.out.M = a.M;
  p.out.N = a.N;
  p.out.KT = a.K / kTileK;
  const int grid = pick_grid(a.M / kTileM, a.K / kTileK, a.num_cus);
  // rounds of 256 words staged per tile: the smallest variant that holds the densest tile
  // (a denser tile is still handled, through a slow path)
  const bool v2 = a.version == 2;
  const uint32_t round_words = v2 ? kRoundWords2 : 256u;
  int R = 8;
  if (a.max_tile_words <= 2 * round_words) R = 2;
  else if (a.max_tile_words <= 3 * round_words) R = 3;
  else if (a.max_tile_words <= 4 * round_words) R = 4;
  else if (a.max_tile_words <= 6 * round_words) R = 6;
  // The 64-column pass stages at most ten rounds of a tile (it has no slow path for more; twelve
  // rounds no longer fit its registers): a matrix with denser tiles - less than 40 % sparse
  // somewhere - takes 32-column passes throughout.
  const bool wide_ok = a.max_tile_words <= 10 * round_words;
  for (uint32_t n0 = 0; n0 < a.N;) {
    p.out.n0 = n0;
    const uint32_t left = a.N - n0;
    hipError_t e;
    if (left <= 16) {
      p.X = a.X;
      e = v2 ? launch_r<1, 8, 2>(R, p, grid, stream) : launch_r<1, 8, 1>(R, p, grid, stream);
      n0 += 16;
    } else if (left <= 32 && a.wide32 && wide32_pays(a.max_tile_words, round_words, a.K / kTileK, a.version, a.M / kTileM, a.num_cus)) {
      e = launch_spmm_wide(a, n0, 1, stream);  // multiplies its first 32-column block only
      n0 += 32;
    } else if (left <= 32 || !wide_ok) {
      p.X = a.X;
      e = v2 ? launch_r<2, 8, 2>(R, p, grid, stream) : launch_r<2, 8, 1>(R, p, grid, stream);
      n0 += 32;
    } else {
      // All the groups of 64 columns in one launch, a last one that is partly empty included: the workgroups of a
      // further group find the words in their XCD's L2, where a narrower pass of its own for the rest would stream
      // W from HBM once more (12288 x 12288 at 90 %: N = 80 in 42.5 us against 54.8, N = 96 in 42.2 against 59.7).
      const uint32_t groups = (left + kSpmmGroupCols - 1u) / kSpmmGroupCols;
      e = launch_spmm_wide(a, n0, groups, stream);
      n0 += groups * kSpmmGroupCols;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace fls
