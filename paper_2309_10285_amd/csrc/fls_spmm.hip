// fls_spmm: Load-as-Sparse / Compute-as-Dense SpMM for gfx950 (Flash-LLM, Alg. 1 re-designed
// for wave64 / MFMA / 160 KB LDS).
//
// One persistent workgroup per CU; every wave owns a contiguous run of Tiled-CSL tiles and a
// private 8 KB LDS tile, so the stages of Alg. 1 run per wave with no workgroup barrier:
//   gmem2reg : the tile's words stream from HBM into VGPRs with 16 B non-temporal loads,
//              two tiles ahead of their use (register double buffer)
//   extract  : each word's fp16 value is stored at its location in the zero-filled LDS tile
//              (Alg. 2); the location field already is the position in the MFMA operand layout
//   smem2tc  : A fragments are 16 B LDS reads, B fragments (X) come straight from L2 as 16 B
//              loads, v_mfma_f32_16x16x32_f16 accumulates in fp32
//   rst_smem : the tile is zeroed again right after its fragments were read (LDS operations of a
//              wave execute in order, so no wait separates the stages)
// Split-K: the tile sequence (band-major) is cut evenly over all waves of the grid; partial
// bands are summed in LDS inside a workgroup and through fp32 slots in HBM between workgroups.
#include "fls_device.h"
#include "fls_launch.h"

// Latency-breakdown builds (the paper's Fig. 11 method: erase the other operations and time what is
// left).  FLS_ABLATE is a bit mask, 0 in the library: 1 no split-K hand-over, 2 no MFMA, 4 no extract,
// 8 no re-zeroing, 16 no LDS fragment reads, 32 no global loads of the words, 64 no hand-over between workgroups, 128 no reduction inside the workgroup.  Results are wrong by design.
#ifndef FLS_ABLATE
#define FLS_ABLATE 0
#endif

namespace fls {

constexpr int kWaveLds = kTileBytes + 16;  // + the slot that padding words land in

struct SpmmParams {
  const uint32_t* offs;   // TileOffsets
  const uint32_t* words;  // NonZeros
  const _Float16* X;
  uint32_t K;
  OutParams out;
};

// A run of at most R*256 words of one tile.
struct Chunk {
  uint32_t begin, n;  // word range [begin, begin + n) in NonZeros
  uint32_t t, kt, band;  // tile id, its K tile and row band
  bool last;   // completes its tile
  bool valid;
};

// TileOffsets are read through the scalar unit: the index is wave-uniform and nothing in the kernel
// writes the blob, so the constant address space is safe and keeps these loads off the vector
// memory counter that paces the word stream.
typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;

template <int R>
struct ChunkWalk {
  const_u32_ptr offs;
  uint32_t t, t_end, KT;
  uint32_t pos, end, end_next;
  uint32_t kt, band;

  __device__ __forceinline__ void init(const uint32_t* offs_, uint32_t t0, uint32_t t1, uint32_t KT_) {
    offs = (const_u32_ptr)offs_;
    t = t0;
    t_end = t1;
    KT = KT_;
    pos = offs[t0];
    end = offs[t0 + 1];
    end_next = offs[t0 + 2];  // guard entries keep this in bounds
    band = t0 / KT;
    kt = t0 - band * KT;
  }
  __device__ __forceinline__ Chunk next() {
    Chunk c;
    c.valid = t < t_end;
    c.begin = pos;
    uint32_t n = end - pos;
    if (n > R * 256u) n = R * 256u;
    c.n = c.valid ? n : 0u;
    c.t = t;
    c.kt = kt;
    c.band = band;
    c.last = (pos + n == end);
    if (c.valid) {
      pos += n;
      if (c.last) {
        ++t;
        pos = end;
        end = end_next;
        end_next = offs[t + 2];
        if (++kt == KT) {
          kt = 0;
          ++band;
        }
      }
    }
    return c;
  }
};

template <int NB, int WAVES, int R, int NS>
__global__ __launch_bounds__(WAVES * 64) void spmm_kernel(SpmmParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t g = blockIdx.x * WAVES + wave, G = gridDim.x * WAVES;
  const uint32_t T = p.out.T;
  const uint32_t t0 = (uint32_t)((uint64_t)g * T / G), t1 = (uint32_t)((uint64_t)(g + 1) * T / G);
  const uint32_t share0 = share_begin(blockIdx.x, T, gridDim.x), share1 = share_begin(blockIdx.x + 1, T, gridDim.x);
  WgReduceLds<NB>* red = (WgReduceLds<NB>*)(lds + WAVES * kWaveLds);
  wg_reduce_init<NB>(red, threadIdx.x, WAVES * 64);
  __syncthreads();  // the only barrier: from here on the waves run independently
  if (t0 >= t1) return;

  unsigned char* tile = lds + wave * kWaveLds;
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
  ChunkWalk<R> walk;
  walk.init(p.offs, t0, t1, p.out.KT);
  uint32_t piece_tiles = 0;
  const unsigned char* frag = tile + ((lane >> 4) * kTileM + (lane & 15)) * 16;

  // gmem2reg: no branch may enclose these loads (the compiler's vmcnt bookkeeping would fall back to
  // "wait for everything" and the register ring would be lost), so a lane past the end of the
  // run, or a whole chunk past the end of the wave's tiles, is turned away by the bounds check of
  // the buffer descriptor instead: it returns 0 and moves no data.
  auto issue = [&](u32x4(&s)[R], half8(&x)[NB], const Chunk& c) {
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(p.words + c.begin), 0, (int)(c.n * 4u), kBufferFlags);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (FLS_ABLATE & 32) s[r] = u32x4{(uint32_t)lane, 1u, 2u, 3u};
      else s[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (r * 64 + lane) * 16, 0, kAuxNonTemporal);
    }
    xf.template load<NB>(x, c.kt);
  };

  // extract (Alg. 2): value = high half of the word, byte address = 2 * location
  auto extract = [&](const u32x4(&s)[R], const Chunk& c) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t q = r * 64 + lane;
      if (q * 4 < c.n) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t w = s[r][j];
          if (FLS_ABLATE & 4) asm volatile("" ::"v"(w));
          else *(uint16_t*)(tile + ((w & 0xffffu) << 1)) = (uint16_t)(w >> 16);
        }
      }
    }
  };

  // smem2tc + rst_smem for a completed tile.  Returns true when the tile ends a band or the wave's run.
  auto compute = [&](const half8(&x)[NB], const Chunk& c) -> bool {
#pragma unroll
    for (int h = 0; h < kRowBlocks; h += 4) {  // fragments of four row blocks at a time
      half8 a[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (FLS_ABLATE & 16) a[j] = x[0];
        else a[j] = *(const half8*)(frag + (h + j) * 256);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          if (FLS_ABLATE & 2) acc[h + j][nb][0] += (float)a[j][0] * (float)x[nb][0];
          else acc[h + j][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[j], x[nb], acc[h + j][nb], 0, 0, 0);
        }
      }
    }
    if (!(FLS_ABLATE & 8)) {
#pragma unroll
      for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
    }
    ++piece_tiles;
    return c.kt + 1 == p.out.KT || c.t + 1 == t1;
  };

  // Hand-over of the piece that just ended in `band` (outside the tile loop on purpose).
  auto hand_over = [&](uint32_t band) {
    if (FLS_ABLATE & 1) {
      float sum = 0.f;  // keeps every accumulator alive
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sum += acc[rb][nb][0] + acc[rb][nb][1] + acc[rb][nb][2] + acc[rb][nb][3];
      if (sum == 1234.5f) p.out.C[lane] = (_Float16)1;
    } else if ((FLS_ABLATE & 128) || piece_tiles == p.out.KT) {
      store_band<NB>(p.out, acc, band, lane);  // this wave alone saw the whole band
      if (!(FLS_ABLATE & 128)) wg_reduce_skip<NB>(red, band - share0 / p.out.KT, lane);
    } else {
      const uint32_t band_lo = band * p.out.KT;
      const uint32_t lo = share0 > band_lo ? share0 : band_lo;
      const uint32_t hi = share1 < band_lo + p.out.KT ? share1 : band_lo + p.out.KT;
      const uint32_t seq = band - share0 / p.out.KT;
      if (wg_reduce_add<NB>(red, acc, seq, piece_tiles, hi - lo, lane))
        finish_band<NB>(red, p.out.C, p.out.parts, p.out.cnt, p.out.M, p.out.N, p.out.n0, p.out.KT, p.out.T, seq, band, lo,
                        hi, share0, blockIdx.x, gridDim.x, (FLS_ABLATE & 64) != 0);
    }
    piece_tiles = 0;
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
  };

  // Register ring of NS chunks in flight.  A stage is refilled as soon as its words are in LDS,
  // before the MFMA work of its tile, so loads lead their use by NS - 1 tiles of work.  The tile
  // loop is straight-line in its global loads - every stage issues the same number, none under
  // a condition - which is what lets the compiler wait for exactly the stage it needs
  // (s_waitcnt vmcnt(n) with n = loads issued since); it is left only when a piece ends.
  u32x4 s[NS][R];
  half8 x[NS][NB];
  Chunk c[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    c[i] = walk.next();
    issue(s[i], x[i], c[i]);
  }
  uint32_t pos = 0, end_band = 0;

#define FLS_RING_STEP(i)                                  \
  if constexpr ((i) < NS) {                               \
    if (!c[i].valid) goto run_done;                       \
    const Chunk cur = c[i];                               \
    extract(s[i], cur);                                   \
    half8 xc[NB];                                         \
    _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) xc[nb] = x[i][nb]; \
    c[i] = walk.next();                                   \
    issue(s[i], x[i], c[i]);                              \
    if (cur.last && compute(xc, cur)) {                   \
      pos = (i);                                          \
      end_band = cur.band;                                \
      goto piece_done;                                    \
    }                                                     \
  }

  for (;;) {
    for (;;) {
      FLS_RING_STEP(0)
      FLS_RING_STEP(1)
      FLS_RING_STEP(2)
      FLS_RING_STEP(3)
    }
  piece_done:
    // bring the oldest stage to position 0 so that the tile loop can be entered from its top
    for (uint32_t k = (pos + 1) % NS; k > 0; --k) {
      u32x4 ts[R];
      half8 tx[NB];
      const Chunk tc = c[0];
#pragma unroll
      for (int r = 0; r < R; ++r) ts[r] = s[0][r];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) tx[nb] = x[0][nb];
#pragma unroll
      for (int i = 0; i + 1 < NS; ++i) {
        c[i] = c[i + 1];
#pragma unroll
        for (int r = 0; r < R; ++r) s[i][r] = s[i + 1][r];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) x[i][nb] = x[i + 1][nb];
      }
      c[NS - 1] = tc;
#pragma unroll
      for (int r = 0; r < R; ++r) s[NS - 1][r] = ts[r];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) x[NS - 1][nb] = tx[nb];
    }
    hand_over(end_band);
  }
run_done:
  return;
#undef FLS_RING_STEP
}

// ---------------------------------------------------------------- host launcher

#ifndef FLS_NSTAGE
#define FLS_NSTAGE 3
#endif
#ifndef FLS_WAVES
#define FLS_WAVES 8
#endif

template <int NB, int WAVES, int R>
static hipError_t launch_variant(const SpmmParams& p, int grid, hipStream_t stream) {
  constexpr int NS = NB == 1 ? FLS_NSTAGE : 2;  // wider accumulators leave room for a shallower ring
  static bool attr_done = false;
  const int lds_bytes = WAVES * kWaveLds + (int)sizeof(WgReduceLds<NB>);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)spmm_kernel<NB, WAVES, R, NS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       lds_bytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL((spmm_kernel<NB, WAVES, R, NS>), dim3(grid), dim3(WAVES * 64), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int NB, int WAVES>
static hipError_t launch_r(int R, const SpmmParams& p, int grid, hipStream_t stream) {
  switch (R) {
    case 2: return launch_variant<NB, WAVES, 2>(p, grid, stream);
    case 4: return launch_variant<NB, WAVES, 4>(p, grid, stream);
    case 6: return launch_variant<NB, WAVES, 6>(p, grid, stream);
    default: return launch_variant<NB, WAVES, 8>(p, grid, stream);
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
  p.out.cnt = a.cnt;
  p.out.M = a.M;
  p.out.N = a.N;
  p.out.KT = a.K / kTileK;
  const int grid = a.num_cus < kMaxGrid ? a.num_cus : kMaxGrid;
  // words staged per chunk: the smallest variant that takes the densest tile in one piece
  int R = 8;
  if (a.max_tile_words <= 2 * 256) R = 2;
  else if (a.max_tile_words <= 4 * 256) R = 4;
  else if (a.max_tile_words <= 6 * 256) R = 6;
  for (uint32_t n0 = 0; n0 < a.N; n0 += 64) {
    p.out.n0 = n0;
    const uint32_t ncols = a.N - n0 < 64 ? a.N - n0 : 64;
    hipError_t e;
    if (ncols <= 16) e = launch_r<1, FLS_WAVES>(R, p, grid, stream);
    else if (ncols <= 32) e = launch_r<2, FLS_WAVES>(R, p, grid, stream);
    else e = launch_r<4, FLS_WAVES>(R, p, grid, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace fls
