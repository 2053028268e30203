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
// Split-K: the tile sequence (band-major) is cut evenly over all waves of the grid; a wave that
// holds only part of a band adds to an fp32 plane and the last arrival writes C.
#include "fls_device.h"
#include "fls_launch.h"

namespace fls {

constexpr int kWaveLds = kTileBytes + 16;  // + the slot that padding words land in

struct SpmmParams {
  const uint32_t* offs;   // TileOffsets
  const uint32_t* words;  // NonZeros
  const _Float16* X;
  uint32_t K;
  uint32_t T;  // tiles in total
  OutParams out;
};

// A run of at most R*256 words of one tile.
struct Chunk {
  uint32_t begin, n;  // word range [begin, begin + n) in NonZeros
  uint32_t t, kt, band;  // tile id, its K tile and row band
  bool last;   // completes its tile
  bool valid;
};

template <int R>
struct ChunkWalk {
  const uint32_t* offs;
  uint32_t t, t_end, KT;
  uint32_t pos, end, end_next;
  uint32_t kt, band;

  __device__ __forceinline__ void init(const uint32_t* offs_, uint32_t t0, uint32_t t1, uint32_t KT_) {
    offs = offs_;
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

template <int NB, int WAVES, int R>
__global__ __launch_bounds__(WAVES * 64) void spmm_kernel(SpmmParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t g = blockIdx.x * WAVES + wave, G = gridDim.x * WAVES;
  const uint32_t t0 = (uint32_t)((uint64_t)g * p.T / G), t1 = (uint32_t)((uint64_t)(g + 1) * p.T / G);
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

  ChunkWalk<R> walk;
  walk.init(p.offs, t0, t1, p.out.KT);
  uint32_t piece_tiles = 0;
  const unsigned char* frag = tile + ((lane >> 4) * kTileM + (lane & 15)) * 16;

  auto issue = [&](u32x4(&s)[R], half8(&x)[NB], const Chunk& c) {
    if (!c.valid) return;
    const u32x4* src = (const u32x4*)(p.words + c.begin);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t q = r * 64 + lane;
      if (q * 4 < c.n) s[r] = __builtin_nontemporal_load(src + q);
    }
    load_x_frags<NB>(x, p.X, p.K, p.out.N, p.out.n0, c.kt, lane);
  };

  auto consume = [&](u32x4(&s)[R], half8(&x)[NB], const Chunk& c) {
    // extract (Alg. 2): value = high half of the word, byte address = 2 * location
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t q = r * 64 + lane;
      if (q * 4 < c.n) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t w = s[r][j];
          *(uint16_t*)(tile + ((w & 0xffffu) << 1)) = (uint16_t)(w >> 16);
        }
      }
    }
    if (!c.last) return;
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb) {
      const half8 a = *(const half8*)(frag + rb * 256);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, x[nb], acc[rb][nb], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kTileBytes / 1024; ++i) *(u32x4*)(tile + i * 1024 + lane * 16) = zero4;
    ++piece_tiles;
    if (c.kt + 1 == p.out.KT || c.t + 1 == t1) {
      // the band ends here, or the wave's run does
      flush_band<NB>(p.out, acc, c.band, piece_tiles, lane);
      piece_tiles = 0;
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
    }
  };

  u32x4 sa[R], sb[R];
  half8 xa[NB], xb[NB];
  Chunk ca = walk.next();
  issue(sa, xa, ca);
  Chunk cb = walk.next();
  issue(sb, xb, cb);
  while (true) {
    if (!ca.valid) break;
    consume(sa, xa, ca);
    ca = walk.next();
    issue(sa, xa, ca);
    if (!cb.valid) break;
    consume(sb, xb, cb);
    cb = walk.next();
    issue(sb, xb, cb);
  }
}

// ---------------------------------------------------------------- host launcher

template <int NB, int WAVES, int R>
static hipError_t launch_variant(const SpmmParams& p, int grid, hipStream_t stream) {
  static bool attr_done = false;
  const int lds_bytes = WAVES * kWaveLds;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)spmm_kernel<NB, WAVES, R>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       lds_bytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL((spmm_kernel<NB, WAVES, R>), dim3(grid), dim3(WAVES * 64), lds_bytes, stream, p);
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
  p.T = (a.M / kTileM) * (a.K / kTileK);
  p.out.C = a.C;
  p.out.plane = a.plane;
  p.out.cnt = a.cnt;
  p.out.M = a.M;
  p.out.N = a.N;
  p.out.n_pad = (a.N + 15) / 16 * 16;
  p.out.KT = a.K / kTileK;
  // words staged per chunk: the smallest variant that takes the densest tile in one piece
  int R = 8;
  if (a.max_tile_words <= 2 * 256) R = 2;
  else if (a.max_tile_words <= 4 * 256) R = 4;
  else if (a.max_tile_words <= 6 * 256) R = 6;
  for (uint32_t n0 = 0; n0 < a.N; n0 += 64) {
    p.out.n0 = n0;
    const uint32_t ncols = a.N - n0 < 64 ? a.N - n0 : 64;
    hipError_t e;
    if (ncols <= 16) e = launch_r<1, 8>(R, p, a.num_cus, stream);
    else if (ncols <= 32) e = launch_r<2, 8>(R, p, a.num_cus, stream);
    else e = launch_r<4, 8>(R, p, a.num_cus, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace fls
