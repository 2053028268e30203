// fls_dense_gemm: the dense fp16 baseline C = W . X for skinny N on gfx950, built like the sparse
// kernel minus its sparse stages (the paper pairs every SpMM point with a dense GEMM, Sec. 6):
// every wave owns a contiguous run of 128 x 32 tiles of W, loads the MFMA A fragments straight
// from HBM (a lane's 8 consecutive k are one 16 B load), keeps two tiles in flight in registers,
// takes X fragments from L2 and accumulates with v_mfma_f32_16x16x32_f16 in fp32.  Split-K as in
// the sparse kernel.
#include "fls_device.h"
#include "fls_launch.h"

namespace fls {

struct DenseParams {
  const _Float16* W;
  const _Float16* X;
  uint32_t K;
  OutParams out;
};

template <int NB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void dense_kernel(DenseParams p) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t g = blockIdx.x * WAVES + wave, G = gridDim.x * WAVES;
  const uint32_t T = p.out.T;
  const uint32_t t0 = (uint32_t)((uint64_t)g * T / G), t1 = (uint32_t)((uint64_t)(g + 1) * T / G);
  const uint32_t share0 = share_begin(blockIdx.x, T, gridDim.x), share1 = share_begin(blockIdx.x + 1, T, gridDim.x);
  extern __shared__ __align__(16) unsigned char lds[];
  WgReduceLds<NB>* red = (WgReduceLds<NB>*)lds;
  wg_reduce_init<NB>(red, threadIdx.x, WAVES * 64);
  __syncthreads();  // the only barrier
  if (t0 >= t1) return;
  const uint32_t KT = p.out.KT;

  float4v acc[kRowBlocks][NB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

  XFrags xf;
  xf.init(p.X, p.K, p.out.N, p.out.n0, lane);
  // lane l of row block rb reads row rb*16 + (l & 15), k chunk (l >> 4)
  const size_t lane_off = (size_t)(lane & 15) * p.K + (lane >> 4) * 8;

  auto issue = [&](half8(&a)[kRowBlocks], half8(&x)[NB], uint32_t t) {
    if (t >= t1) return;
    const uint32_t band = t / KT, kt = t - band * KT;
    const _Float16* src = p.W + (size_t)band * kTileM * p.K + kt * kTileK + lane_off;
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
      a[rb] = __builtin_nontemporal_load((const half8*)(src + (size_t)rb * 16 * p.K));
    xf.template load<NB>(x, kt);
  };

  uint32_t piece_tiles = 0;
  HandoverState hs;
  auto consume = [&](half8(&a)[kRowBlocks], half8(&x)[NB], uint32_t t) {
    const uint32_t band = t / KT, kt = t - band * KT;
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[rb], x[nb], acc[rb][nb], 0, 0, 0);
    ++piece_tiles;
    if (kt + 1 == KT || t + 1 == t1) {
      hand_over_piece<NB>(p.out, red, acc, hs, band, piece_tiles, share0, share1, blockIdx.x, lane, false);
      piece_tiles = 0;
    }
  };

  half8 aa[kRowBlocks], ab[kRowBlocks], xa[NB], xb[NB];
  issue(aa, xa, t0);
  issue(ab, xb, t0 + 1);
  for (uint32_t t = t0; t < t1; t += 2) {
    consume(aa, xa, t);
    issue(aa, xa, t + 2);
    if (t + 1 >= t1) break;
    consume(ab, xb, t + 1);
    issue(ab, xb, t + 3);
  }
  hand_over_finish<NB>(p.out, acc, hs, blockIdx.x, gridDim.x, lane);
}

template <int NB, int WAVES>
static hipError_t launch_dense_variant(const DenseParams& p, int grid, hipStream_t stream) {
  static bool attr_done = false;
  const int lds_bytes = (int)sizeof(WgReduceLds<NB>);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)dense_kernel<NB, WAVES>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL((dense_kernel<NB, WAVES>), dim3(grid), dim3(WAVES * 64), lds_bytes, stream, p);
  return hipGetLastError();
}

hipError_t launch_dense(const DenseLaunch& a, hipStream_t stream) {
  DenseParams p;
  p.W = a.W;
  p.X = a.X;
  p.K = a.K;
  p.out.T = (a.M / kTileM) * (a.K / kTileK);
  p.out.C = a.C;
  p.out.parts = a.parts;
  p.out.flags = a.flags;
  p.out.M = a.M;
  p.out.N = a.N;
  p.out.KT = a.K / kTileK;
  const int grid = pick_grid(a.M / kTileM, a.num_cus);
  for (uint32_t n0 = 0; n0 < a.N; n0 += 64) {
    p.out.n0 = n0;
    p.out.epoch = a.epoch0 + n0 / 64;
    const uint32_t ncols = a.N - n0 < 64 ? a.N - n0 : 64;
    hipError_t e;
    if (ncols <= 16) e = launch_dense_variant<1, 8>(p, grid, stream);
    else if (ncols <= 32) e = launch_dense_variant<2, 8>(p, grid, stream);
    else e = launch_dense_variant<4, 8>(p, grid, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace fls
