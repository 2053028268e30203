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
  uint32_t T;
  OutParams out;
};

template <int NB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void dense_kernel(DenseParams p) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t g = blockIdx.x * WAVES + wave, G = gridDim.x * WAVES;
  const uint32_t t0 = (uint32_t)((uint64_t)g * p.T / G), t1 = (uint32_t)((uint64_t)(g + 1) * p.T / G);
  if (t0 >= t1) return;
  const uint32_t KT = p.out.KT;

  float4v acc[kRowBlocks][NB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

  // lane l of row block rb reads row rb*16 + (l & 15), k chunk (l >> 4)
  const size_t lane_off = (size_t)(lane & 15) * p.K + (lane >> 4) * 8;

  auto issue = [&](half8(&a)[kRowBlocks], half8(&x)[NB], uint32_t t) {
    if (t >= t1) return;
    const uint32_t band = t / KT, kt = t - band * KT;
    const _Float16* src = p.W + (size_t)band * kTileM * p.K + kt * kTileK + lane_off;
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
      a[rb] = __builtin_nontemporal_load((const half8*)(src + (size_t)rb * 16 * p.K));
    load_x_frags<NB>(x, p.X, p.K, p.out.N, p.out.n0, kt, lane);
  };

  uint32_t piece_tiles = 0;
  auto consume = [&](half8(&a)[kRowBlocks], half8(&x)[NB], uint32_t t) {
    const uint32_t band = t / KT, kt = t - band * KT;
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[rb], x[nb], acc[rb][nb], 0, 0, 0);
    ++piece_tiles;
    if (kt + 1 == KT || t + 1 == t1) {
      flush_band<NB>(p.out, acc, band, piece_tiles, lane);
      piece_tiles = 0;
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
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
}

template <int NB, int WAVES>
static hipError_t launch_dense_variant(const DenseParams& p, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((dense_kernel<NB, WAVES>), dim3(grid), dim3(WAVES * 64), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_dense(const DenseLaunch& a, hipStream_t stream) {
  DenseParams p;
  p.W = a.W;
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
  for (uint32_t n0 = 0; n0 < a.N; n0 += 64) {
    p.out.n0 = n0;
    const uint32_t ncols = a.N - n0 < 64 ? a.N - n0 : 64;
    hipError_t e;
    if (ncols <= 16) e = launch_dense_variant<1, 8>(p, a.num_cus, stream);
    else if (ncols <= 32) e = launch_dense_variant<2, 8>(p, a.num_cus, stream);
    else e = launch_dense_variant<4, 8>(p, a.num_cus, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace fls
