// fls_dense_gemm: the dense fp16 baseline C = W . X for skinny N on gfx950, built like the sparse
// kernel minus its sparse stages (the paper pairs every SpMM point with a dense GEMM, Sec. 6):
// every wave owns a contiguous run of 128 x 64 steps of W, loads the MFMA A fragments straight
// from HBM (a lane's 8 consecutive k are one 16 B load), keeps a few tiles in flight in registers,
// takes X fragments from L2 and accumulates with v_mfma_f32_16x16x32_f16 in fp32.  Split-K as in
// the sparse kernel.
#include <atomic>

#include "fls_device.h"
#include "fls_launch.h"

namespace fls {

struct DenseParams {
  const _Float16* W;
  const _Float16* X;
  uint32_t K;
  OutParams out;
};

// A dense step covers 128 rows x 32*H k, i.e. H MFMA K-steps (H = 1 or 2).  With H = 2 lane l of
// row block rb reads 32 contiguous bytes of row rb*16 + (l & 15), so the four lanes of a row
// together read one whole 128 B line; the first 16 B feed the first MFMA, the second 16 B the
// second one (which 8 k a lane contributes to an MFMA is free as long as the B operand, X, uses
// the same ones, and it does).  H = 1 halves the registers a step holds, for the wider N.

template <int NB, int WAVES, int NS, int H>
__global__ __launch_bounds__(WAVES * 64) void dense_kernel(DenseParams p) {
  constexpr int kDenseK = 32 * H;
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t T = p.out.T, KT = p.out.KT;  // steps of 128 x 64 here
  const uint32_t share0 = share_begin(blockIdx.x, T, gridDim.x), share1 = share_begin(blockIdx.x + 1, T, gridDim.x);
  // The waves of a workgroup take the steps of its share in turn (wave w: share0 + w, + WAVES,
  // ...), so at any time they read neighbouring 128 B pieces of the same rows: 1 KB runs for the
  // DRAM instead of eight unrelated ones.
  const uint32_t t0 = share0 + wave, t1 = share1;
  extern __shared__ __align__(16) unsigned char lds[];
  WgReduceLds<NB>* red = (WgReduceLds<NB>*)lds;
  wg_reduce_init<NB>(red, threadIdx.x, WAVES * 64);
  __syncthreads();  // the only barrier
  if (t0 >= t1) return;

  float4v acc[kRowBlocks][NB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

  const uint32_t K = p.K;
  const uint32_t kgrp = (lane >> 4) * (8 * H);  // first of this lane's 8*H k inside a step
  const uint32_t lane_off = ((lane & 15) * K + kgrp) * 2u;
  const uint32_t rb_step = 16u * K * 2u;
  // X through a descriptor that ends after column N - 1 (padding columns read 0)
  const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)p.X, 0, (int)(p.out.N * K * 2u), kBufferFlags);
  const uint32_t x_lane_off = ((p.out.n0 + (lane & 15)) * K + kgrp) * 2u;
  const uint32_t x_col_step = 16u * K * 2u;
  // K need not be a multiple of 64: in the last step of a band the lanes whose k lie past K drop out
  const bool ragged = (K % kDenseK) != 0;
  const bool lane_past = kgrp + 8 * H > (K % kDenseK);  // this lane's k are past K in a ragged last step

  // load side (ti) runs NS steps ahead of the consume side (tc)
  uint32_t ti = t0, kti = t0 % KT, bandi = t0 / KT;
  uint32_t tc = t0, ktc = kti, bandc = bandi, piece_tiles = 0;

  // No branch encloses the ring's loads: a step past the end of the wave's run gets an empty
  // buffer descriptor, whose loads return 0 and move no data.  In a ragged last step the lanes
  // past K read the next row's first bytes (inside the descriptor); they are zeroed before use.
  auto issue = [&](half8(&a)[kRowBlocks][H], half8(&x)[NB][H]) {
    const _Float16* base = p.W + ((size_t)bandi * kTileM * K + (size_t)kti * kDenseK);
    const uint32_t kleft = K - kti * kDenseK;  // k from this step's start to the end of the row
    const uint32_t span = (127u * K + (kleft < (uint32_t)kDenseK ? kleft : (uint32_t)kDenseK)) * 2u;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, ti < t1 ? (int)span : 0, kBufferFlags);
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int h = 0; h < H; ++h)
        a[rb][h] = __builtin_bit_cast(
            half8, __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + rb * rb_step + h * 16, 0, kAuxNonTemporal));
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int h = 0; h < H; ++h)
        x[nb][h] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, x_lane_off + nb * x_col_step + h * 16,
                                                                                 kti * (kDenseK * 2u), 0));
    ti += WAVES;
    kti += WAVES;
    while (kti >= KT) {
      kti -= KT;
      ++bandi;
    }
  };

  HandoverState hs;
  half8 a[NS][kRowBlocks][H], x[NS][NB][H];
#pragma unroll
  for (int i = 0; i < NS; ++i) issue(a[i], x[i]);

  auto step = [&](half8(&sa)[kRowBlocks][H], half8(&sx)[NB][H]) {
    if (ragged && ktc + 1 == KT && lane_past) {
      // k past the end of the row: take them out of the product (X side is enough)
      const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int h = 0; h < H; ++h) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sx[nb][h] = z;
#pragma unroll
        for (int rb = 0; rb < kRowBlocks; ++rb) sa[rb][h] = z;
      }
    }
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int h = 0; h < H; ++h)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(sa[rb][h], sx[nb][h], acc[rb][nb], 0, 0, 0);
    issue(sa, sx);
    ++piece_tiles;
    tc += WAVES;
    ktc += WAVES;
    if (ktc >= KT || tc >= t1) {  // the wave's next step is in another band, or there is none
      hand_over_piece<NB>(p.out, red, acc, hs, bandc, piece_tiles, share0, share1, blockIdx.x, lane, false, false);
      piece_tiles = 0;
      while (ktc >= KT) {
        ktc -= KT;
        ++bandc;
      }
    }
  };

  while (tc + (NS - 1) * WAVES < t1) {
#pragma unroll
    for (int i = 0; i < NS; ++i) step(a[i], x[i]);
  }
#pragma unroll
  for (int i = 0; i < NS - 1; ++i)
    if (tc < t1) step(a[i], x[i]);
  hand_over_finish<NB>(p.out, acc, hs, blockIdx.x, gridDim.x, lane);
}

template <int NB, int WAVES, int NS, int H>
static hipError_t launch_dense_variant(const DenseParams& p, int grid, hipStream_t stream) {
  static std::atomic<bool> attr_done{false};  // per kernel variant; setting the attribute twice from two threads is harmless
  const int lds_bytes = (int)sizeof(WgReduceLds<NB>);
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)dense_kernel<NB, WAVES, NS, H>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((dense_kernel<NB, WAVES, NS, H>), dim3(grid), dim3(WAVES * 64), lds_bytes, stream, p);
  return hipGetLastError();
}

// ---------------------------------------------------------------- 64 columns per pass
//
// More than 32 columns: W is streamed once per 64 columns.  Four waves per workgroup, one per SIMD
// with the whole register file (128 accumulator registers), each on its own row band; work is cut
// as (group of four bands) x (K slice) as in the sparse kernel's 64-column pass, whose repacked X
// (one coalesced 1 KB block per K tile and column block) and slice-adding kernel it shares.  No
// LDS, no barrier, no waiting between workgroups.  A step covers 128 rows x 64 k: lane l reads 32
// contiguous bytes of its row, so four lanes read a whole 128 B line, and the two MFMA K-steps of
// a step take the first and the second 16 B; X follows the same assignment of k to lanes.
constexpr int kDenseWideRing = 2;  // steps of 128 x 64 in flight per wave

template <int NS>
__global__ __launch_bounds__(256) void dense_wide_kernel(WideParams p) {
  constexpr int NB = 4;
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // (group of four bands, K slice) pair and group of 64 columns of this workgroup: as in the sparse
  // pass, the G workgroups that stream the same rows of W get ids 8 apart, which puts them on one
  // XCD one after the other, so that all but the first find W in its L2
  const uint32_t pairs = ((p.bands + 3u) / 4u) * p.S;
  const uint32_t cg = (blockIdx.x >> 3) % p.G, pair = ((blockIdx.x >> 3) / p.G) * 8u + (blockIdx.x & 7u);
  if (pair >= pairs) return;
  const uint32_t group = pair / p.S, slice = pair - group * p.S;
  const uint32_t n0 = p.n0 + cg * 64u;
  const uint32_t band = group * 4 + wave;
  if (band >= p.bands) return;
  const uint32_t K = p.K, KT = p.KT;  // KT: steps of 64 k per band (the last one may be half)
  const uint32_t s0 = (uint32_t)((uint64_t)slice * KT / p.S), s1 = (uint32_t)((uint64_t)(slice + 1) * KT / p.S);

  float4v acc[kRowBlocks][NB];
#pragma unroll
  for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

  const uint32_t g = lane >> 4, c = lane & 15;
  const _Float16* wband = p.W + (size_t)band * kTileM * K;
  const uint32_t lane_off = (c * K + g * 16u) * 2u, rb_step = 16u * K * 2u;
  // X: K tile 2 s + (g >> 1) of step s; inside its block, the slot of k chunk 2 (g & 1) + h
  const uint32_t ktiles = K / kTileK, xblocks = (p.N + 15u) / 16u;
  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.Xp, 0, (int)(ktiles * xblocks * 1024u), kBufferFlags);
  const uint32_t xlane = (n0 / 16u) * 1024u + ((2u * (g & 1u)) * 16u + c) * 16u;
  const uint32_t xvalid = n0 / 16u < xblocks ? xblocks - n0 / 16u : 0u;  // column blocks left from n0 on: the others read as zero
  // a half last step (K = 64 j + 32): the lanes of its upper 32 k drop out
  const bool half_last = (K & 63u) != 0;
  const bool upper = g >= 2;

  uint32_t si = s0;  // next step to request
  auto issue = [&](half8(&a)[kRowBlocks][2], half8(&x)[NB][2]) {
    // past the slice: an empty descriptor, loads return 0 and move no data
    const uint32_t kleft = K - si * 64u;
    const uint32_t span = (127u * K + (kleft < 64u ? kleft : 64u)) * 2u;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(wband + (size_t)si * 64u), 0, si < s1 ? (int)span : 0, kBufferFlags);
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int h = 0; h < 2; ++h)
        a[rb][h] = __builtin_bit_cast(
            half8, __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + rb * rb_step + h * 16, 0, kAuxNonTemporal));
    const uint32_t kt = 2u * si + (g >> 1);
    const bool live = si < s1 && kt < ktiles;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int h = 0; h < 2; ++h)
        x[nb][h] = __builtin_bit_cast(
            half8, __builtin_amdgcn_raw_buffer_load_b128(
                       xrsrc, live && (uint32_t)nb < xvalid ? kt * xblocks * 1024u + xlane + nb * 1024u + h * 256u : 0xffffff00u, 0, 0));
    ++si;
  };

  half8 a[NS][kRowBlocks][2], x[NS][NB][2];
#pragma unroll
  for (int i = 0; i < NS; ++i) issue(a[i], x[i]);
  uint32_t sc = s0;
  auto step = [&](half8(&sa)[kRowBlocks][2], half8(&sx)[NB][2]) {
    if (half_last && sc + 1 == KT && upper) {
      // k past the end of the row: X read as zero there, W must not bring Inf or NaN either
      const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
        for (int h = 0; h < 2; ++h) sa[rb][h] = z;
    }
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb)
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(sa[rb][h], sx[nb][h], acc[rb][nb], 0, 0, 0);
    issue(sa, sx);
    ++sc;
  };
  while (sc + NS <= s1) {
#pragma unroll
    for (int i = 0; i < NS; ++i) step(a[i], x[i]);
  }
#pragma unroll
  for (int i = 0; i < NS - 1; ++i)
    if (sc < s1) step(a[i], x[i]);

  if (p.S == 1) {
    OutParams o;
    o.C = p.C;
    o.M = p.M;
    o.N = p.N;
    o.n0 = n0;
    store_band<NB>(o, acc, band, lane);
  } else {
    float4v* dst = (float4v*)p.parts + ((size_t)((band * p.G + cg) * p.S + slice) * (NB * kRowBlocks)) * 64 + lane;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb) dst[(nb * kRowBlocks + rb) * 64] = acc[rb][nb];
  }
}

// `col_groups` groups of 64 columns from column n0 on, in one launch (the last group may reach past N)
static hipError_t launch_dense_wide(const DenseLaunch& a, uint32_t n0, uint32_t col_groups, hipStream_t stream) {
  WideParams p;
  p.cb = 2;
  p.offs = nullptr;
  p.words = nullptr;
  p.W = a.W;
  p.X = nullptr;
  p.G = col_groups;
  p.Xp = a.xpack;
  p.C = a.C;
  p.parts = a.parts;
  p.M = a.M;
  p.K = a.K;
  p.N = a.N;
  p.n0 = n0;
  p.KT = (a.K + 63u) / 64u;
  p.bands = a.M / kTileM;
  p.S = wide_slices(p.bands, col_groups, p.KT, a.num_cus);
  const uint32_t groups = (p.bands + 3u) / 4u;
  const uint32_t grid = (groups * p.S + 7u) / 8u * 8u * col_groups;
  hipLaunchKernelGGL((dense_wide_kernel<kDenseWideRing>), dim3(grid), dim3(256), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && p.S > 1) e = launch_wide_reduce(p, false, stream);
  return e;
}

hipError_t launch_dense(const DenseLaunch& a, hipStream_t stream) {
  DenseParams p;
  p.W = a.W;
  p.X = a.X;
  p.K = a.K;
  p.out.C = a.C;
  p.out.parts = a.parts;
  p.out.flags = a.flags;
  p.out.M = a.M;
  p.out.N = a.N;
  const int grid = pick_grid(a.M / kTileM, a.K / kTileK, a.num_cus);
  if (a.N > kGroupCols) {
    hipError_t e = launch_xpack(a.X, a.xpack, a.K, a.N, stream);  // the 64-column passes read X in fragment order
    if (e != hipSuccess) return e;
  }
  for (uint32_t n0 = 0; n0 < a.N;) {
    p.out.n0 = n0;
    const uint32_t left = a.N - n0;
    hipError_t e;
    if (left > kGroupCols) {
      const uint32_t col_groups = left / kSpmmGroupCols + (left % kSpmmGroupCols > kGroupCols ? 1u : 0u);
      e = launch_dense_wide(a, n0, col_groups, stream);
      n0 += col_groups * kSpmmGroupCols;
    } else {
      const uint32_t h = left <= 16 ? 2 : 1;
      p.out.KT = (a.K + 32 * h - 1) / (32 * h);
      p.out.T = (a.M / kTileM) * p.out.KT;
      if (left <= 16) e = launch_dense_variant<1, 8, 2, 2>(p, grid, stream);
      else e = launch_dense_variant<2, 8, 2, 1>(p, grid, stream);
      n0 += kGroupCols;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace fls
