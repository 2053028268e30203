// Device-side building blocks shared by the sparse and the dense kernel: MFMA operand types,
// the split-K accumulation plane and the band arrival protocol.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fls {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTileM = 128;               // rows of a tile (one row band)
constexpr int kTileK = 32;                // K extent of a tile = K of one 16x16x32 MFMA
constexpr int kTileElems = kTileM * kTileK;
constexpr int kTileBytes = kTileElems * 2;  // dense fp16 tile in LDS
constexpr int kRowBlocks = kTileM / 16;     // 16-row MFMA blocks per tile

// What both kernels need to find their work and to hand results over.
struct OutParams {
  _Float16* C;      // column-major M x N
  float* plane;     // split-K accumulation plane [band][n_pad][128] fp32, all zero between calls
  uint32_t* cnt;    // [band] arrived K tiles, all zero between calls
  uint32_t M, N;    // N = columns of the whole problem
  uint32_t n0;      // first column of this launch's column group
  uint32_t n_pad;   // columns of the plane = N rounded up to 16
  uint32_t KT;      // K tiles per band
};

// One wave adds its 128 x (NB*16) partial result for `band` to the plane, announces that it
// covered `tiles` K tiles, and - if that completes the band - turns the plane into fp16 C and
// leaves plane and counter clear for the next call.
//
// MFMA 16x16 accumulator layout: lane l holds column (l & 15), rows 4*(l >> 4) .. +3.
template <int NB>
__device__ __forceinline__ void flush_band(const OutParams& o, float4v (&acc)[kRowBlocks][NB], uint32_t band,
                                           uint32_t tiles, int lane) {
  const uint32_t col = lane & 15, rsub = (lane >> 4) * 4;
  if (tiles == o.KT) {
    // the wave saw every K tile of this band: no other contribution exists, write C directly
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const uint32_t n = o.n0 + nb * 16 + col;
      if (n < o.N) {
#pragma unroll
        for (int rb = 0; rb < kRowBlocks; ++rb) {
          half4 h;
#pragma unroll
          for (int r = 0; r < 4; ++r) h[r] = (_Float16)acc[rb][nb][r];
          *(half4*)(o.C + (size_t)n * o.M + band * kTileM + rb * 16 + rsub) = h;
        }
      }
    }
    return;
  }
  float* plane = o.plane + ((size_t)band * o.n_pad + o.n0) * kTileM;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const uint32_t nl = nb * 16 + col;
    if (o.n0 + nl < o.N) {
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          __hip_atomic_fetch_add(plane + nl * kTileM + rb * 16 + rsub + r, acc[rb][nb][r], __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  // every add above is performed before the counter moves
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  uint32_t old = 0;
  if (lane == 0) old = __hip_atomic_fetch_add(o.cnt + band, tiles, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old + tiles != o.KT) return;
  // last arrival: every contribution is in the plane
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  const uint32_t ncols = (o.N - o.n0) < (uint32_t)(NB * 16) ? (o.N - o.n0) : (uint32_t)(NB * 16);
  for (uint32_t i = lane; i < ncols * kTileM; i += 64) {
    const float v = __hip_atomic_exchange(plane + i, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t nl = i / kTileM, m = i % kTileM;
    o.C[(size_t)(o.n0 + nl) * o.M + band * kTileM + m] = (_Float16)v;
  }
  if (lane == 0) __hip_atomic_store(o.cnt + band, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// B operand fragments (X) of one K tile, straight from global memory: lane l supplies column
// (l & 15) and the 8 consecutive k of chunk (l >> 4); X is column-major so they are one 16 B load.
template <int NB>
__device__ __forceinline__ void load_x_frags(half8 (&x)[NB], const _Float16* __restrict__ X, uint32_t K, uint32_t N,
                                             uint32_t n0, uint32_t kt, int lane) {
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const uint32_t n = n0 + nb * 16 + (lane & 15);
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (n < N) v = *(const half8*)(X + (size_t)n * K + kt * kTileK + (lane >> 4) * 8);
    x[nb] = v;
  }
}

}  // namespace fls
