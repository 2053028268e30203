// Device-side building blocks shared by the sparse and the dense kernel: MFMA operand types,
// the split-K hand-over of partial bands.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fls {

// Debug builds only (-DFLS_TRACE): 100 MHz timestamps of the hand-over steps, kept in the unused
// tail of the counter area: cnt[65536 + 16 * workgroup + k].
#ifdef FLS_TRACE
#define FLS_STAMP(cnt, wg, k)                                                             \
  do {                                                                                    \
    if ((threadIdx.x & 63) == 0) (cnt)[65536 + 16 * (wg) + (k)] = (uint32_t)wall_clock64(); \
  } while (0)
#else
#define FLS_STAMP(cnt, wg, k) \
  do {                        \
  } while (0)
#endif

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTileM = 128;               // rows of a tile (one row band)
constexpr int kTileK = 32;                // K extent of a tile = K of one 16x16x32 MFMA
constexpr int kTileElems = kTileM * kTileK;
constexpr int kTileBytes = kTileElems * 2;  // dense fp16 tile in LDS
constexpr int kRowBlocks = kTileM / 16;     // 16-row MFMA blocks per tile

constexpr int kAccPerBlock = kTileM * 16;   // fp32 values of one 128 x 16 column block
constexpr int kMaxGrid = 512;               // workgroups a launch may use (sizes the workspace)
constexpr int kBufferFlags = 0x00020000;    // raw buffer, 32-bit data format (gfx9 descriptor word 3)
constexpr int kAuxNonTemporal = 2;          // nt: streamed once, do not keep in the caches
constexpr int kAuxCoherent = 16;            // sc1: device scope - through to memory / past the per-XCD L2

// What both kernels need to hand results over.
//
// Split-K: the band-major tile sequence [0, T) is cut evenly over the workgroups, then over the
// waves of a workgroup.  Partial results of one band meet in two steps:
//   1. inside a workgroup, in LDS (wg_reduce): waves add their accumulators to one of two band
//      slots and count their tiles; the wave that completes the workgroup's share takes the sum;
//   2. between workgroups, in HBM (band_handover): that wave stores the sum to its workgroup's
//      slot, counts the share in the band's arrival counter, and the workgroup that completes
//      the band adds up the slots in workgroup order and writes fp16 C.
// No floating-point atomics touch HBM; counters return to zero, so the workspace is reusable.
struct OutParams {
  _Float16* C;      // column-major M x N
  float* parts;     // [workgroup][2][NB * 2048] fp32 partial sums in accumulator order
  uint32_t* cnt;    // [band] arrived K tiles, all zero between calls
  uint32_t M, N;    // N = columns of the whole problem
  uint32_t n0;      // first column of this launch's column group
  uint32_t KT;      // K tiles per band
  uint32_t T;       // tiles in total
};

// First tile of workgroup q's share when T tiles are cut over P workgroups.
__device__ __forceinline__ uint32_t share_begin(uint32_t q, uint32_t T, uint32_t P) {
  return (uint32_t)((uint64_t)q * T / P);
}

// MFMA 16x16 accumulator layout: lane l holds column (l & 15), rows 4*(l >> 4) .. +3 of its block.
// Converts a wave's 128 x (NB*16) accumulators to fp16 and stores them to column-major C.
template <int NB>
__device__ __forceinline__ void store_band(const OutParams& o, const float4v (&acc)[kRowBlocks][NB], uint32_t band,
                                           int lane) {
  const uint32_t col = lane & 15, rsub = (lane >> 4) * 4;
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
}

// LDS area of the in-workgroup step: two band slots and their control words.
// A slot keeps a band's running sum as [column block][row block][lane] float4.
template <int NB>
struct WgReduceLds {
  float4v slot[2][NB * kRowBlocks * 64];
  uint32_t cnt[2];   // tiles added to the slot so far
  uint32_t gen[2];   // how many bands the slot has served
  uint32_t lock[2];  // 1 while a wave is adding to the slot
};

template <int NB>
__device__ __forceinline__ void wg_reduce_init(WgReduceLds<NB>* red, int tid, int nthreads) {
  for (int i = tid; i < 2 * NB * kRowBlocks * 64; i += nthreads) (&red->slot[0][0])[i] = float4v{0.f, 0.f, 0.f, 0.f};
  if (tid < 2) {
    red->cnt[tid] = 0;
    red->gen[tid] = 0;
    red->lock[tid] = 0;
  }
}

// Adds a wave's accumulators for the seq-th band of its workgroup (seq counts from the
// workgroup's first band) to the band's slot.  Returns true for exactly one wave per band: the
// one whose tiles complete `expected`; the slot then holds the workgroup's sum (wg_reduce_take
// collects it).  Waves take turns on a slot under a spin lock and add with plain 16 B
// read-add-write; LDS floating-point atomics would need no lock but run about fifty times
// slower per instruction on this chip than a plain LDS access.
template <int NB>
__device__ __forceinline__ bool wg_reduce_add(WgReduceLds<NB>* red, const float4v (&acc)[kRowBlocks][NB], uint32_t seq,
                                              uint32_t tiles, uint32_t expected, int lane) {
  const uint32_t s = seq & 1u, turn = seq >> 1;
  // the slot may still serve band seq - 2 (only when a workgroup's share spans more than two bands)
  while (__hip_atomic_load(&red->gen[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != turn)
    __builtin_amdgcn_s_sleep(2);
  for (;;) {
    uint32_t got = 1;
    if (lane == 0) got = __hip_atomic_exchange(&red->lock[s], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (__builtin_amdgcn_readfirstlane(got) == 0) break;
    __builtin_amdgcn_s_sleep(1);
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  float4v* d = &red->slot[s][lane];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb) d[(nb * kRowBlocks + rb) * 64] += acc[rb][nb];
  uint32_t old = 0;
  if (lane == 0) {
    old = red->cnt[s];
    red->cnt[s] = old + tiles;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  if (lane == 0) __hip_atomic_store(&red->lock[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  old = __builtin_amdgcn_readfirstlane(old);
  return old + tiles == expected;
}

// Run by the wave wg_reduce_add picked: moves the slot's sum into acc and frees the slot for band seq + 2.
template <int NB>
__device__ __forceinline__ void wg_reduce_take(WgReduceLds<NB>* red, float4v (&acc)[kRowBlocks][NB], uint32_t seq,
                                               int lane) {
  const uint32_t s = seq & 1u, turn = seq >> 1;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  float4v* d = &red->slot[s][lane];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb) {
      acc[rb][nb] = d[(nb * kRowBlocks + rb) * 64];
      d[(nb * kRowBlocks + rb) * 64] = float4v{0.f, 0.f, 0.f, 0.f};
    }
  if (lane == 0) red->cnt[s] = 0;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  if (lane == 0) __hip_atomic_store(&red->gen[s], turn + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// A wave that saw a whole band by itself has nothing to reduce, but the band still takes its turn
// on the slot so that the turn count of later bands stays right.
template <int NB>
__device__ __forceinline__ void wg_reduce_skip(WgReduceLds<NB>* red, uint32_t seq, int lane) {
  const uint32_t s = seq & 1u, turn = seq >> 1;
  while (__hip_atomic_load(&red->gen[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != turn)
    __builtin_amdgcn_s_sleep(2);
  if (lane == 0) __hip_atomic_store(&red->gen[s], turn + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// The between-workgroups step, run by the one wave per (workgroup, band) that wg_reduce picked.
// acc is the workgroup's sum over tiles [lo, hi) of `band`; share0 is the first tile of the
// workgroup's share, wg its index, P the number of workgroups.
template <int NB>
__device__ __forceinline__ void band_handover(const OutParams& o, float4v (&acc)[kRowBlocks][NB], uint32_t band,
                                              uint32_t lo, uint32_t hi, uint32_t share0, uint32_t wg, uint32_t P,
                                              int lane) {
  const uint32_t band_lo = band * o.KT, band_hi = band_lo + o.KT;
  if (lo == band_lo && hi == band_hi) {
    store_band<NB>(o, acc, band, lane);  // the workgroup saw the whole band
    return;
  }
  // slot 0: the band in which the workgroup's share begins; slot 1: a later band (only its last,
  // cut-off band can be partial, so each slot is used at most once per call)
  const uint32_t my_slot = share0 < band_lo ? 1u : 0u;
  // Partial sums cross between the L2 caches of different XCDs.  They are written through to
  // memory and read past the caches access by access (sc1 on the instruction), so that no
  // cache-wide write-back or invalidate - what a device-scope fence costs - is needed: waiting
  // for the stores to be acknowledged orders them before the counter.  A slot is kept as
  // [column block][row block][lane] float4, 1 KB per instruction.
  constexpr int kSlotBytes = NB * kAccPerBlock * 4;
  FLS_STAMP(o.cnt, wg, 2 + 6 * my_slot);
  {
    const __amdgpu_buffer_rsrc_t mine = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(o.parts + ((size_t)wg * 2 + my_slot) * (NB * kAccPerBlock)), 0, kSlotBytes, kBufferFlags);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rb = 0; rb < kRowBlocks; ++rb)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[rb][nb]), mine,
                                               ((nb * kRowBlocks + rb) * 64 + lane) * 16, 0, kAuxCoherent);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // s_waitcnt vmcnt(0): the stores are done
  FLS_STAMP(o.cnt, wg, 3 + 6 * my_slot);
  uint32_t old = 0;
  if (lane == 0) old = __hip_atomic_fetch_add(o.cnt + band, hi - lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  old = __builtin_amdgcn_readfirstlane(old);
  FLS_STAMP(o.cnt, wg, 4 + 6 * my_slot);
  if (old + (hi - lo) != o.KT) return;
  // last arrival: every share of this band is stored; add them in workgroup order.  The loads
  // of up to kBatch shares are all issued before the first is used: each is a trip to memory,
  // and this code runs when the kernel is about to end, with nothing left to hide it behind.
  constexpr int kBatch = NB == 1 ? 4 : (NB == 2 ? 2 : 1);
  uint32_t q = (uint32_t)((uint64_t)band_lo * P / o.T);
  while (q > 0 && share_begin(q, o.T, P) > band_lo) --q;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rb = 0; rb < kRowBlocks; ++rb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};
  while (q < P && share_begin(q, o.T, P) < band_hi) {
    u32x4 v[kBatch][NB][kRowBlocks];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      // next share that overlaps the band; past the last one the descriptor is empty and reads 0
      uint32_t qb = 0, qe = 0;
      bool found = false;
      while (!found && q < P && share_begin(q, o.T, P) < band_hi) {
        qb = share_begin(q, o.T, P);
        qe = share_begin(q + 1, o.T, P);
        found = qe > band_lo && qe != qb;
        if (!found) ++q;
      }
      const uint32_t slot = qb < band_lo ? 1u : 0u;
      const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(o.parts + ((size_t)(found ? q : 0u) * 2 + slot) * (NB * kAccPerBlock)), 0, found ? kSlotBytes : 0,
          kBufferFlags);
      if (found) ++q;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int rb = 0; rb < kRowBlocks; ++rb)
          v[j][nb][rb] = __builtin_amdgcn_raw_buffer_load_b128(src, ((nb * kRowBlocks + rb) * 64 + lane) * 16, 0, kAuxCoherent);
    }
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int rb = 0; rb < kRowBlocks; ++rb) acc[rb][nb] += __builtin_bit_cast(float4v, v[j][nb][rb]);
  }
  FLS_STAMP(o.cnt, wg, 5 + 6 * my_slot);
  store_band<NB>(o, acc, band, lane);
  if (lane == 0) __hip_atomic_store(o.cnt + band, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  FLS_STAMP(o.cnt, wg, 6 + 6 * my_slot);
}

// Everything the picked wave does after its own contribution, kept out of line: it runs at most
// twice per workgroup and call, and inlined into the tile loop it would cost the loop its registers.
template <int NB>
__device__ __noinline__ void finish_band(WgReduceLds<NB>* red, _Float16* C, float* parts, uint32_t* cnt, uint32_t M,
                                         uint32_t N, uint32_t n0, uint32_t KT, uint32_t T, uint32_t seq, uint32_t band,
                                         uint32_t lo, uint32_t hi, uint32_t share0, uint32_t wg, uint32_t P,
                                         bool local_only) {
  const int lane = threadIdx.x & 63;
  OutParams o;
  o.C = C;
  o.parts = parts;
  o.cnt = cnt;
  o.M = M;
  o.N = N;
  o.n0 = n0;
  o.KT = KT;
  o.T = T;
  float4v acc[kRowBlocks][NB];
  wg_reduce_take<NB>(red, acc, seq, lane);
  if (local_only) store_band<NB>(o, acc, band, lane);
  else band_handover<NB>(o, acc, band, lo, hi, share0, wg, P, lane);
}

// B operand fragments (X) of one K tile, straight from global memory (they stay in L2): lane l
// supplies column (l & 15) and the 8 consecutive k of chunk (l >> 4); X is column-major so they
// are one 16 B load.  The loads go through a buffer descriptor that ends after column N - 1, so
// the columns that pad N up to a multiple of 16 read as zero without a branch or a select after
// the load (either would make the compiler wait for the load on the spot).
struct XFrags {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t lane_off;  // byte offset of this lane's column and k chunk
  uint32_t col_step;  // bytes between column blocks

  __device__ __forceinline__ void init(const _Float16* X, uint32_t K, uint32_t N, uint32_t n0, int lane) {
    rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)(N * K * 2u), kBufferFlags);
    lane_off = ((n0 + (lane & 15)) * K + (lane >> 4) * 8) * 2u;
    col_step = 16u * K * 2u;
  }
  template <int NB>
  __device__ __forceinline__ void load(half8 (&x)[NB], uint32_t kt) const {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      x[nb] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + nb * col_step,
                                                                              kt * (kTileK * 2u), 0));
  }
};

}  // namespace fls
