// Host-side launch descriptors: the C ABI layer fills these, each kernel file implements its launcher.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fls {

struct SpmmLaunch {
  const uint32_t* offs;   // TileOffsets section of the blob
  const uint32_t* words;  // NonZeros section of the blob
  const _Float16* X;
  _Float16* C;
  float* parts;
  uint32_t* flags;
  _Float16* xpack;  // workspace area of xpack_bytes(K, N) for X in MFMA fragment order (used when N > 32)
  uint32_t M, K, N;
  uint32_t max_tile_words;
  uint32_t version;  // format version of the blob (1 or 2)
  int num_cus;
  // the partial-sum area was sized by parts_floats(N): a call of 17 - 32 columns may take the 64-column pass
  // (false for the static scratch of the entry point that allocates nothing, which has the narrow kernel's area only)
  bool wide32;
};

struct DenseLaunch {
  const _Float16* W;
  const _Float16* X;
  _Float16* C;
  float* parts;
  uint32_t* flags;
  _Float16* xpack;  // as in SpmmLaunch
  uint32_t M, K, N;
  int num_cus;
};

struct CompressLaunch {
  const uint16_t* W;
  unsigned char* out;  // blob
  uint32_t M, K;
  uint32_t policy;
  uint32_t version;  // 1: 32-bit words (value, location); 2: groups of four entries in three words, three bytes per entry
};

// Columns are processed in groups, one pass over W per group.  The dense baseline and the sparse
// kernel's narrow variants take up to kGroupCols columns (1 or 2 MFMA column blocks of 16 per
// wave); more than that goes to the sparse kernel's 64-column pass (four column blocks, four waves
// per workgroup with the whole register file each).
constexpr uint32_t kGroupCols = 32;
constexpr uint32_t kSpmmGroupCols = 64;
inline uint32_t group_blocks(uint32_t ncols) { return ncols <= 16 ? 1u : (ncols <= 32 ? 2u : 4u); }
constexpr uint32_t kMaxWorkgroups = 512;    // must equal fls::kMaxGrid of the device code
// The 64-column pass of the dense kernel cuts its work as (group of 4 bands) x (K slice), one wave
// per band, and keeps one 128 x 64 fp32 partial result per band and slice.  Slices per group: as
// many as fill the CUs, but none shorter than 16 steps.  groups * slices <= kMaxWorkgroups, so
// bands * slices <= 4 * kMaxWorkgroups partial results at most (what parts_floats provides).
inline uint32_t wide_slices(uint32_t bands, uint32_t col_groups, uint32_t KT, int cus) {
  if (cus > (int)kMaxWorkgroups) cus = (int)kMaxWorkgroups;
  const uint64_t units = (uint64_t)((bands + 3) / 4) * col_groups;  // (group of four bands, group of 64 columns)
  uint32_t S = units < (uint64_t)cus ? (uint32_t)((uint64_t)cus / units) : 1u;
  const uint32_t by_length = KT / 16u > 0 ? KT / 16u : 1u;
  return S < by_length ? S : by_length;
}
// The sparse 64-column pass: a workgroup takes four bands (one per wave), a group of 64 columns and a
// K slice made of whole loop bodies of `body` tiles, and writes one partial result per band, column
// group and slice.  Slices per (group of four bands, column group): as many as fill the CUs, none
// shorter than two bodies.  With S > 1, groups of bands x column groups x S <= CUs <= kMaxWorkgroups,
// so at most 4 * kMaxWorkgroups partial results exist (what parts_floats provides).
inline uint32_t wide_quad_slices(uint32_t bands, uint32_t col_groups, uint32_t KT, int cus, uint32_t body) {
  if (cus > (int)kMaxWorkgroups) cus = (int)kMaxWorkgroups;
  const uint64_t units = (uint64_t)((bands + 3) / 4) * col_groups;
  uint32_t S = units < (uint64_t)cus ? (uint32_t)((uint64_t)cus / units) : 1u;
  const uint32_t by_length = KT / (2u * body) > 0 ? KT / (2u * body) : 1u;
  return S < by_length ? S : by_length;
}
// fp32 values of the split-K partial sums: [workgroup][column blocks][128 x 16] for the passes of
// up to 32 columns, [band][slice][4][128 x 16] for the 64-column pass
inline size_t parts_floats(uint32_t N) {
  // (from 17 columns on: a call of 17 - 32 columns takes the 64-column pass where that is faster, see wide32_pays)
  if (N > 16u) return (size_t)4 * kMaxWorkgroups * 4 * 2048;
  return (size_t)kMaxWorkgroups * group_blocks(N) * 2048;
}

// A call (or the rest of a call) of 17 - 32 columns: the narrow kernel with two column blocks per wave, or the
// 64-column pass multiplying only its first 32-column block.  Every tile asks for 2 KB of X here, as much as a
// sparse tile's words, and the narrow kernel's waves fetch X from L2 each for themselves; the pass shares X between
// four bands through LDS.  Measured in format version 1 (us, narrow / pass): 12288 x 49152 at 90 % 73.7 / 63.2, 80 %
// 105.0 / 93.7, 70 % 135.5 / 117.5, 60 % 164.4 / 150.0, 50 % 200.1 / 184.7; 49152 x 12288 at 90 - 60 % 74.3 / 70.0,
// 104.6 / 101.7, 134.7 / 128.6, 164.4 / 157.6; 12288 x 24576 at 70 % 73.1 / 66.5; 12288 x 12288 at 90 - 50 % 28.2 / 27.3,
// 37.0 / 35.3, 44.2 / 41.3, 51.7 / 49.6, 60.8 / 58.5; but 28672 x 7168 at 90 % 28.7 / 31.4, at 80 % 40.3 / 41.6,
// 7168 x 7168 16.0 / 19.0: the pass pays its second kernel and needs long bands.  So, in version 1: bands of at
// least 384 K tiles, any tile the pass can stage (ten rounds).
// In format version 2 the narrow kernel has a quarter fewer bytes to wait for and stays ahead longer (12288 x
// 12288: 32.9 / 34.7 at 80 %, 26.2 / 27.2 at 90 %; 12288 x 49152 at 90 %: 65.6 / 62.7, at 70 %: 114.1 / 116.1; 49152 x
// 12288 at 70 %: 113.8 / 136.6): tiles of up to four rounds on bands of at least 1024 K tiles.
// Bands of 288 - 383 K tiles: the pass still wins where its K slices come out even and the tiles are not the
// sparsest (27648 x 9216 at 70 % 61.9 / 59.0, at 80 % 49.0 / 47.2, at 90 % 34.8 / 35.1; 20480 x 9216 at 80 % 42.1 /
// 37.7; 12288 x 10240 at 80 % 32.6 / 31.2, at 60 % 45.3 / 43.8; but 12288 x 9216 at 80 %, whose ten slices are
// three or four bodies long, 30.5 / 31.0, and 12288 x 8192 at 80 % 27.5 / 30.6).
inline bool wide32_pays(uint32_t max_tile_words, uint32_t round_words, uint32_t KT, uint32_t version, uint32_t bands, int cus) {
  if (version == 2u) return max_tile_words <= 4u * round_words && KT >= 1024u;
  if (max_tile_words > 10u * round_words) return false;
  if (KT >= 384u) return true;
  if (KT < 288u || max_tile_words <= 2u * round_words) return false;
  // the longest K slice at most a tenth above the mean (bodies of 8 tiles up to four rounds, of 4 beyond: as the pass picks them)
  const uint32_t body = max_tile_words <= 4u * round_words ? 8u : 4u;
  const uint32_t bodies = KT / body, S = wide_quad_slices(bands, 1u, KT, cus, body);
  return (uint64_t)((bodies + S - 1u) / S) * S * 10u <= (uint64_t)bodies * 11u;
}

// Workspace bytes for X repacked into MFMA fragment order, [K tile][column block][lane][8 halves]
// (the sparse kernel's wide variant reads it instead of X; narrower calls do not need it).
inline size_t xpack_bytes(uint32_t K, uint32_t N) {
  return N > kGroupCols ? (size_t)K * ((N + 15u) / 16u * 16u) * 2u : 0;
}

// Number of workgroups for a matrix of `bands` row bands on `cus` compute units (one workgroup
// per CU at most).  A count of the form bands * k gives every band to exactly k workgroups: with
// k = 1 no partial sum ever crosses between workgroups, and the serial hand-over chain at the end
// of the kernel (store, count, read back: a few microseconds with the whole chip waiting) goes
// away.  That is worth leaving up to a fifth of the CUs without a workgroup: the kernel is paced by
// HBM, not by the CUs.  Otherwise every CU gets an equal share, cut wherever it falls (see below
// for the one exception).
// A workgroup should also have enough tiles to amortise its start and its hand-over: small
// problems get fewer workgroups (at least kMinShare tiles each).
constexpr uint32_t kMinShare = 32;
inline int pick_grid(uint32_t bands, uint32_t tiles_per_band, int cus) {
  if (cus > (int)kMaxWorkgroups) cus = (int)kMaxWorkgroups;
  const uint64_t by_size = (uint64_t)bands * tiles_per_band / kMinShare;
  if (by_size < (uint64_t)cus) cus = by_size > 0 ? (int)by_size : 1;
  if ((int)bands <= cus) {
    const int aligned = (int)bands * (cus / (int)bands);
    if (aligned * 5 >= cus * 4) return aligned;
    // next best: every pair of bands to an odd number of workgroups (only the middle one of each
    // group spans two bands), if that leaves next to no CU idle - 168 bands on 256 CUs: 252
    // workgroups measured 3 % faster than 256
    const int j = 2 * cus / (int)bands;
    const int halves = (int)bands * j;
    if (halves % 2 == 0 && halves / 2 * 100 >= cus * 97) return halves / 2;
  }
  return cus;
}

// Arguments of the 64-column passes (sparse and dense) and of the kernel that adds their K slices.
struct WideParams {
  const uint32_t* offs;   // TileOffsets (sparse pass)
  const uint32_t* words;  // NonZeros (sparse pass)
  const _Float16* W;      // dense matrix (dense pass)
  const _Float16* X;      // X as the caller lays it out, column-major K x N (sparse pass)
  const _Float16* Xp;     // X in fragment order: [K tile][column block of all N][lane][8 halves] (dense pass)
  _Float16* C;
  float* parts;           // [band][slice][column block][row block][lane] float4, used when S > 1
  uint32_t M, K, N, n0, KT, bands, S;
  uint32_t G;  // groups of 64 columns in the launch, from column n0 on (sparse pass; 1 in the dense pass)
  uint32_t cb; // 32-column blocks of a group that are multiplied and hold sums (sparse pass: 2, or 1 for a call of at most 32 columns)
};

hipError_t launch_spmm(const SpmmLaunch& a, hipStream_t stream);
// X -> xpack (fragment order, all N columns): the dense 64-column passes read it
// `groups` groups of 64 columns of the sparse 64-column pass from column n0 on, in one launch
hipError_t launch_xpack(const _Float16* X, _Float16* xpack, uint32_t K, uint32_t N, hipStream_t stream);
hipError_t launch_spmm_wide(const SpmmLaunch& a, uint32_t n0, uint32_t groups, hipStream_t stream);
// C = sum over the S slices of parts, in slice order (the second kernel of a 64-column pass with S > 1);
// layout32: the partial results are in the 32x32 accumulator layout (sparse pass), else 16x16 (dense pass)
hipError_t launch_wide_reduce(const WideParams& p, bool layout32, hipStream_t stream);
hipError_t launch_dense(const DenseLaunch& a, hipStream_t stream);
// phase 1: per-tile counts, prefix sums, header (everything but the words)
hipError_t launch_compress_index(const CompressLaunch& a, hipStream_t stream);
// phase 2: the words
hipError_t launch_compress_emit(const CompressLaunch& a, hipStream_t stream);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);

}  // namespace fls
