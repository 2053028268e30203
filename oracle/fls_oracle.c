/*
 * CPU oracle for the Load-as-Sparse / Compute-as-Dense SpMM (Flash-LLM, arxiv 2309.10285).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
 * library is checked against.  Nothing in the product path may call it, and it shares
 * no code, header, table or helper with the HIP sources.  It is written from the paper:
 *
 *   - problem statement  C = A x B, A = weights [M,K], B = activations [K,N]   (Sec. 2.2)
 *   - Tiled-CSL: per-tile runs of 32-bit words, value in the high 16 bits and the
 *     in-tile location in the low 16 bits, plus a TileOffsets array of run starts
 *     (Sec. 4.3.1, Sec. 4.3.2, Alg. 3)
 *   - ahead-of-time reordering of a tile's words by target memory bank (Sec. 4.3.3, Alg. 3)
 *   - "no computation is skipped": zeros take part as zeros, so the SpMM result is the
 *     dense product of the masked matrix (Sec. 6.2)
 *
 * Parity status of each function
 *   flso_half_to_double, flso_double_to_half : pinned (exhaustive / library cross-check)
 *   flso_compress, flso_decompress (policy 0): pinned (hand-worked tile, independent decoder,
 *                                              bit-exact round trip, closed-form sizes)
 *   flso_compress policy 1 (bank-aware order): the multiset of words is pinned by the same
 *       tests; the exact sequence is fixed only by this build's reading of Alg. 3, whose
 *       printed listing is inconsistent -> "parity unpinned" with respect to the paper for
 *       the sequence, pinned for the invariants (every group drawn while all banks are
 *       non-empty holds distinct banks; same multiset as policy 0).
 *   flso_spmm_f64 : pinned (library fp64 matmul, identity X, exact small-integer cases)
 *
 * Layouts (all little endian):
 *   W  : M x K fp16 bit patterns, row-major (ld = K)             (Alg. 3 addresses A + x*K + y)
 *   X  : K x N fp16, column-major (ld = K)  == row-major [N][K]
 *   C  : M x N, column-major (ld = M)       == row-major [N][M]
 *
 * Compressed blob:
 *   [0,64)    header: u32 magic 'FLS1', u32 version, u32 tile_m, u32 tile_k, u32 pad_words,
 *             u32 order_policy, u32 max_tile_words, u32 reserved(0),
 *             u64 M, u64 K, u64 nnz, u64 total_words
 *   [64, 64+4*n_off)  TileOffsets, u32 word offsets into NonZeros; entry t is the start of
 *             tile t, entry num_tiles is total_words, and every further entry up to
 *             n_off = round_up(num_tiles + 4, 16) repeats total_words (look-ahead guard,
 *             Alg. 1 reads two tiles ahead)
 *   then      NonZeros, u32 words, total_words of them
 *   Tiles are visited band by band: tile id t = i*(K/tile_k) + j for row band i, K tile j (Alg. 3).
 *   An element is stored iff its 16-bit pattern is not 0x0000 (so -0.0, NaN, Inf and subnormals
 *   are kept and the round trip is bit exact).
 *   word = (bits << 16) | loc, loc = (y/8)*(tile_m*8) + x*8 + (y%8) for row x and column y of
 *   the tile: the position of the element in the on-chip dense tile, which is kept as
 *   [K-chunk of 8][row][8 halves] so that a matrix-core operand fragment is one contiguous 16 B read.
 *   Each run is padded to a multiple of pad_words with the word (0x0000 << 16) | tile_m*tile_k.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FLSO_MAGIC 0x31534C46u /* "FLS1" */
#define FLSO_VERSION 1u
#define FLSO_HEADER_BYTES 64u

/* ---------------------------------------------------------------- fp16 <-> fp64 */

/* Exact widening of an IEEE binary16 bit pattern. */
double flso_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int f = h & 0x3ff;
  double v;
  if (e == 0) {
    v = ldexp((double)f, -24); /* zero and subnormals: f * 2^-24 */
  } else if (e == 31) {
    v = f ? NAN : INFINITY;
  } else {
    v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */
  }
  return sign ? -v : v;
}

/* Round to nearest, ties to even, fp64 -> binary16 bit pattern. */
uint16_t flso_double_to_half(double d) {
  uint16_t sign = signbit(d) ? 0x8000u : 0u;
  if (isnan(d)) return (uint16_t)(sign | 0x7e00u);
  double a = fabs(d);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* halfway to 2^16 rounds to even = Inf */
  if (a < ldexp(1.0, -14)) {
    /* subnormal range (and the carry into the smallest normal): units of 2^-24 */
    double q = rint(ldexp(a, 24)); /* rint = current mode = nearest-even */
    return (uint16_t)(sign | (uint16_t)q);
  }
  int ex;
  double m = frexp(a, &ex); /* a = m * 2^ex, m in [0.5,1) */
  int e = ex - 1;           /* a = (2m) * 2^e, 2m in [1,2) */
  double q = rint(ldexp(m, 11)); /* (2m)*1024 in [1024,2048] */
  if (q >= 2048.0) {
    q = 1024.0;
    e += 1;
  }
  if (e + 15 >= 31) return (uint16_t)(sign | 0x7c00u);
  return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)q - 1024));
}

void flso_half_to_double_array(const uint16_t* in, double* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = flso_half_to_double(in[i]);
}

void flso_double_to_half_array(const double* in, uint16_t* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = flso_double_to_half(in[i]);
}

/* ---------------------------------------------------------------- blob helpers */

static void put_u32(uint8_t* p, uint32_t v) { memcpy(p, &v, 4); }
static void put_u64(uint8_t* p, uint64_t v) { memcpy(p, &v, 8); }
static uint32_t get_u32(const uint8_t* p) {
  uint32_t v;
  memcpy(&v, p, 4);
  return v;
}
static uint64_t get_u64(const uint8_t* p) {
  uint64_t v;
  memcpy(&v, p, 8);
  return v;
}

static uint64_t round_up_u64(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

static int geometry_ok(int64_t M, int64_t K, uint32_t tile_m, uint32_t tile_k, uint32_t pad) {
  if (M <= 0 || K <= 0 || tile_m == 0 || tile_k == 0 || pad == 0) return 0;
  if (tile_k % 8 != 0) return 0;
  if ((uint64_t)tile_m * tile_k > 65535u) return 0; /* loc and the sentinel must fit 16 bits */
  if (M % tile_m != 0 || K % tile_k != 0) return 0;
  return 1;
}

/* Position of tile element (x,y) in the on-chip dense tile (the word's low 16 bits). */
static uint32_t loc_of(uint32_t x, uint32_t y, uint32_t tile_m) {
  return (y / 8u) * (tile_m * 8u) + x * 8u + (y % 8u);
}

/* Memory bank that a 16-bit store to half-index loc falls in: banks are 4 bytes wide,
 * so two neighbouring halves share a bank; `banks` of them interleave. */
static uint32_t bank_of(uint32_t loc, uint32_t banks) { return (loc >> 1) % banks; }

/* ---------------------------------------------------------------- compressor (Alg. 3) */

/*
 * Orders the nz words of one tile (already in ascending-loc order in `w`) by the bank-aware
 * policy and writes them to `out`.
 *
 * Reading of Alg. 3 used here: words are bucketed by target bank; the run is emitted in
 * groups of `group` words; a group takes at most one word from each bank, visiting banks in
 * order of decreasing remaining count (ties: lower bank first), each bank giving its
 * lowest-loc remaining word; if fewer than `group` banks are non-empty the group is filled by
 * repeating that visit order over the banks that still hold words.
 */
static void order_bank_aware(const uint32_t* w, uint32_t nz, uint32_t banks, uint32_t group,
                             uint32_t* out) {
  uint32_t* count = (uint32_t*)calloc(banks, sizeof(uint32_t));
  uint32_t* head = (uint32_t*)calloc(banks, sizeof(uint32_t));
  uint32_t* start = (uint32_t*)calloc(banks + 1, sizeof(uint32_t));
  uint32_t* bucket = (uint32_t*)malloc((nz ? nz : 1) * sizeof(uint32_t));
  uint32_t* order = (uint32_t*)malloc(banks * sizeof(uint32_t));
  for (uint32_t i = 0; i < nz; ++i) count[bank_of(w[i] & 0xffffu, banks)]++;
  for (uint32_t b = 0; b < banks; ++b) start[b + 1] = start[b] + count[b];
  {
    uint32_t* fill = (uint32_t*)calloc(banks, sizeof(uint32_t));
    for (uint32_t i = 0; i < nz; ++i) { /* stable: ascending loc inside a bucket */
      uint32_t b = bank_of(w[i] & 0xffffu, banks);
      bucket[start[b] + fill[b]++] = w[i];
    }
    free(fill);
  }
  uint32_t emitted = 0;
  while (emitted < nz) {
    uint32_t want = nz - emitted < group ? nz - emitted : group;
    uint32_t got = 0;
    while (got < want) {
      /* visit order for this sweep: remaining count descending, bank id ascending */
      uint32_t live = 0;
      for (uint32_t b = 0; b < banks; ++b)
        if (head[b] < count[b]) order[live++] = b;
      for (uint32_t i = 1; i < live; ++i) { /* insertion sort, stable */
        uint32_t b = order[i];
        uint32_t rb = count[b] - head[b];
        uint32_t j = i;
        while (j > 0 && (count[order[j - 1]] - head[order[j - 1]]) < rb) {
          order[j] = order[j - 1];
          --j;
        }
        order[j] = b;
      }
      for (uint32_t i = 0; i < live && got < want; ++i) {
        uint32_t b = order[i];
        out[emitted + got] = bucket[start[b] + head[b]];
        head[b]++;
        got++;
      }
    }
    emitted += want;
  }
  free(count);
  free(head);
  free(start);
  free(bucket);
  free(order);
}

/*
 * Dense masked W -> blob.  Returns the number of bytes the blob needs; writes it only if
 * out != NULL and cap is large enough.  Returns 0 on bad geometry.
 * policy 0: ascending loc.  policy 1: bank-aware order with `banks` banks, groups of `group`.
 */
size_t flso_compress(const uint16_t* W, int64_t M, int64_t K, uint32_t tile_m, uint32_t tile_k,
                     uint32_t pad, uint32_t policy, uint32_t banks, uint32_t group, uint8_t* out,
                     size_t cap) {
  if (!geometry_ok(M, K, tile_m, tile_k, pad)) return 0;
  if (policy > 1) return 0;
  if (policy == 1 && (banks == 0 || group == 0)) return 0;
  const uint64_t tiles_k = (uint64_t)K / tile_k;
  const uint64_t num_tiles = ((uint64_t)M / tile_m) * tiles_k;
  const uint64_t n_off = round_up_u64(num_tiles + 4, 16);
  const uint32_t sentinel = tile_m * tile_k; /* value bits 0x0000, loc one past the tile */

  /* pass 1: sizes */
  uint64_t nnz = 0, total_words = 0, max_tile_words = 0;
  for (uint64_t t = 0; t < num_tiles; ++t) {
    const uint64_t i = t / tiles_k, j = t % tiles_k;
    uint64_t nz = 0;
    for (uint32_t x = 0; x < tile_m; ++x)
      for (uint32_t y = 0; y < tile_k; ++y)
        if (W[(i * tile_m + x) * (uint64_t)K + j * tile_k + y] != 0) nz++;
    uint64_t words = round_up_u64(nz, pad);
    nnz += nz;
    total_words += words;
    if (words > max_tile_words) max_tile_words = words;
  }
  if (total_words > 0xffffffffull) return 0; /* u32 offsets */
  const size_t need = (size_t)(FLSO_HEADER_BYTES + 4 * n_off + 4 * total_words);
  if (out == NULL || cap < need) return need;

  put_u32(out + 0, FLSO_MAGIC);
  put_u32(out + 4, FLSO_VERSION);
  put_u32(out + 8, tile_m);
  put_u32(out + 12, tile_k);
  put_u32(out + 16, pad);
  put_u32(out + 20, policy);
  put_u32(out + 24, (uint32_t)max_tile_words);
  put_u32(out + 28, 0);
  put_u64(out + 32, (uint64_t)M);
  put_u64(out + 40, (uint64_t)K);
  put_u64(out + 48, nnz);
  put_u64(out + 56, total_words);

  uint8_t* offs = out + FLSO_HEADER_BYTES;
  uint8_t* nzw = offs + 4 * n_off;
  uint32_t* tmp = (uint32_t*)malloc((size_t)tile_m * tile_k * sizeof(uint32_t));
  uint32_t* tmp2 = (uint32_t*)malloc((size_t)tile_m * tile_k * sizeof(uint32_t));
  uint64_t pos = 0;
  for (uint64_t t = 0; t < num_tiles; ++t) {
    const uint64_t i = t / tiles_k, j = t % tiles_k;
    put_u32(offs + 4 * t, (uint32_t)pos);
    uint32_t nz = 0;
    /* ascending loc = K-chunk of 8, then row, then position in the chunk */
    for (uint32_t c = 0; c < tile_k / 8; ++c)
      for (uint32_t x = 0; x < tile_m; ++x)
        for (uint32_t e = 0; e < 8; ++e) {
          uint32_t y = c * 8 + e;
          uint16_t bits = W[(i * tile_m + x) * (uint64_t)K + j * tile_k + y];
          if (bits != 0) tmp[nz++] = ((uint32_t)bits << 16) | loc_of(x, y, tile_m);
        }
    const uint32_t* src = tmp;
    if (policy == 1) {
      order_bank_aware(tmp, nz, banks, group, tmp2);
      src = tmp2;
    }
    for (uint32_t q = 0; q < nz; ++q) put_u32(nzw + 4 * (pos + q), src[q]);
    pos += nz;
    while (pos % pad != 0) {
      put_u32(nzw + 4 * pos, sentinel);
      pos++;
    }
  }
  for (uint64_t t = num_tiles; t < n_off; ++t) put_u32(offs + 4 * t, (uint32_t)pos);
  free(tmp);
  free(tmp2);
  return need;
}

/* Worst-case blob size (every element stored). */
size_t flso_compress_bound(int64_t M, int64_t K, uint32_t tile_m, uint32_t tile_k, uint32_t pad) {
  if (!geometry_ok(M, K, tile_m, tile_k, pad)) return 0;
  const uint64_t num_tiles = ((uint64_t)M / tile_m) * ((uint64_t)K / tile_k);
  const uint64_t n_off = round_up_u64(num_tiles + 4, 16);
  const uint64_t per_tile = round_up_u64((uint64_t)tile_m * tile_k, pad);
  return (size_t)(FLSO_HEADER_BYTES + 4 * n_off + 4 * num_tiles * per_tile);
}

/*
 * Header fields -> out[12] = {magic, version, tile_m, tile_k, pad, policy, max_tile_words,
 * reserved, M, K, nnz, total_words}.  Returns 0 if the header is well formed and consistent
 * with `bytes`, else a negative code naming the first failed check.
 */
int flso_inspect(const uint8_t* blob, size_t bytes, uint64_t* out) {
  if (bytes < FLSO_HEADER_BYTES) return -1;
  for (int q = 0; q < 8; ++q) out[q] = get_u32(blob + 4 * q);
  for (int q = 0; q < 4; ++q) out[8 + q] = get_u64(blob + 32 + 8 * q);
  if (out[0] != FLSO_MAGIC) return -2;
  if (out[1] != FLSO_VERSION) return -3;
  if (!geometry_ok((int64_t)out[8], (int64_t)out[9], (uint32_t)out[2], (uint32_t)out[3],
                   (uint32_t)out[4]))
    return -4;
  const uint64_t num_tiles = (out[8] / out[2]) * (out[9] / out[3]);
  const uint64_t n_off = round_up_u64(num_tiles + 4, 16);
  if (bytes < FLSO_HEADER_BYTES + 4 * n_off + 4 * out[11]) return -5;
  return 0;
}

/* blob -> dense M x K bit patterns.  Returns 0, or a negative code on a malformed blob. */
int flso_decompress(const uint8_t* blob, size_t bytes, uint16_t* W, int64_t M, int64_t K) {
  uint64_t h[12];
  int rc = flso_inspect(blob, bytes, h);
  if (rc != 0) return rc;
  if ((int64_t)h[8] != M || (int64_t)h[9] != K) return -6;
  const uint32_t tile_m = (uint32_t)h[2], tile_k = (uint32_t)h[3];
  const uint64_t tiles_k = (uint64_t)K / tile_k;
  const uint64_t num_tiles = ((uint64_t)M / tile_m) * tiles_k;
  const uint64_t n_off = round_up_u64(num_tiles + 4, 16);
  const uint8_t* offs = blob + FLSO_HEADER_BYTES;
  const uint8_t* nzw = offs + 4 * n_off;
  const uint32_t sentinel_loc = tile_m * tile_k;
  memset(W, 0, (size_t)M * (size_t)K * sizeof(uint16_t));
  for (uint64_t t = 0; t < num_tiles; ++t) {
    const uint64_t i = t / tiles_k, j = t % tiles_k;
    const uint32_t a = get_u32(offs + 4 * t), b = get_u32(offs + 4 * (t + 1));
    if (b < a || b > h[11]) return -7;
    for (uint32_t q = a; q < b; ++q) {
      const uint32_t word = get_u32(nzw + 4 * (uint64_t)q);
      const uint32_t loc = word & 0xffffu;
      const uint16_t bits = (uint16_t)(word >> 16);
      if (loc == sentinel_loc) {
        if (bits != 0) return -8;
        continue;
      }
      if (loc > sentinel_loc) return -9;
      const uint32_t c = loc / (tile_m * 8u);
      const uint32_t x = (loc % (tile_m * 8u)) / 8u;
      const uint32_t y = c * 8u + loc % 8u;
      uint16_t* dst = &W[(i * tile_m + x) * (uint64_t)K + j * tile_k + y];
      if (*dst != 0) return -10; /* a location may be given once */
      *dst = bits;
    }
  }
  return 0;
}

/* ---------------------------------------------------------------- SpMM definition */

/*
 * C[n*M + m] = sum_k W[m][k] * X[k][n], k ascending, every operand widened exactly to fp64,
 * products and sums in fp64 (Sec. 2.2 problem statement; zeros are not skipped, Sec. 6.2).
 * W row-major M x K, X column-major K x N (X[n*K + k]), C column-major M x N.
 * Rows of W are independent; they are split over OpenMP threads, each row keeps its own
 * ascending-k order, so the result does not depend on the thread count.
 */
void flso_spmm_f64_rows(const uint16_t* W, const uint16_t* X, double* C, int64_t M, int64_t K,
                        int64_t N, int64_t m0, int64_t m1);

void flso_spmm_f64(const uint16_t* W, const uint16_t* X, double* C, int64_t M, int64_t K,
                   int64_t N) {
  flso_spmm_f64_rows(W, X, C, M, K, N, 0, M);
}

/* The definition on rows [m0, m1) only (C is still addressed with ld = M; other rows untouched). */
void flso_spmm_f64_rows(const uint16_t* W, const uint16_t* X, double* C, int64_t M, int64_t K,
                        int64_t N, int64_t m0, int64_t m1) {
  double* Xd = (double*)malloc((size_t)K * (size_t)N * sizeof(double));
  for (int64_t q = 0; q < K * N; ++q) Xd[q] = flso_half_to_double(X[q]);
#pragma omp parallel
  {
    double* row = (double*)malloc((size_t)K * sizeof(double));
#pragma omp for schedule(static)
    for (int64_t m = m0; m < m1; ++m) {
      for (int64_t k = 0; k < K; ++k) row[k] = flso_half_to_double(W[m * K + k]);
      for (int64_t n = 0; n < N; ++n) {
        double s = 0.0;
        for (int64_t k = 0; k < K; ++k) s += row[k] * Xd[n * K + k];
        C[n * M + m] = s;
      }
    }
    free(row);
  }
  free(Xd);
}

#ifdef _OPENMP
#include <omp.h>
int flso_threads(void) { return omp_get_max_threads(); }
#else
int flso_threads(void) { return 1; }
#endif
