/*
 * CPU oracle, format version 2: Tiled-CSL with the in-tile locations of four entries packed into one
 * word - the first one in full, the others as 6-bit distances (3 bytes per nonzero instead of 4).
 *
 * TEST INFRASTRUCTURE ONLY, like fls_oracle.c: the slow, plain definition the HIP library's
 * version-2 compressor is checked against bit for bit.  Nothing in the product path may call it,
 * and it shares no code with the HIP sources.
 *
 * Where it comes from.  The paper stores every nonzero as a 32-bit word, 16 bits of value and 16
 * bits of location (Sec. 4.3.2), and notes under Eq. 2 that its intensity model leaves the bytes
 * of the sparse indices out: with them the sparse load moves 4 B per kept weight, so it only breaks
 * even with the dense load at 50 % sparsity.  Version 2 is this build's own narrowing of that
 * overhead: a tile's entries are kept in ascending location order (Alg. 3's order before the bank
 * reordering) and go in groups of four that share one word of location data.  What the format
 * decodes to - the dense tile - is unchanged, so the SpMM definition (fls_oracle.c) is too.
 *
 * Parity status: flso2_compress / flso2_decompress / flso2_inspect are pinned by a tile encoded by
 * hand from the rules below (tests/golden/tiled_csl_v2_hand_tile.json), by an independent decoder
 * written in the test, by bit-exact round trips (special values, empty and full tiles, gaps at and
 * beyond 63 locations) and by closed-form sizes.  The format itself is this build's, not the paper's.
 *
 * Blob (little endian):
 *   [0,64)   header as in version 1 with magic 'FLS2', version 2, pad = 4 (entries per group),
 *            order_policy 0; max_tile_words and total_words count 32-bit words of NonZeros
 *   [64, 64 + 4 n_off)  TileOffsets as in version 1 (u32 word offsets, n_off = round_up(tiles + 4, 16),
 *            entries from num_tiles on repeat total_words); every offset is a multiple of 3
 *   then     NonZeros: groups of four entries in three words:
 *              word 0 = value0 | value1 << 16,  word 1 = value2 | value3 << 16,
 *              word 2 = loc0 | dist1 << 12 | dist2 << 18 | dist3 << 24   (12 + 3 x 6 bits; bits 30, 31 are 0)
 *            loc0 = the location of entry 0, distK = location of entry K minus location of entry K - 1.
 *   Locations are those of version 1 (loc = (y/8)*(tile_m*8) + x*8 + y%8; a tile has at most 4096).
 *   The entries of a tile, in ascending location, are of three kinds:
 *     - a stored element (16-bit pattern != 0x0000) at its location;
 *     - a bridge, value 0x0000, wherever the next stored element lies more than 63 locations behind
 *       the entry before it (behind location 0 for the first): bridges stand 63, 126, ... locations
 *       behind that entry until 63 or fewer are left.  A bridge names a location between two stored
 *       elements, which is empty, so decoding it (a zero written to a zero) changes nothing.  The
 *       rule is the same wherever in a group the next entry falls, also where it starts a group and
 *       would not need it: the number of entries of a tile then does not depend on how they fall
 *       into groups;
 *     - padding up to a multiple of four entries, value 0x0000 and distance 1: the locations behind
 *       the tile's last entry (empty), possibly up to three past the end of the tile.  A group never
 *       starts with padding.
 *   A group is decoded by itself - nothing is carried from one group to the next - which is what the
 *   format is for: on the GPU a lane takes a group, and its four scatter addresses cost it three
 *   additions, with no sum across lanes.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FLSO2_MAGIC 0x32534C46u /* "FLS2" */
#define FLSO2_VERSION 2u
#define FLSO2_HEADER_BYTES 64u
#define FLSO2_GROUP 4u /* entries per group */
#define FLSO2_REACH 63u /* largest distance a 6-bit field holds */

static void put32(uint8_t* p, uint32_t v) { memcpy(p, &v, 4); }
static void put64(uint8_t* p, uint64_t v) { memcpy(p, &v, 8); }
static uint32_t get32(const uint8_t* p) {
  uint32_t v;
  memcpy(&v, p, 4);
  return v;
}
static uint64_t get64(const uint8_t* p) {
  uint64_t v;
  memcpy(&v, p, 8);
  return v;
}
static uint64_t round_up64(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

static int geometry2_ok(int64_t M, int64_t K, uint32_t tile_m, uint32_t tile_k) {
  if (M <= 0 || K <= 0 || tile_m == 0 || tile_k == 0) return 0;
  if (tile_k % 8 != 0) return 0;
  if ((uint64_t)tile_m * tile_k > 4096u) return 0; /* loc0 has 12 bits */
  if (M % tile_m != 0 || K % tile_k != 0) return 0;
  return 1;
}

/*
 * The entries of tile (i, j), in order: values to val[], locations to loc[] (each with room for
 * tile_m*tile_k + 8 entries: a bridge stands for 63 empty locations, so entries never outnumber
 * locations).  Returns the number of entries (a multiple of four); *stored = elements stored.
 */
static uint32_t tile_entries(const uint16_t* W, int64_t K, uint64_t i, uint64_t j, uint32_t tile_m,
                             uint32_t tile_k, uint16_t* val, uint32_t* locs, uint64_t* stored) {
  uint32_t n = 0, last = 0; /* last = location of the entry before (0 before the first) */
  uint64_t nz = 0;
  /* ascending location = K-chunk of 8, then row, then position in the chunk */
  for (uint32_t c = 0; c < tile_k / 8; ++c)
    for (uint32_t x = 0; x < tile_m; ++x)
      for (uint32_t e = 0; e < 8; ++e) {
        const uint32_t y = c * 8 + e;
        const uint16_t bits = W[(i * tile_m + x) * (uint64_t)K + j * tile_k + y];
        if (bits == 0) continue;
        const uint32_t loc = c * (tile_m * 8u) + x * 8u + e;
        while (loc - last > FLSO2_REACH) { /* bridge over a long run of empty locations */
          last += FLSO2_REACH;
          val[n] = 0;
          locs[n] = last;
          n++;
        }
        val[n] = bits;
        locs[n] = loc;
        last = loc;
        n++;
        nz++;
      }
  while (n % FLSO2_GROUP != 0) { /* padding: the next (empty) locations */
    last += 1;
    val[n] = 0;
    locs[n] = last;
    n++;
  }
  *stored = nz;
  return n;
}

/*
 * Dense masked W -> version-2 blob.  Returns the number of bytes the blob needs; writes it only if
 * out != NULL and cap is large enough.  Returns 0 on bad geometry.
 */
size_t flso2_compress(const uint16_t* W, int64_t M, int64_t K, uint32_t tile_m, uint32_t tile_k, uint8_t* out,
                      size_t cap) {
  if (!geometry2_ok(M, K, tile_m, tile_k)) return 0;
  const uint64_t tiles_k = (uint64_t)K / tile_k;
  const uint64_t num_tiles = ((uint64_t)M / tile_m) * tiles_k;
  const uint64_t n_off = round_up64(num_tiles + 4, 16);
  const size_t room = (size_t)tile_m * tile_k + 8;
  uint16_t* val = (uint16_t*)malloc(room * sizeof(uint16_t));
  uint32_t* locs = (uint32_t*)malloc(room * sizeof(uint32_t));

  /* pass 1: sizes */
  uint64_t nnz = 0, total_words = 0, max_tile_words = 0;
  for (uint64_t t = 0; t < num_tiles; ++t) {
    uint64_t nz;
    const uint32_t n = tile_entries(W, K, t / tiles_k, t % tiles_k, tile_m, tile_k, val, locs, &nz);
    const uint64_t words = (uint64_t)n / FLSO2_GROUP * 3u;
    nnz += nz;
    total_words += words;
    if (words > max_tile_words) max_tile_words = words;
  }
  const size_t need = (size_t)(FLSO2_HEADER_BYTES + 4 * n_off + 4 * total_words);
  if (total_words > 0xffffffffull || out == NULL || cap < need) {
    free(val);
    free(locs);
    return total_words > 0xffffffffull ? 0 : need;
  }

  put32(out + 0, FLSO2_MAGIC);
  put32(out + 4, FLSO2_VERSION);
  put32(out + 8, tile_m);
  put32(out + 12, tile_k);
  put32(out + 16, FLSO2_GROUP);
  put32(out + 20, 0);
  put32(out + 24, (uint32_t)max_tile_words);
  put32(out + 28, 0);
  put64(out + 32, (uint64_t)M);
  put64(out + 40, (uint64_t)K);
  put64(out + 48, nnz);
  put64(out + 56, total_words);

  uint8_t* offs = out + FLSO2_HEADER_BYTES;
  uint8_t* nzw = offs + 4 * n_off;
  uint64_t pos = 0; /* in words */
  for (uint64_t t = 0; t < num_tiles; ++t) {
    uint64_t nz;
    put32(offs + 4 * t, (uint32_t)pos);
    const uint32_t n = tile_entries(W, K, t / tiles_k, t % tiles_k, tile_m, tile_k, val, locs, &nz);
    for (uint32_t g = 0; g < n / FLSO2_GROUP; ++g) {
      const uint16_t* v = val + 4 * g;
      const uint32_t* l = locs + 4 * g;
      put32(nzw + 4 * (pos + 0), (uint32_t)v[0] | ((uint32_t)v[1] << 16));
      put32(nzw + 4 * (pos + 1), (uint32_t)v[2] | ((uint32_t)v[3] << 16));
      put32(nzw + 4 * (pos + 2), l[0] | ((l[1] - l[0]) << 12) | ((l[2] - l[1]) << 18) | ((l[3] - l[2]) << 24));
      pos += 3;
    }
  }
  for (uint64_t t = num_tiles; t < n_off; ++t) put32(offs + 4 * t, (uint32_t)pos);
  free(val);
  free(locs);
  return need;
}

/* Worst-case blob size: every element stored (no bridges are needed then). */
size_t flso2_compress_bound(int64_t M, int64_t K, uint32_t tile_m, uint32_t tile_k) {
  if (!geometry2_ok(M, K, tile_m, tile_k)) return 0;
  const uint64_t num_tiles = ((uint64_t)M / tile_m) * ((uint64_t)K / tile_k);
  const uint64_t n_off = round_up64(num_tiles + 4, 16);
  const uint64_t per_tile = round_up64((uint64_t)tile_m * tile_k, FLSO2_GROUP) / FLSO2_GROUP * 12u;
  return (size_t)(FLSO2_HEADER_BYTES + 4 * n_off + num_tiles * per_tile);
}

/* Header fields -> out[12] (as flso_inspect).  0 if well formed and consistent with `bytes`. */
int flso2_inspect(const uint8_t* blob, size_t bytes, uint64_t* out) {
  if (bytes < FLSO2_HEADER_BYTES) return -1;
  for (int q = 0; q < 8; ++q) out[q] = get32(blob + 4 * q);
  for (int q = 0; q < 4; ++q) out[8 + q] = get64(blob + 32 + 8 * q);
  if (out[0] != FLSO2_MAGIC) return -2;
  if (out[1] != FLSO2_VERSION) return -3;
  if (out[4] != FLSO2_GROUP || !geometry2_ok((int64_t)out[8], (int64_t)out[9], (uint32_t)out[2], (uint32_t)out[3])) return -4;
  const uint64_t num_tiles = (out[8] / out[2]) * (out[9] / out[3]);
  const uint64_t n_off = round_up64(num_tiles + 4, 16);
  if (out[11] % 3 != 0 || bytes < FLSO2_HEADER_BYTES + 4 * n_off + 4 * out[11]) return -5;
  return 0;
}

/* blob -> dense M x K bit patterns.  Returns 0, or a negative code on a malformed blob. */
int flso2_decompress(const uint8_t* blob, size_t bytes, uint16_t* W, int64_t M, int64_t K) {
  uint64_t h[12];
  int rc = flso2_inspect(blob, bytes, h);
  if (rc != 0) return rc;
  if ((int64_t)h[8] != M || (int64_t)h[9] != K) return -6;
  const uint32_t tile_m = (uint32_t)h[2], tile_k = (uint32_t)h[3];
  const uint64_t tiles_k = (uint64_t)K / tile_k;
  const uint64_t num_tiles = ((uint64_t)M / tile_m) * tiles_k;
  const uint64_t n_off = round_up64(num_tiles + 4, 16);
  const uint8_t* offs = blob + FLSO2_HEADER_BYTES;
  const uint8_t* nzw = offs + 4 * n_off;
  const uint32_t elems = tile_m * tile_k;
  memset(W, 0, (size_t)M * (size_t)K * sizeof(uint16_t));
  for (uint64_t t = 0; t < num_tiles; ++t) {
    const uint64_t i = t / tiles_k, j = t % tiles_k;
    const uint32_t a = get32(offs + 4 * t), b = get32(offs + 4 * (t + 1));
    if (b < a || b > h[11] || a % 3 != 0 || b % 3 != 0) return -7;
    uint32_t behind = 0; /* one past the location of the entry before: locations ascend through the tile */
    for (uint32_t q = a; q < b; q += 3) {
      const uint32_t w0 = get32(nzw + 4 * (uint64_t)q), w1 = get32(nzw + 4 * (uint64_t)(q + 1)), w2 = get32(nzw + 4 * (uint64_t)(q + 2));
      const uint16_t v[4] = {(uint16_t)w0, (uint16_t)(w0 >> 16), (uint16_t)w1, (uint16_t)(w1 >> 16)};
      if (w2 >> 30) return -8;
      uint32_t loc = 0;
      for (int e = 0; e < 4; ++e) {
        if (e == 0) loc = w2 & 0xfffu;
        else loc += (w2 >> (6 + 6 * e)) & 0x3fu;
        if (loc < behind) return -12; /* entries ascend: a distance of 0 is not an entry */
        behind = loc + 1;
        if (v[e] == 0) continue; /* bridge or padding */
        if (loc >= elems) return -9;
        const uint32_t c = loc / (tile_m * 8u);
        const uint32_t x = (loc % (tile_m * 8u)) / 8u;
        const uint32_t y = c * 8u + loc % 8u;
        uint16_t* dst = &W[(i * tile_m + x) * (uint64_t)K + j * tile_k + y];
        if (*dst != 0) return -10; /* a location may be given once */
        *dst = v[e];
      }
    }
    if (behind > elems + 3u) return -11;
  }
  return 0;
}
