/*
 * libfls - Load-as-Sparse / Compute-as-Dense SpMM for AMD MI355X (gfx950).
 *
 * C ABI of the hot path of Flash-LLM (arxiv 2309.10285): C = W . X with W an fp16 weight
 * matrix [M, K] whose pruned entries are zero, kept in HBM in the Tiled-CSL compressed
 * format, and X a skinny fp16 activation matrix [K, N] (paper Sec. 2.2: C = A x B,
 * A = weights [M, K], B = feature map [K, N]).
 *
 * Conventions shared by every call
 *   - "dev" pointers are device (HBM) addresses owned by the caller; "host" pointers are host
 *     addresses.  The library never allocates or frees device memory.
 *   - W dense    : fp16, row-major M x K, leading dimension K      (Alg. 3: A + x*K + y)
 *   - X          : fp16, column-major K x N, leading dimension K   (== row-major [N][K])
 *   - C          : fp16, column-major M x N, leading dimension M   (== row-major [N][M])
 *   - products are exact, accumulation is fp32, C is rounded once to fp16 (nearest even)
 *   - M must be a multiple of FLS_TILE_M, K of FLS_TILE_K; 1 <= N <= FLS_MAX_N
 *   - device pointers must be 16-byte aligned
 *   - kernels are enqueued on `stream` and the call returns without waiting, except
 *     fls_compress, which waits for its own work (it is an offline step, Sec. 5), the first
 *     fls_spmm on a blob address (header read-back) and fls_check_workspace
 *   - every function returns FLS_OK (0) or a negative error code; arguments are checked on
 *     the host before anything is launched, so a failed call has launched nothing
 *   - one device per process is assumed: calls act on the current HIP device
 */
#ifndef FLS_H_
#define FLS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLS_TILE_M 128u /* rows of a Tiled-CSL tile                        (Sec. 4.3.1) */
#define FLS_TILE_K 32u  /* columns (K extent) of a Tiled-CSL tile */
#define FLS_PAD_WORDS 4u /* a tile's run is padded to a multiple of this many words */
#define FLS_MAX_N 8192 /* the skinny case is N <= 256; wider N runs as passes of 64 columns (Sec. 6.2, non-skinny shapes) */
#define FLS_FORMAT_VERSION 1u
#define FLS_FORMAT_VERSION_2 2u /* four entries share a word of locations, 3 bytes per entry: fls_compress_v2 */
#define FLS_HEADER_BYTES 64u

enum {
  FLS_OK = 0,
  FLS_EINVAL = -1,     /* null pointer, M/K not multiples of the tile, N out of range, bad policy */
  FLS_EALIGN = -2,     /* a device pointer is not 16-byte aligned */
  FLS_ECAPACITY = -3,  /* output buffer too small; stats->bytes_total holds the size needed */
  FLS_EFORMAT = -4,    /* blob header: bad magic / version / geometry, or M, K differ from the call */
  FLS_EWORKSPACE = -5, /* no workspace registered, or it is too small for this call */
  FLS_EHIP = -6,       /* a HIP call failed (the HIP error stays readable with hipGetLastError) */
  FLS_EHANDOVER = -7,  /* a kernel gave up waiting for another workgroup's partial sum: results of the calls
                          since the last check are not to be trusted (fls_check_workspace) */
  FLS_ESCRATCH = -8    /* fls_spmm_noalloc: the call needs more scratch than the library's static array holds */
};

/* opaque stream handle: pass a hipStream_t (NULL = the default stream) */
typedef void* fls_stream_t;

/* Word order inside a tile's run (Sec. 4.3.3).  Both orders decode to the same tile. */
enum {
  FLS_ORDER_LOCATION = 0, /* ascending in-tile location */
  FLS_ORDER_BANK = 1      /* ahead-of-time reordering by LDS bank (Alg. 3) */
};

typedef struct {
  uint32_t format_version, tile_m, tile_k, order_policy;
  uint64_t M, K, nnz, num_tiles, max_tile_words;
  uint64_t bytes_total;    /* the whole blob: what fls_spmm streams from HBM */
  uint64_t bytes_header;   /* 64 */
  uint64_t bytes_offsets;  /* TileOffsets incl. look-ahead guard entries */
  uint64_t bytes_nonzeros; /* NonZeros incl. padding words */
} fls_stats;

/*
 * Compressed blob ("Tiled-CSL", Sec. 4.3.1; word layout Sec. 4.3.2; tile walk Alg. 3), little endian:
 *   [0,64)   header: u32 magic "FLS1", u32 version, u32 tile_m, u32 tile_k, u32 pad_words,
 *            u32 order_policy, u32 max_tile_words, u32 0, u64 M, u64 K, u64 nnz, u64 total_words
 *   [64, 64 + 4*n_off)  TileOffsets: u32 word offset of each tile's run in NonZeros; tile id =
 *            band*(K/tile_k) + ktile (row bands outer); entry num_tiles = total_words, repeated
 *            up to n_off = round_up(num_tiles + 4, 16) entries
 *   then     NonZeros: u32 words = (fp16 bits << 16) | location, location =
 *            (y/8)*(tile_m*8) + x*8 + y%8 for row x, column y of the tile (the element's place in
 *            the on-chip [K-chunk][row][8] tile); every element whose bit pattern is not 0x0000 is
 *            stored; runs are padded with the word tile_m*tile_k (value +0, location one past the tile).
 */

/* Size in bytes of the largest blob an M x K matrix can produce (every element stored).
 * Errors: FLS_EINVAL. */
int fls_compress_bound(int64_t M, int64_t K, size_t* bytes_host);

/*
 * Dense masked W -> Tiled-CSL blob (the paper's offline weight reformatting step, Sec. 5, Alg. 3).
 *   W_dev        in : fp16 row-major M x K, pruned entries exactly +0 (0x0000)
 *   out_dev      out: blob; caller-owned, out_capacity bytes, 16-byte aligned
 *   order_policy in : FLS_ORDER_LOCATION (FLS_ORDER_BANK blobs are accepted by fls_spmm, but this
 *                     call does not produce them: FLS_EINVAL)
 *   stats_host   out: may be NULL; filled on FLS_OK; on FLS_ECAPACITY bytes_total holds a size that is enough
 *                     (the exact size once the tiles are counted, the worst-case bound if out_capacity
 *                     did not even hold header and TileOffsets)
 * The result is a pure function of (W bits, M, K, order_policy).  Waits for its own kernels.
 * Uses the start of out_dev as scratch, so out_capacity must cover header and TileOffsets even
 * for an all-zero matrix.  Errors: FLS_EINVAL, FLS_EALIGN, FLS_ECAPACITY, FLS_EHIP.
 */
int fls_compress(const void* W_dev, int64_t M, int64_t K, void* out_dev, size_t out_capacity,
                 int order_policy, fls_stats* stats_host, fls_stream_t stream);

/*
 * Format version 2: the same tiles, walk and stored elements, with the 16-bit locations of four entries
 * packed into one word - 3 bytes per nonzero instead of 4.  The paper's byte model leaves
 * the index bytes out (footnote under Eq. 2, Sec. 3.2.2) while its format pays 2 of them per kept
 * weight (Sec. 4.3.2); this is this build's own narrowing of that overhead.  Blob:
 *   header as above with magic "FLS2", version 2, pad_words 4 (entries per group), order_policy 0
 *   TileOffsets as above (u32 offsets in 32-bit words, all multiples of 3)
 *   NonZeros: groups of four entries in three words: word 0 = value0 | value1 << 16,
 *            word 1 = value2 | value3 << 16, word 2 = loc0 | dist1 << 12 | dist2 << 18 | dist3 << 24
 *            (loc0: the location of entry 0, 12 bits; distK: location of entry K minus location of
 *            entry K - 1, 6 bits; bits 30 and 31 are 0).  A group decodes by itself.
 *   The entries of a tile are the stored elements in ascending location; a bridge (value 0x0000)
 *   every 63 locations wherever the next stored element lies more than 63 locations behind the entry
 *   before it (behind location 0 for the first) - it names an empty location - whether or not the
 *   next entry starts a group; padding (value 0x0000, distance 1) up to a multiple of four entries -
 *   the empty locations behind the tile's last entry, at most three past the end of the tile.
 * fls_compress_v2 is fls_compress for this format (same arguments without the order policy, same
 * errors, same waiting); fls_compress_bound_v2 its capacity bound.  fls_inspect and fls_spmm take
 * blobs of either version (fls_spmm tells them apart by the header) and run the same passes on both.
 */
int fls_compress_bound_v2(int64_t M, int64_t K, size_t* bytes_host);
int fls_compress_v2(const void* W_dev, int64_t M, int64_t K, void* out_dev, size_t out_capacity,
                    fls_stats* stats_host, fls_stream_t stream);

/* Validates a 64-byte header copied to the host and derives the section sizes.
 * Errors: FLS_EINVAL (null), FLS_EFORMAT. */
int fls_inspect(const void* header_host, fls_stats* stats_host);

/*
 * Bytes of device workspace fls_spmm / fls_dense_gemm need for this shape: a 4 MiB control area
 * (per-workgroup flags of the split-K hand-over, an error word), the fp32 partial sums (4 MiB
 * for N <= 16, 64 MiB above: from 17 columns on a call may take the 64-column pass, which keeps
 * one partial result per band and K slice) and, for N > 32, K x N x 2 bytes for X repacked into
 * MFMA fragment order.  Returns 0 on invalid arguments.
 */
size_t fls_workspace_bytes(int64_t M, int64_t K, int64_t N);

/*
 * Registers a caller-owned workspace (16-byte aligned) and clears it on `stream`.  The
 * workspace must stay valid, and untouched by the caller, until replaced.  Nothing has to be
 * cleared between calls (every launch leaves the flags it raised lowered again), so one
 * registration serves any number of calls of any shape it is large enough for; calls that share
 * it must not overlap in time.  Errors: FLS_EINVAL, FLS_EALIGN, FLS_EHIP.
 */
int fls_set_workspace(void* ws_dev, size_t bytes, fls_stream_t stream);

/*
 * Waits for `stream` and reads the workspace's error word.  The split-K hand-over (Alg. 1 has
 * none: a thread block there walks the whole K) makes one workgroup wait for the partial sums of
 * others; that wait is bounded (about a second), and a kernel that gives up says so here instead
 * of hanging.  Returns FLS_OK, or FLS_EHANDOVER after clearing the control area again so that
 * later calls start clean; FLS_EWORKSPACE if none is registered; FLS_EHIP.
 */
int fls_check_workspace(fls_stream_t stream);

/*
 * C = W . X with W given as a Tiled-CSL blob (the SpMM of Alg. 1): streams the blob from HBM
 * (once per 64 columns for N > 32 - N = 8192 is 128 passes over W - else once), rebuilds each tile densely in LDS, multiplies
 * with MFMA, fp32 accumulation.  Partial sums of different workgroups are added in a fixed order;
 * inside a workgroup the waves' sums are added in the order they finish unless the workgroup's
 * tiles lie in one row band (then in wave order), so two runs may differ in the last bit of an
 * fp32 sum, never by more.  2*K*N and 2*M*N must stay below 2^31 (32-bit byte offsets into X and C).
 *   Wc_dev in : blob made by fls_compress (or byte-identical); its header must match M, K
 *   X_dev  in : fp16 column-major K x N;  C_dev out: fp16 column-major M x N (fully overwritten)
 * The first call on a given blob address reads its 64-byte header back (a copy on `stream`, waited for) to
 * validate it and to pick the kernel variant; later calls on that address do not.  Call
 * fls_forget when the memory at that address comes to hold a different blob by other means than
 * fls_compress (a copy, a freed buffer handed out again).  A remembered header that is out of date
 * but of the same M, K costs speed only (a variant sized for other tile lengths, down to a plain
 * slow path); the kernels take every tile's length from the blob itself.
 * Stream capture: a call on a blob address the library already knows enqueues kernels only (no
 * copies, no memsets, no host-side per-launch state in their arguments), so it may be recorded
 * into a HIP graph and replayed; make one ordinary call on that address and shape first.
 * Only the 64-byte header is validated; TileOffsets and NonZeros are the caller's responsibility (a blob
 * from fls_compress is right by construction).  As a guard for blobs that were stored and read back, the
 * passes of up to 32 columns take no offset to lie beyond the header's word count, so a truncated or
 * damaged TileOffsets section gives wrong results, not loads outside NonZeros; the 64-column pass
 * (N > 32, and calls of 17 - 32 columns on long bands of sparse tiles, where sharing X between
 * bands makes it the faster one) trusts TileOffsets.
 * Errors: FLS_EINVAL, FLS_EALIGN, FLS_EFORMAT, FLS_EWORKSPACE, FLS_EHIP.
 */
int fls_spmm(const void* Wc_dev, const void* X_dev, void* C_dev, int64_t M, int64_t K, int64_t N,
             fls_stream_t stream);

/*
 * fls_spmm without the library's memory of blob addresses: the blob's statistics come from the caller
 * (stats_host: as filled by fls_compress, fls_compress_v2 or fls_inspect for this blob; read during
 * the call only) instead of a header read-back, so the call copies nothing, waits for nothing on
 * any blob address - first sight included - and keeps no state about the blob.  Otherwise as fls_spmm
 * (same kernels, same registered workspace, any N up to FLS_MAX_N).  stats_host must describe the
 * blob at Wc_dev (same M, K, tile geometry): FLS_EFORMAT otherwise; a max_tile_words smaller than the
 * blob's costs speed only.  Errors: FLS_EINVAL, FLS_EALIGN, FLS_EFORMAT, FLS_EWORKSPACE, FLS_EHIP.
 */
int fls_spmm_stats(const void* Wc_dev, const fls_stats* stats_host, const void* X_dev, void* C_dev, int64_t M,
                   int64_t K, int64_t N, fls_stream_t stream);

/*
 * fls_spmm for callers that cannot allocate device memory or wait on a stream: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same results as fls_spmm, always
 * through the kernel of up to 32 columns per pass, but
 *   - the split-K scratch (hand-over flags, error word, fp32 partial sums) is a static device array
 *     inside the library, FLS_NOALLOC_SCRATCH_BYTES large, present on every GPU the library runs on
 *     from load time to the end of the process: no workspace has to be registered, and none is used;
 *   - the blob's statistics come from the caller (stats_host: as filled by fls_compress or
 *     fls_inspect for this blob; read during the call only) instead of a header read-back, so the
 *     call copies nothing, waits for nothing and keeps no state about the blob.
 * It calls no hipMalloc, hipFree or allocating library routine.  Limit: N <= FLS_NOALLOC_MAX_N (wider
 * calls need repacked X and larger partial sums than the array holds): FLS_ESCRATCH beyond it.
 * stats_host must describe the blob at Wc_dev (same M, K, tile geometry): FLS_EFORMAT otherwise; a
 * max_tile_words smaller than the blob's costs speed only, as with fls_spmm.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race, and must be serialised by the caller.  Each call clears the array's control
 * words first (a small kernel on `stream`).  fls_check_workspace also reports a hand-over that
 * gave up inside this call.
 * Errors: FLS_EINVAL, FLS_EALIGN, FLS_EFORMAT, FLS_ESCRATCH, FLS_EHIP.
 */
#define FLS_NOALLOC_MAX_N 32
#define FLS_NOALLOC_SCRATCH_BYTES (8192u + 512u * 2u * 2048u * 4u)
int fls_spmm_noalloc(const void* Wc_dev, const fls_stats* stats_host, const void* X_dev, void* C_dev, int64_t M,
                     int64_t K, int64_t N, fls_stream_t stream);

/* Drops what fls_spmm remembers about a blob address (NULL: about all of them). */
void fls_forget(const void* Wc_dev);

/*
 * C = W . X with W dense (fp16 row-major M x K): the dense baseline every sparse point is
 * paired with (the paper's own re-implemented dense GEMM, Sec. 6.2).  Same X, C, N rules and
 * workspace as fls_spmm.  Errors: FLS_EINVAL, FLS_EALIGN, FLS_EWORKSPACE, FLS_EHIP.
 */
int fls_dense_gemm(const void* W_dev, const void* X_dev, void* C_dev, int64_t M, int64_t K,
                   int64_t N, fls_stream_t stream);

/* Static description of an error code. */
const char* fls_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* FLS_H_ */
