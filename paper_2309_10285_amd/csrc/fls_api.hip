// C ABI of libfls (see include/fls.h): argument checks on the host, blob header bookkeeping,
// workspace registration, kernel launches.  No device memory is allocated here.
#include "../../include/fls.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <unordered_map>

#include "fls_launch.h"

namespace {

constexpr uint32_t kMagic = 0x31534C46u;   // "FLS1"
constexpr uint32_t kMagic2 = 0x32534C46u;  // "FLS2"

struct BlobInfo {
  uint64_t M, K;
  uint32_t max_tile_words;
  uint32_t version;
  uint64_t n_off;
};

std::mutex g_mu;
std::unordered_map<const void*, BlobInfo> g_blobs;  // blob address -> validated header
constexpr size_t kMaxRememberedBlobs = 4096;  // beyond this the map is emptied (entries only save a header read-back)
void* g_ws = nullptr;
size_t g_ws_bytes = 0;
int g_num_cus = 0;

// Scratch of fls_spmm_noalloc: the same areas a registered workspace has (control words, then the
// fp32 partial sums of up to 32 columns), in device memory that exists from the moment the library
// is loaded.  Host code never uses the array's name as an address: hipGetSymbolAddress gives the
// address on the current device (every device has its own copy), looked up once per device.
constexpr size_t kScratchControlBytes = 8192;  // 512 flags, the error word, spare
constexpr size_t kScratchPartsBytes = (size_t)fls::kMaxWorkgroups * 2 * 2048 * sizeof(float);  // 8 MiB
constexpr size_t kScratchBytes = kScratchControlBytes + kScratchPartsBytes;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};  // by device id; guarded by g_mu

// Address of `scratch` on the current device (nullptr after setting *err on failure).
unsigned char* scratch_on_current_device(int* err) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *err = FLS_EHIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      *err = FLS_EHIP;
      return nullptr;
    }
    g_scratch_ptr[dev] = (unsigned char*)ptr;
  }
  return g_scratch_ptr[dev];
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline uint64_t round_up(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

bool shape_ok(int64_t M, int64_t K) {
  if (M <= 0 || K <= 0) return false;
  if (M % FLS_TILE_M != 0 || K % FLS_TILE_K != 0) return false;
  // K: byte offsets inside a 128-row band (and inside X) are 32 bit
  if (M > 0x7fffffffll || K > (1ll << 23)) return false;
  // word offsets are 32 bit: the densest possible blob must stay below 2^32 words
  if ((uint64_t)M * (uint64_t)K >= (1ull << 32)) return false;
  return true;
}

uint64_t num_tiles(int64_t M, int64_t K) { return (uint64_t)(M / FLS_TILE_M) * (uint64_t)(K / FLS_TILE_K); }
uint64_t n_off_of(uint64_t tiles) { return round_up(tiles + 4, 16); }

int parse_header(const unsigned char* h, fls_stats* st, BlobInfo* info) {
  uint32_t u[8];
  uint64_t q[4];
  memcpy(u, h, 32);
  memcpy(q, h + 32, 32);
  const bool v2 = u[0] == kMagic2 && u[1] == FLS_FORMAT_VERSION_2;
  if (!v2 && (u[0] != kMagic || u[1] != FLS_FORMAT_VERSION)) return FLS_EFORMAT;
  if (u[2] != FLS_TILE_M || u[3] != FLS_TILE_K || u[4] != FLS_PAD_WORDS || u[5] > (v2 ? 0u : 1u)) return FLS_EFORMAT;
  if (q[0] > 0x7fffffffull || q[1] > 0x7fffffffull || !shape_ok((int64_t)q[0], (int64_t)q[1])) return FLS_EFORMAT;
  const uint64_t tiles = num_tiles((int64_t)q[0], (int64_t)q[1]);
  if (v2) {
    // three words per group of four entries; a tile has at most 4096 stored elements and no bridge then
    if (q[3] % 3 != 0 || q[3] > tiles * (uint64_t)(FLS_TILE_M * FLS_TILE_K / 4 * 3) || q[2] > q[3] / 3 * 4) return FLS_EFORMAT;
    if (u[6] % 3 != 0 || u[6] > FLS_TILE_M * FLS_TILE_K / 4 * 3) return FLS_EFORMAT;
  } else {
    if (q[2] > q[3] || q[3] > tiles * (uint64_t)(FLS_TILE_M * FLS_TILE_K) || q[3] % FLS_PAD_WORDS != 0) return FLS_EFORMAT;
    if (u[6] > FLS_TILE_M * FLS_TILE_K || u[6] % FLS_PAD_WORDS != 0) return FLS_EFORMAT;
  }
  if (st) {
    st->format_version = u[1];
    st->tile_m = u[2];
    st->tile_k = u[3];
    st->order_policy = u[5];
    st->M = q[0];
    st->K = q[1];
    st->nnz = q[2];
    st->num_tiles = tiles;
    st->max_tile_words = u[6];
    st->bytes_header = FLS_HEADER_BYTES;
    st->bytes_offsets = 4 * n_off_of(tiles);
    st->bytes_nonzeros = 4 * q[3];
    st->bytes_total = st->bytes_header + st->bytes_offsets + st->bytes_nonzeros;
  }
  if (info) {
    info->M = q[0];
    info->K = q[1];
    info->max_tile_words = u[6];
    info->version = u[1];
    info->n_off = n_off_of(tiles);
  }
  return FLS_OK;
}

int num_cus() {
  if (g_num_cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    g_num_cus = n;
  }
  return g_num_cus;
}

int check_mm_args(const void* W, const void* X, void* C, int64_t M, int64_t K, int64_t N) {
  if (!W || !X || !C) return FLS_EINVAL;
  if (!shape_ok(M, K) || N < 1 || N > FLS_MAX_N) return FLS_EINVAL;
  // X and C are addressed with 32-bit byte offsets through buffer descriptors
  if ((uint64_t)K * (uint64_t)N * 2u > 0x7fffffffull || (uint64_t)M * (uint64_t)N * 2u > 0x7fffffffull) return FLS_EINVAL;
  if (!aligned16(W) || !aligned16(X) || !aligned16(C)) return FLS_EALIGN;
  return FLS_OK;
}

// Workspace: a fixed 4 MiB control area (one u32 flag per workgroup and an error word; the rest
// is spare; cleared when the workspace is registered, and every launch leaves its flags cleared),
// then the split-K partial slots (fp32), then, for N > 32, X repacked into MFMA fragment order
// (K x N rounded up to 16 columns, fp16).  The control area has the same place for every shape, so
// partial sums of one call can never be read as flags by the next.
constexpr size_t kCounterAreaBytes = (size_t)4 << 20;

void workspace_layout(int64_t K, int64_t N, size_t* total, size_t* xpack_offset) {
  const size_t parts = fls::parts_floats((uint32_t)N) * sizeof(float);
  if (xpack_offset) *xpack_offset = kCounterAreaBytes + parts;
  *total = kCounterAreaBytes + parts + fls::xpack_bytes((uint32_t)K, (uint32_t)N);
}

}  // namespace

extern "C" {

int fls_compress_bound(int64_t M, int64_t K, size_t* bytes_host) {
  if (!bytes_host || !shape_ok(M, K)) return FLS_EINVAL;
  const uint64_t tiles = num_tiles(M, K);
  *bytes_host = (size_t)(FLS_HEADER_BYTES + 4 * n_off_of(tiles) + 4 * tiles * (uint64_t)(FLS_TILE_M * FLS_TILE_K));
  return FLS_OK;
}

int fls_inspect(const void* header_host, fls_stats* stats_host) {
  if (!header_host || !stats_host) return FLS_EINVAL;
  return parse_header((const unsigned char*)header_host, stats_host, nullptr);
}

static int compress_impl(const void* W_dev, int64_t M, int64_t K, void* out_dev, size_t out_capacity, int order_policy,
                         uint32_t version, fls_stats* stats_host, fls_stream_t stream) {
  if (!W_dev || !out_dev || !shape_ok(M, K)) return FLS_EINVAL;
  if (order_policy != FLS_ORDER_LOCATION) return FLS_EINVAL;  // FLS_ORDER_BANK: not built yet
  if (!aligned16(W_dev) || !aligned16(out_dev)) return FLS_EALIGN;
  const uint64_t tiles = num_tiles(M, K);
  const size_t index_bytes = (size_t)(FLS_HEADER_BYTES + 4 * n_off_of(tiles));
  if (out_capacity < index_bytes) {
    if (stats_host) {
      memset(stats_host, 0, sizeof(*stats_host));
      // the words are not counted yet: the worst case is a size that is certainly enough
      size_t bound = 0;
      if (version == FLS_FORMAT_VERSION_2) fls_compress_bound_v2(M, K, &bound);
      else fls_compress_bound(M, K, &bound);
      stats_host->bytes_total = bound;
    }
    return FLS_ECAPACITY;
  }
  hipStream_t s = (hipStream_t)stream;
  fls::CompressLaunch a;
  a.W = (const uint16_t*)W_dev;
  a.out = (unsigned char*)out_dev;
  a.M = (uint32_t)M;
  a.K = (uint32_t)K;
  a.policy = (uint32_t)order_policy;
  a.version = version;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    g_blobs.erase(out_dev);
  }
  if (fls::launch_compress_index(a, s) != hipSuccess) return FLS_EHIP;
  unsigned char hdr[FLS_HEADER_BYTES];
  if (hipMemcpyAsync(hdr, out_dev, FLS_HEADER_BYTES, hipMemcpyDeviceToHost, s) != hipSuccess) return FLS_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return FLS_EHIP;
  fls_stats st;
  BlobInfo info;
  if (parse_header(hdr, &st, &info) != FLS_OK) return FLS_EHIP;  // our own kernels wrote it
  if (st.bytes_total > out_capacity) {
    if (stats_host) *stats_host = st;
    return FLS_ECAPACITY;
  }
  if (fls::launch_compress_emit(a, s) != hipSuccess) return FLS_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return FLS_EHIP;
  if (stats_host) *stats_host = st;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_blobs.size() >= kMaxRememberedBlobs) g_blobs.clear();
    g_blobs[out_dev] = info;
  }
  return FLS_OK;
}

int fls_compress(const void* W_dev, int64_t M, int64_t K, void* out_dev, size_t out_capacity, int order_policy,
                 fls_stats* stats_host, fls_stream_t stream) {
  return compress_impl(W_dev, M, K, out_dev, out_capacity, order_policy, FLS_FORMAT_VERSION, stats_host, stream);
}

int fls_compress_bound_v2(int64_t M, int64_t K, size_t* bytes_host) {
  if (!bytes_host || !shape_ok(M, K)) return FLS_EINVAL;
  const uint64_t tiles = num_tiles(M, K);
  *bytes_host = (size_t)(FLS_HEADER_BYTES + 4 * n_off_of(tiles) + 3 * tiles * (uint64_t)(FLS_TILE_M * FLS_TILE_K));
  return FLS_OK;
}

int fls_compress_v2(const void* W_dev, int64_t M, int64_t K, void* out_dev, size_t out_capacity, fls_stats* stats_host,
                    fls_stream_t stream) {
  return compress_impl(W_dev, M, K, out_dev, out_capacity, FLS_ORDER_LOCATION, FLS_FORMAT_VERSION_2, stats_host, stream);
}

size_t fls_workspace_bytes(int64_t M, int64_t K, int64_t N) {
  if (!shape_ok(M, K) || N < 1 || N > FLS_MAX_N) return 0;
  size_t total;
  workspace_layout(K, N, &total, nullptr);
  return total;
}

int fls_set_workspace(void* ws_dev, size_t bytes, fls_stream_t stream) {
  if (!ws_dev && bytes != 0) return FLS_EINVAL;
  if (!aligned16(ws_dev) || bytes % 16 != 0) return FLS_EALIGN;
  if (bytes && fls::launch_fill_zero(ws_dev, bytes, (hipStream_t)stream) != hipSuccess) return FLS_EHIP;
  std::lock_guard<std::mutex> lk(g_mu);
  g_ws = ws_dev;
  g_ws_bytes = bytes;
  return FLS_OK;
}

int fls_check_workspace(fls_stream_t stream) {
  void* ws;
  unsigned char* st = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) st = g_scratch_ptr[dev];
    if (!st && (!g_ws || g_ws_bytes < kCounterAreaBytes)) return FLS_EWORKSPACE;
    ws = g_ws && g_ws_bytes >= kCounterAreaBytes ? g_ws : nullptr;
  }
  hipStream_t s = (hipStream_t)stream;
  uint32_t word = 0;
  if (st) {  // the scratch of fls_spmm_noalloc, if this device has used it
    if (hipMemcpyAsync(&word, (const uint32_t*)st + fls::kMaxWorkgroups, sizeof(word), hipMemcpyDeviceToHost, s) != hipSuccess)
      return FLS_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return FLS_EHIP;
    if (word != 0) {
      if (fls::launch_fill_zero(st, kScratchControlBytes, s) != hipSuccess) return FLS_EHIP;
      return FLS_EHANDOVER;
    }
    if (!ws) return FLS_OK;
  }
  if (hipMemcpyAsync(&word, (const uint32_t*)ws + fls::kMaxWorkgroups, sizeof(word), hipMemcpyDeviceToHost, s) != hipSuccess)
    return FLS_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return FLS_EHIP;
  if (word == 0) return FLS_OK;
  // flags of the launch that gave up may have stayed up
  if (fls::launch_fill_zero(ws, kCounterAreaBytes, s) != hipSuccess) return FLS_EHIP;
  return FLS_EHANDOVER;
}

void fls_forget(const void* Wc_dev) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (Wc_dev) g_blobs.erase(Wc_dev);
  else g_blobs.clear();
}

int fls_spmm(const void* Wc_dev, const void* X_dev, void* C_dev, int64_t M, int64_t K, int64_t N,
             fls_stream_t stream) {
  int rc = check_mm_args(Wc_dev, X_dev, C_dev, M, K, N);
  if (rc != FLS_OK) return rc;
  size_t need, xpack_offset;
  workspace_layout(K, N, &need, &xpack_offset);
  void* ws;
  BlobInfo info;
  bool known;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_ws || g_ws_bytes < need) return FLS_EWORKSPACE;
    ws = g_ws;
    auto it = g_blobs.find(Wc_dev);
    known = it != g_blobs.end();
    if (known) info = it->second;
  }
  if (!known || info.M != (uint64_t)M || info.K != (uint64_t)K) {
    // unknown address, or the memory now holds another blob than the one remembered: read the header
    // on the call's stream: the blob may have been put there by work still queued on it
    unsigned char hdr[FLS_HEADER_BYTES];
    if (hipMemcpyAsync(hdr, Wc_dev, FLS_HEADER_BYTES, hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess) return FLS_EHIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return FLS_EHIP;
    rc = parse_header(hdr, nullptr, &info);
    std::lock_guard<std::mutex> lk(g_mu);
    if (rc != FLS_OK) {
      g_blobs.erase(Wc_dev);
      return rc;
    }
    if (g_blobs.size() >= kMaxRememberedBlobs) g_blobs.clear();
    g_blobs[Wc_dev] = info;
  }
  if (info.M != (uint64_t)M || info.K != (uint64_t)K) return FLS_EFORMAT;
  const int cus = num_cus();
  if (cus <= 0) return FLS_EHIP;
  fls::SpmmLaunch a;
  a.offs = (const uint32_t*)((const unsigned char*)Wc_dev + FLS_HEADER_BYTES);
  a.words = a.offs + info.n_off;
  a.X = (const _Float16*)X_dev;
  a.C = (_Float16*)C_dev;
  a.flags = (uint32_t*)ws;
  a.parts = (float*)((unsigned char*)ws + kCounterAreaBytes);
  a.xpack = (_Float16*)((unsigned char*)ws + xpack_offset);
  a.M = (uint32_t)M;
  a.K = (uint32_t)K;
  a.N = (uint32_t)N;
  a.max_tile_words = info.max_tile_words;
  a.version = info.version;
  a.num_cus = cus;
  a.wide32 = true;
  return fls::launch_spmm(a, (hipStream_t)stream) == hipSuccess ? FLS_OK : FLS_EHIP;
}

// Do the caller's statistics describe a blob of this shape?  (They stand in for the header read-back of fls_spmm.)
static bool stats_match(const fls_stats* st, int64_t M, int64_t K) {
  return (st->format_version == FLS_FORMAT_VERSION || st->format_version == FLS_FORMAT_VERSION_2) && st->tile_m == FLS_TILE_M &&
         st->tile_k == FLS_TILE_K && st->M == (uint64_t)M && st->K == (uint64_t)K && st->num_tiles == num_tiles(M, K) &&
         st->max_tile_words <= FLS_TILE_M * FLS_TILE_K && st->bytes_offsets == 4 * n_off_of(num_tiles(M, K));
}

int fls_spmm_stats(const void* Wc_dev, const fls_stats* stats_host, const void* X_dev, void* C_dev, int64_t M, int64_t K,
                   int64_t N, fls_stream_t stream) {
  if (!stats_host) return FLS_EINVAL;
  int rc = check_mm_args(Wc_dev, X_dev, C_dev, M, K, N);
  if (rc != FLS_OK) return rc;
  if (!stats_match(stats_host, M, K)) return FLS_EFORMAT;
  size_t need, xpack_offset;
  workspace_layout(K, N, &need, &xpack_offset);
  void* ws;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_ws || g_ws_bytes < need) return FLS_EWORKSPACE;
    ws = g_ws;
  }
  const int cus = num_cus();
  if (cus <= 0) return FLS_EHIP;
  fls::SpmmLaunch a;
  a.offs = (const uint32_t*)((const unsigned char*)Wc_dev + FLS_HEADER_BYTES);
  a.words = a.offs + n_off_of(num_tiles(M, K));
  a.X = (const _Float16*)X_dev;
  a.C = (_Float16*)C_dev;
  a.flags = (uint32_t*)ws;
  a.parts = (float*)((unsigned char*)ws + kCounterAreaBytes);
  a.xpack = (_Float16*)((unsigned char*)ws + xpack_offset);
  a.M = (uint32_t)M;
  a.K = (uint32_t)K;
  a.N = (uint32_t)N;
  a.max_tile_words = (uint32_t)stats_host->max_tile_words;
  a.version = stats_host->format_version;
  a.num_cus = cus;
  a.wide32 = true;
  return fls::launch_spmm(a, (hipStream_t)stream) == hipSuccess ? FLS_OK : FLS_EHIP;
}

int fls_spmm_noalloc(const void* Wc_dev, const fls_stats* stats_host, const void* X_dev, void* C_dev, int64_t M,
                     int64_t K, int64_t N, fls_stream_t stream) {
  if (!stats_host) return FLS_EINVAL;
  int rc = check_mm_args(Wc_dev, X_dev, C_dev, M, K, N);
  if (rc != FLS_OK) return rc;
  if (N > FLS_NOALLOC_MAX_N) return FLS_ESCRATCH;  // partial sums of wider calls do not fit the static array
  // the caller's stats stand in for the header read-back of fls_spmm: nothing is copied, nothing is waited for
  if (!stats_match(stats_host, M, K)) return FLS_EFORMAT;
  unsigned char* ptr = scratch_on_current_device(&rc);
  if (!ptr) return rc;
  const int cus = num_cus();
  if (cus <= 0) return FLS_EHIP;
  hipStream_t s = (hipStream_t)stream;
  // the array keeps what the last call left: flags and error word start every call at zero (a fill
  // kernel, not a memset node, so that the call can be recorded into a graph)
  if (fls::launch_fill_zero(ptr, kScratchControlBytes, s) != hipSuccess) return FLS_EHIP;
  fls::SpmmLaunch a;
  a.offs = (const uint32_t*)((const unsigned char*)Wc_dev + FLS_HEADER_BYTES);
  a.words = a.offs + n_off_of(num_tiles(M, K));
  a.X = (const _Float16*)X_dev;
  a.C = (_Float16*)C_dev;
  a.flags = (uint32_t*)ptr;
  a.parts = (float*)(ptr + kScratchControlBytes);
  a.xpack = nullptr;  // only calls of more than 32 columns repack X
  a.M = (uint32_t)M;
  a.K = (uint32_t)K;
  a.N = (uint32_t)N;
  a.max_tile_words = (uint32_t)stats_host->max_tile_words;
  a.version = stats_host->format_version;
  a.num_cus = cus;
  a.wide32 = false;  // the static array has the narrow kernel's partial sums only
  return fls::launch_spmm(a, s) == hipSuccess ? FLS_OK : FLS_EHIP;
}

int fls_dense_gemm(const void* W_dev, const void* X_dev, void* C_dev, int64_t M, int64_t K, int64_t N,
                   fls_stream_t stream) {
  int rc = check_mm_args(W_dev, X_dev, C_dev, M, K, N);
  if (rc != FLS_OK) return rc;
  size_t need, xpack_offset;
  workspace_layout(K, N, &need, &xpack_offset);
  void* ws;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_ws || g_ws_bytes < need) return FLS_EWORKSPACE;
    ws = g_ws;
  }
  const int cus = num_cus();
  if (cus <= 0) return FLS_EHIP;
  fls::DenseLaunch a;
  a.W = (const _Float16*)W_dev;
  a.X = (const _Float16*)X_dev;
  a.C = (_Float16*)C_dev;
  a.flags = (uint32_t*)ws;
  a.parts = (float*)((unsigned char*)ws + kCounterAreaBytes);
  a.xpack = (_Float16*)((unsigned char*)ws + xpack_offset);
  a.M = (uint32_t)M;
  a.K = (uint32_t)K;
  a.N = (uint32_t)N;
  a.num_cus = cus;
  return fls::launch_dense(a, (hipStream_t)stream) == hipSuccess ? FLS_OK : FLS_EHIP;
}

const char* fls_strerror(int code) {
  switch (code) {
    case FLS_OK: return "ok";
    case FLS_EINVAL: return "invalid argument (null pointer, shape not a multiple of the tile, N out of range, or policy)";
    case FLS_EALIGN: return "device pointer or size not 16-byte aligned";
    case FLS_ECAPACITY: return "output buffer too small";
    case FLS_EFORMAT: return "compressed blob header is malformed or does not match M, K";
    case FLS_EWORKSPACE: return "workspace missing or too small (see fls_workspace_bytes / fls_set_workspace)";
    case FLS_EHIP: return "a HIP runtime call failed";
    case FLS_ESCRATCH: return "the call needs more scratch than the library's static array holds (fls_spmm_noalloc: N <= 32)";
    case FLS_EHANDOVER: return "a kernel gave up waiting for another workgroup's partial sum; results since the last check are not to be trusted";
    default: return "unknown error code";
  }
}

}  // extern "C"
