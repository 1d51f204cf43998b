// Host-side internals of libcoop: error helpers, the launch/profiling hook, shared prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "coop.h"

namespace coop {

// Kernel ids for the profiling table (coop_profile_*).
enum KernelId {
  K_FILL = 0,        // memory fill (table clear, control words)
  K_LABOR_COUNT,     // LABOR-0 count pass
  K_LABOR_FILL,      // LABOR-0 fill pass (copy of the staged rows)
  K_LABOR_OVERFLOW,  // LABOR-0 second scan of overflowed rows
  K_LABOR_EXACT,     // LABOR-0, c > 0: exact blend of the candidates
  K_SEGMENTS,        // LABOR-0 per-destination list records and keep thresholds
  K_ENUM_LIST,       // LABOR-0 from the other side: vertices with a small variate, listed through the inverse mixer
  K_ENUM_WALK,       // LABOR-0 from the other side: their lists walked, kept edges of the long destinations found
  K_NS_COUNT,        // NS count pass (min(k, d))
  K_NS_FILL,         // NS selection + fill pass
  K_NS_SELECT,       // NS, c > 0: exact blend of the candidates + selection
  K_RW_WALK,         // random walks + visit tally + top-k
  K_RW_FILL,         // random-walk fill pass
  K_SCAN_LOCAL,      // scan: per-tile exclusive scan + tile sums
  K_SCAN_OFFSET,     // scan: add the sum of the preceding tiles
  K_UNIQ_INSERT,     // hash table insert (atomic CAS / min)
  K_UNIQ_FLAG,       // first-occurrence lookup
  K_UNIQ_RELABEL,    // new-id compaction + col_local
  K_PART_COUNT,      // dedup by partition: bucket sizes per block
  K_PART_SCATTER,    // dedup by partition: (key, position) pairs to their buckets
  K_PART_FIRST,      // dedup by partition: first positions through a table in LDS, one bucket per block
  K_COPY_IDS,        // seed copy / src_ids prefix copy
  K_GATHER,          // feature row gather
  K_GATHER_MEAN,     // neighbour mean fused with the feature load
  K_OWNER_COUNT,     // ids by owner: per-wave counts
  K_OWNER_SCATTER,   // ids by owner: stable placement
  K_VALIDATE,        // CSR validation
  K_CACHE_LOOKUP,
  K_CACHE_SELECT,    // one pass of the radix select of the eviction threshold
  K_CACHE_EVICT,
  K_CACHE_UPDATE,
  K_CACHE_GATHER,
  K_COUNT_
};

void prof_begin(int id, hipStream_t s);
void prof_end(int id, hipStream_t s);

#define COOP_HIP_TRY(expr)                         \
  do {                                             \
    hipError_t e__ = (expr);                       \
    if (e__ != hipSuccess) return COOP_E_HIP;      \
  } while (0)

// Launches `kernel` on `stream`, bracketed by profiling events when profiling is on.
#define COOP_LAUNCH(id, kernel, grid, block, shmem, stream, ...)                  \
  do {                                                                            \
    ::coop::prof_begin((id), (stream));                                           \
    hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);          \
    ::coop::prof_end((id), (stream));                                             \
  } while (0)

// Control block in device memory, mirrored to pinned host memory at every size read-back.
struct Ctl {
  int64_t total_edges;   // m_l
  int64_t total_new;     // |S^{l+1}| - |S^l|
  int32_t err_range;     // a seed / id out of range
  int32_t err_dup;       // a duplicate in the seed list
  int32_t err_capacity;  // NS candidate buffer could not be sized
  int32_t n_overflow;    // LABOR-0 destinations whose staging row overflowed (this layer and earlier)
  int32_t cand_overflow; // blended LABOR-0: the candidate buffer of the exact stage was too small (the pass is redone)
  int32_t uniq_overflow; // dedup by partition: a bucket held more distinct vertices than its table (redone with the table in HBM)
  uint32_t scan_done;    // one-kernel scans: tiles finished so far (the block that finishes last puts it back to zero)
  int32_t pad[1];
};

// Landing pad of the control block in mapped pinned host memory (see read_ctl).
struct HostCtl {
  Ctl ctl;               // must stay the first member
  uint64_t ticket;       // written by the device after ctl
  uint64_t next_ticket;  // host side only
};

// A size read-back in flight: the device stores the control block and then `ticket` into the landing pad.
struct Publish {
  const Ctl* d_ctl = nullptr;
  HostCtl* h = nullptr;
  uint64_t ticket = 0;
};

// Device-wide exclusive scans; `tmp` needs scan_tmp_bytes(n) bytes.  out has n + 1 entries, out[n] = total;
// the total also goes to *total_out (device) when that is not null.  With `pub`, the thread that stores the total then
// publishes the control block (total_out normally points into it), which saves the read-back a kernel of its own.
size_t scan_tmp_bytes(int64_t n);
void scan_i32_to_i64(const int32_t* in, int64_t n, int64_t* out, int64_t* total_out, void* tmp, hipStream_t s,
                     const Publish* pub = nullptr);
// the same over an input that lies in up to four pieces: element i is ptr[p][i - start[p]] for the last p with start[p] <= i
struct ChunkedI32 {
  const int32_t* ptr[4];
  int64_t start[4];
  int n_chunks;
};
void scan_chunks_to_i64(const ChunkedI32& in, int64_t n, int64_t* out, int64_t* total_out, void* tmp, hipStream_t s,
                        const Publish* pub = nullptr);
// exclusive scan of n uint32 (sum below 2^32); out has n + 1 entries, the last one the total
void scan_u32_to_u32(const uint32_t* in, int64_t n, uint32_t* out, void* tmp, hipStream_t s);
// (n_bits_dev, device, optional: only bits [0, *n_bits_dev) count; n_words is then an upper bound known to the host)
void scan_popc_to_u32(const uint64_t* bits, int64_t n_words, uint32_t* out, int64_t* total_out, void* tmp, hipStream_t s,
                      const Publish* pub = nullptr, const int64_t* n_bits_dev = nullptr);

// One-kernel exclusive scans for the library's own consumers.  Every block scans its tile and leaves the tile's sum; the
// block that finishes last (a counter in the call's control block tells it) scans the tile sums.  The result stays in two
// parts, the position inside the tile and the sum of the tiles in front, and a consumer adds them when it reads an
// element: the second kernel of the two-kernel scan, which only did that addition, is gone.  No block waits for another.
constexpr int kScanTileLog2 = 11;  // elements per tile (2048)
template <typename T>
struct TiledScan {
  const T* local;        // [n + 1] exclusive scan inside each tile; local[n] = the total
  const T* tile_prefix;  // [tiles] sum of the tiles in front, or null when `local` is already the whole scan (short inputs)
  int64_t n;
#ifdef __HIPCC__
  __device__ __forceinline__ T at(int64_t i) const {
    const T v = local[i];
    return (tile_prefix != nullptr && i < n) ? (T)(v + tile_prefix[i >> kScanTileLog2]) : v;
  }
#endif
};
// (`done` points at a zeroed uint32 that no other scan in flight uses; it is zero again when the scan has run.)
TiledScan<uint32_t> scan_u32_tiled(const uint32_t* in, int64_t n, uint32_t* out, void* tmp, uint32_t* done, hipStream_t s);
TiledScan<uint32_t> scan_popc_tiled(const uint64_t* bits, int64_t n_words, uint32_t* out, int64_t* total_out, void* tmp, uint32_t* done,
                                    hipStream_t s, const Publish* pub = nullptr, const int64_t* n_bits_dev = nullptr);

void fill_u64(uint64_t* p, int64_t n, uint64_t v, hipStream_t s);

// The current device's sticky "an id was out of range" word (device memory; read and cleared by coop_gather_status).
int32_t* bad_flag();

// Per-call scratch allocator wrapper: 256-byte rounding, NULL check.
struct Alloc {
  coop_alloc_fn fn;
  void* ctx;
  bool failed = false;
  template <typename T>
  T* get(int64_t count, int tag) {
    size_t bytes = (size_t)(count > 0 ? count : 1) * sizeof(T);
    bytes = (bytes + 255) & ~(size_t)255;
    void* p = fn(ctx, bytes, tag);
    if (!p) failed = true;
    return (T*)p;
  }
};

// Size read-back: read_ctl = begin_publish + a one-thread publishing kernel + wait_ctl.  A caller whose last kernel
// is a scan hands the Publish to the scan instead of launching that kernel.  wait_ctl returns the error the control
// block reports (range, duplicate, capacity), COOP_E_HIP, or COOP_OK.
Publish begin_publish(Ctl* d_ctl, Ctl* h_ctl);
int launch_publish(const Publish& pub, hipStream_t s);
int wait_ctl(const Publish& pub, Ctl* h_ctl, hipStream_t s);
int read_ctl(Ctl* d_ctl, Ctl* h_ctl, hipStream_t s);

// Dedup + relabel of one layer (Eq. 2), in two halves around the size read-back.
//   front: finds every edge's first occurrence in [dst ; col_global] and counts the new vertices.  `m` is the number of
//          edges, or, when m_dev is given, an upper bound of it known to the host (the exact number is then *m_dev, on
//          the device, and comes back in the control block's total_edges together with everything else: one read-back
//          serves the sampler and the dedup).
//   back:  writes src_ids and col_local.
extern int g_unique_mode;  // COOP_TUNE_UNIQUE
struct UniqueWork {
  uint32_t* first = nullptr;
  uint64_t* bits = nullptr;
  uint32_t* word_rank = nullptr;
  TiledScan<uint32_t> rank{nullptr, nullptr, 0};  // scanned bit counts of the words of `bits` (over word_rank)
  void* scan_tmp = nullptr;
  int64_t n_buckets = 0;
  bool by_partition = false;
  Publish pub{};
  int64_t n_new = 0;
};
// launch: every kernel of the front half, ending with the scan that sends the sizes to the host; does not wait.
int unique_front_launch(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, UniqueWork* w,
                        Alloc& alloc, Ctl* d_ctl, Ctl* h_ctl, hipStream_t s);
// finish: waits for the sizes (h_ctl then holds total_edges, total_new and the flags; w->n_new is set).  If the dedup
// had to be run again (*redone), a relabelling launched in between has to be launched again.
int unique_front_finish(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, UniqueWork* w,
                        Alloc& alloc, Ctl* d_ctl, Ctl* h_ctl, hipStream_t s, bool* redone);
// back: writes src_ids (S^l, then the new vertices) and col_local[m]; src must have room for n_dst + (number of new
// vertices) entries.  May be launched between launch and finish with room for n_dst + m entries.
int unique_back(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, const UniqueWork& w,
                int32_t* col_local, int32_t* src, hipStream_t s);

}  // namespace coop

struct coop_graph {
  const int64_t* indptr;
  const int32_t* indices;
  int64_t n_vertices, n_edges;
  bool symmetric;     // COOP_SYMMETRIC: sorted lists, every edge stored both ways
  uint32_t* rev_pos;  // then: for the edge t -> s at position e of indices, the position of s in t's list (owned, device)
  int64_t long_mass;  // then: entries in lists longer than kLongListDegree
  bool own_rev;       // rev_pos was allocated by the library (hipMalloc) and is released by coop_graph_free
  bool have_census = false;  // the graph was looked at when it was registered (COOP_VALIDATE or COOP_SYMMETRIC); then:
  int64_t census[32] = {};   // census[k] = vertices whose list has at least 2^k and fewer than 2^(k+1) entries
  // at most this many vertices have a list longer than `len` entries (len >= 1); n_vertices if the graph was not looked at
  int64_t lists_longer_than(uint32_t len) const {
    if (!have_census) return n_vertices;
    int k = 0;
    while (k < 31 && (2u << k) <= len) ++k;  // 2^k <= len < 2^(k+1): the counters from k on cover every list longer than len
    int64_t n = 0;
    for (; k < 32; ++k) n += census[k];
    return n;
  }
};
constexpr int64_t kLongListDegree = 8192;  // default of COOP_TUNE_ENUM_DEGREE
