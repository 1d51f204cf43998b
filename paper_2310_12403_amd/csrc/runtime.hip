// libcoop runtime pieces: error names, arena allocator, profiling table, graph handle, fill and scan kernels.
#include <mutex>
#include <new>
#include <vector>

#include "coop_internal.h"
#include "device_utils.h"

namespace coop {

// ---- profiling ------------------------------------------------------------------------------------------------
namespace {
struct Pending { int id; hipEvent_t a, b; };
struct Prof {
  std::mutex mu;
  bool on = false;
  int only = -1;  // when >= 0, the one kernel id that is timed
  double ms[K_COUNT_] = {};
  int64_t launches[K_COUNT_] = {};
  std::vector<Pending> pending;
  std::vector<hipEvent_t> pool;
  hipEvent_t open[K_COUNT_] = {};
} g_prof;

const char* const kKernelNames[K_COUNT_] = {
    "fill", "labor_scan", "labor_fill", "labor_fill_overflow", "labor_exact", "segments", "enum_list", "enum_walk", "ns_count", "ns_fill", "ns_select", "rw_walk", "rw_fill", "scan_local", "scan_offset",
    "unique_insert", "unique_flag", "unique_relabel", "unique_part_count", "unique_part_scatter", "unique_part_first", "copy_ids", "gather", "gather_mean", "owner_count", "owner_scatter", "validate_csr",
    "cache_lookup", "cache_select", "cache_evict", "cache_miss_rows", "cache_hit_rows"};

hipEvent_t take_event() {
  if (!g_prof.pool.empty()) { hipEvent_t e = g_prof.pool.back(); g_prof.pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// folds finished event pairs into the table; caller holds the lock
void collect_locked() {
  for (auto& p : g_prof.pending) {
    float ms = 0.f;
    if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
      g_prof.ms[p.id] += ms;
      g_prof.launches[p.id] += 1;
    }
    g_prof.pool.push_back(p.a);
    g_prof.pool.push_back(p.b);
  }
  g_prof.pending.clear();
}
}  // namespace

void prof_begin(int id, hipStream_t s) {
  if (!g_prof.on || (g_prof.only >= 0 && g_prof.only != id)) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  hipEvent_t a = take_event();
  if (!a) return;
  (void)hipEventRecord(a, s);
  g_prof.open[id] = a;
}

void prof_end(int id, hipStream_t s) {
  if (!g_prof.on || (g_prof.only >= 0 && g_prof.only != id)) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  hipEvent_t a = g_prof.open[id];
  if (!a) return;
  g_prof.open[id] = nullptr;
  hipEvent_t b = take_event();
  if (!b) { g_prof.pool.push_back(a); return; }
  (void)hipEventRecord(b, s);
  g_prof.pending.push_back({id, a, b});
  if (g_prof.pending.size() >= 4096) collect_locked();
}

// ---- fill -----------------------------------------------------------------------------------------------------
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(kBlock) void k_fill_u64(uint64_t* __restrict__ p, int64_t n, uint64_t v) {
  // 16-byte stores over the even part when the base allows it, single words for the rest
  const bool wide = ((uintptr_t)p & 15) == 0;
  const int64_t n2 = wide ? n / 2 : 0;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  const u64x2 vv = {v, v};
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n2; i += stride) reinterpret_cast<u64x2*>(p)[i] = vv;
  for (int64_t i = 2 * n2 + (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) p[i] = v;
}

void fill_u64(uint64_t* p, int64_t n, uint64_t v, hipStream_t s) {
  if (n <= 0) return;
  int64_t blocks = (n / 2 + kBlock - 1) / kBlock;
  if (blocks > 256 * 64) blocks = 256 * 64;
  if (blocks < 1) blocks = 1;
  COOP_LAUNCH(K_FILL, k_fill_u64, dim3((unsigned)blocks), dim3(kBlock), 0, s, p, n, v);
}

// ---- device-wide exclusive scan -------------------------------------------------------------------------------
// Two kernels, no inter-block waiting: (1) every block scans its own tile of kTile consecutive elements and records
// the tile's sum; (2) every block adds up the sums of the tiles in front of it (a few thousand words at most, read
// from L2) and shifts its tile by that offset; the last block also publishes the grand total.
constexpr int kItems = 8;
constexpr int kTile = kBlock * kItems;  // 2048
static_assert(kTile == (1 << kScanTileLog2), "TiledScan::at() finds an element's tile by a shift");

// inclusive block scan of one int64 per thread; returns the thread's inclusive prefix, *total = block sum
__device__ __forceinline__ int64_t block_incl_scan(int64_t v, int64_t* total, int64_t* lds /* [kWavesPerBlock] */) {
  const int lane = lane_id(), w = wave_in_block();
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int64_t o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  if (lane == kWave - 1) lds[w] = v;
  __syncthreads();
  int64_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kWavesPerBlock; ++i) {
    const int64_t x = lds[i];
    if (i < w) base += x;
    tot += x;
  }
  __syncthreads();
  *total = tot;
  return v + base;
}

// what a one-thread publishing kernel would do, done by the thread that has just stored the scan's total
__device__ __forceinline__ void publish_ctl(const Publish& pub) {
  if (pub.h == nullptr) return;
  pub.h->ctl = *pub.d_ctl;
  __threadfence_system();
  __hip_atomic_store(&pub.h->ticket, pub.ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

struct LoadI32 {
  const int32_t* in;
  __device__ __forceinline__ int64_t operator()(int64_t i) const { return in[i]; }
};
struct LoadChunks {
  ChunkedI32 c;
  __device__ __forceinline__ int64_t operator()(int64_t i) const {
    int p = 0;
#pragma unroll
    for (int q = 1; q < 4; ++q)
      if (q < c.n_chunks && i >= c.start[q]) p = q;
    return c.ptr[p][i - c.start[p]];
  }
};
struct LoadU32 {
  const uint32_t* in;
  __device__ __forceinline__ int64_t operator()(int64_t i) const { return in[i]; }
};
struct LoadPopc {  // element i = number of set bits of word i
  const uint64_t* bits;
  const int64_t* n_bits;  // when not null: only the words that hold bits [0, *n_bits) count (a size that the host does not know yet)
  __device__ __forceinline__ int64_t operator()(int64_t i) const {
    if (n_bits != nullptr && i >= ((*n_bits + 63) >> 6)) return 0;
    return __popcll(bits[i]);
  }
};

template <typename Load, typename Out>
__global__ __launch_bounds__(kBlock) void k_scan_local(Load load, int64_t n, Out* __restrict__ out, int64_t* __restrict__ tile_sum) {
  __shared__ int64_t lds[kWavesPerBlock];
  const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;  // a thread owns 8 in a row
  int64_t x[kItems];
  int64_t sum = 0;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int64_t i = base + j;
    x[j] = i < n ? load(i) : 0;
    sum += x[j];
  }
  int64_t tot;
  const int64_t incl = block_incl_scan(sum, &tot, lds);
  int64_t run = incl - sum;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int64_t i = base + j;
    if (i < n) out[i] = (Out)run;
    run += x[j];
  }
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = tot;
}

template <typename Out>
__global__ __launch_bounds__(kBlock) void k_scan_offset(int64_t n, Out* __restrict__ out, const int64_t* __restrict__ tile_sum,
                                                        Out* __restrict__ end_out, int64_t* total_out, Publish pub) {
  __shared__ int64_t lds[kWavesPerBlock];
  int64_t part = 0;
  for (int64_t t = threadIdx.x; t < (int64_t)blockIdx.x; t += kBlock) part += tile_sum[t];
  part = wave_sum_i64(part);
  if (lane_id() == 0) lds[wave_in_block()] = part;
  __syncthreads();
  int64_t off = 0;
#pragma unroll
  for (int i = 0; i < kWavesPerBlock; ++i) off += lds[i];
  const int64_t base = (int64_t)blockIdx.x * kTile;
  if (off != 0) {
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      const int64_t i = base + (int64_t)j * kBlock + threadIdx.x;
      if (i < n) out[i] = (Out)((int64_t)out[i] + off);
    }
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
    const int64_t total = off + tile_sum[blockIdx.x];
    if (end_out) *end_out = (Out)total;  // the entry one past the end holds the grand total
    if (total_out) *total_out = total;
    publish_ctl(pub);
  }
}

// The same per-tile scan, and the scan of the tile sums by whichever block finishes last: one launch.  The consumer adds
// tile_prefix[tile] to an element when it reads it (TiledScan::at).
template <typename Load, typename Out>
__global__ __launch_bounds__(kBlock) void k_scan_tiled(Load load, int64_t n, Out* __restrict__ out, int64_t* __restrict__ tile_sum,
                                                       Out* __restrict__ tile_prefix, uint32_t* done, int64_t* total_out, Publish pub) {
  __shared__ int64_t lds[kWavesPerBlock];
  __shared__ uint32_t s_last;
  const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;  // a thread owns 8 in a row
  int64_t x[kItems];
  int64_t sum = 0;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int64_t i = base + j;
    x[j] = i < n ? load(i) : 0;
    sum += x[j];
  }
  int64_t tot;
  const int64_t incl = block_incl_scan(sum, &tot, lds);
  int64_t run = incl - sum;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int64_t i = base + j;
    if (i < n) out[i] = (Out)run;
    run += x[j];
  }
  if (threadIdx.x == 0) {
    __hip_atomic_store(&tile_sum[blockIdx.x], tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();  // the tile's sum is visible device-wide before the tile counts as finished
    s_last = atomicAdd(done, 1u) == gridDim.x - 1 ? 1u : 0u;
  }
  __syncthreads();
  if (s_last == 0) return;
  __threadfence();  // every other tile's sum was published before its block counted itself
  const int64_t tiles = gridDim.x;
  int64_t carry = 0;
  for (int64_t first = 0; first < tiles; first += kBlock) {
    const int64_t t = first + threadIdx.x;
    const int64_t v = t < tiles ? __hip_atomic_load(&tile_sum[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
    int64_t all;
    const int64_t upto = block_incl_scan(v, &all, lds);
    if (t < tiles) tile_prefix[t] = (Out)(carry + upto - v);
    carry += all;
  }
  if (threadIdx.x == 0) {
    out[n] = (Out)carry;  // the entry one past the end holds the grand total
    if (total_out) *total_out = carry;
    *done = 0;            // ready for the next scan of this call (the stream keeps them apart)
    publish_ctl(pub);
  }
}

// Short inputs: one block walks over the tiles with a running carry (one launch instead of two).
constexpr int64_t kScanSmall = 2 * kTile;  // 4096 elements (beyond that two parallel launches are quicker)
template <typename Load, typename Out>
__global__ __launch_bounds__(kBlock) void k_scan_small(Load load, int64_t n, Out* __restrict__ out, Out* __restrict__ end_out,
                                                       int64_t* total_out, Publish pub) {
  __shared__ int64_t lds[kWavesPerBlock];
  int64_t carry = 0;
  for (int64_t tile = 0; tile < n; tile += kTile) {
    const int64_t base = tile + (int64_t)threadIdx.x * kItems;
    int64_t x[kItems];
    int64_t sum = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      const int64_t i = base + j;
      x[j] = i < n ? load(i) : 0;
      sum += x[j];
    }
    int64_t tot;
    const int64_t incl = block_incl_scan(sum, &tot, lds);
    int64_t run = carry + incl - sum;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      const int64_t i = base + j;
      if (i < n) out[i] = (Out)run;
      run += x[j];
    }
    carry += tot;
  }
  if (threadIdx.x == 0) {
    if (end_out) *end_out = (Out)carry;
    if (total_out) *total_out = carry;
    publish_ctl(pub);
  }
}

size_t scan_tmp_bytes(int64_t n) {  // tile sums, and the one-kernel scans' tile prefixes
  const int64_t tiles = (n + kTile - 1) / kTile;
  return (size_t)(tiles + 2) * sizeof(int64_t) * 2;
}

constexpr int64_t kScanTiledMax = 64;  // tiles (131,072 elements) up to which the one-kernel scan is used
template <typename Load>
static TiledScan<uint32_t> scan_tiled_impl(Load load, int64_t n, uint32_t* out, int64_t* total_out, void* tmp, uint32_t* done, hipStream_t s,
                                           const Publish* p) {
  const Publish pub = p ? *p : Publish{};
  if (n <= kScanSmall) {  // one block; `out` is the whole scan
    COOP_LAUNCH(K_SCAN_LOCAL, (k_scan_small<Load, uint32_t>), dim3(1), dim3(kBlock), 0, s, load, n, out, out + n, total_out, pub);
    return TiledScan<uint32_t>{out, nullptr, n};
  }
  const int64_t tiles = (n + kTile - 1) / kTile;
  int64_t* tile_sum = (int64_t*)tmp;
  if (tiles > kScanTiledMax) {  // long inputs: two kernels (measured: the fences of many tiles cost more than the second launch)
    COOP_LAUNCH(K_SCAN_LOCAL, (k_scan_local<Load, uint32_t>), dim3((unsigned)tiles), dim3(kBlock), 0, s, load, n, out, tile_sum);
    COOP_LAUNCH(K_SCAN_OFFSET, k_scan_offset<uint32_t>, dim3((unsigned)tiles), dim3(kBlock), 0, s, n, out, (const int64_t*)tile_sum, out + n, total_out, pub);
    return TiledScan<uint32_t>{out, nullptr, n};
  }
  uint32_t* tile_prefix = (uint32_t*)(tile_sum + tiles + 2);
  COOP_LAUNCH(K_SCAN_LOCAL, (k_scan_tiled<Load, uint32_t>), dim3((unsigned)tiles), dim3(kBlock), 0, s, load, n, out, tile_sum, tile_prefix, done,
              total_out, pub);
  return TiledScan<uint32_t>{out, tile_prefix, n};
}

template <typename Load, typename Out>
static void scan_impl(Load load, int64_t n, Out* out, Out* end_out, int64_t* total_out, void* tmp, hipStream_t s, const Publish* p) {
  const Publish pub = p ? *p : Publish{};
  if (n <= kScanSmall) {
    COOP_LAUNCH(K_SCAN_LOCAL, (k_scan_small<Load, Out>), dim3(1), dim3(kBlock), 0, s, load, n, out, end_out, total_out, pub);
    return;
  }
  int64_t* tile_sum = (int64_t*)tmp;
  const int64_t tiles = (n + kTile - 1) / kTile;
  COOP_LAUNCH(K_SCAN_LOCAL, (k_scan_local<Load, Out>), dim3((unsigned)tiles), dim3(kBlock), 0, s, load, n, out, tile_sum);
  COOP_LAUNCH(K_SCAN_OFFSET, k_scan_offset<Out>, dim3((unsigned)tiles), dim3(kBlock), 0, s, n, out, tile_sum, end_out, total_out, pub);
}

__global__ void k_store_total(int64_t* p, int64_t* total_out, Publish pub) {
  *p = 0;
  if (total_out) *total_out = 0;
  publish_ctl(pub);
}

void scan_i32_to_i64(const int32_t* in, int64_t n, int64_t* out, int64_t* total_out, void* tmp, hipStream_t s, const Publish* pub) {
  if (n <= 0) {  // out[0] = 0
    COOP_LAUNCH(K_FILL, k_store_total, dim3(1), dim3(1), 0, s, out, total_out, pub ? *pub : Publish{});
    return;
  }
  scan_impl<LoadI32, int64_t>(LoadI32{in}, n, out, out + n, total_out, tmp, s, pub);
}

void scan_chunks_to_i64(const ChunkedI32& in, int64_t n, int64_t* out, int64_t* total_out, void* tmp, hipStream_t s, const Publish* pub) {
  if (n <= 0) {
    COOP_LAUNCH(K_FILL, k_store_total, dim3(1), dim3(1), 0, s, out, total_out, pub ? *pub : Publish{});
    return;
  }
  scan_impl<LoadChunks, int64_t>(LoadChunks{in}, n, out, out + n, total_out, tmp, s, pub);
}

void scan_u32_to_u32(const uint32_t* in, int64_t n, uint32_t* out, void* tmp, hipStream_t s) {
  scan_impl<LoadU32, uint32_t>(LoadU32{in}, n, out, out + n, nullptr, tmp, s, nullptr);
}

TiledScan<uint32_t> scan_u32_tiled(const uint32_t* in, int64_t n, uint32_t* out, void* tmp, uint32_t* done, hipStream_t s) {
  return scan_tiled_impl<LoadU32>(LoadU32{in}, n, out, nullptr, tmp, done, s, nullptr);
}

TiledScan<uint32_t> scan_popc_tiled(const uint64_t* bits, int64_t n_words, uint32_t* out, int64_t* total_out, void* tmp, uint32_t* done,
                                    hipStream_t s, const Publish* pub, const int64_t* n_bits_dev) {
  return scan_tiled_impl<LoadPopc>(LoadPopc{bits, n_bits_dev}, n_words, out, total_out, tmp, done, s, pub);
}

void scan_popc_to_u32(const uint64_t* bits, int64_t n_words, uint32_t* out, int64_t* total_out, void* tmp, hipStream_t s,
                      const Publish* pub, const int64_t* n_bits_dev) {
  scan_impl<LoadPopc, uint32_t>(LoadPopc{bits, n_bits_dev}, n_words, out, (uint32_t*)nullptr, total_out, tmp, s, pub);
}

// ---- CSR validation -------------------------------------------------------------------------------------------
// Also a census of the degrees: census[k] = number of vertices whose list has 2^k entries or more but fewer than 2^(k+1)
// (k = 0..31; lists of 2^31 entries and more in the last counter).  The samplers size the part of a grid that is set
// aside for long lists from it.
__global__ __launch_bounds__(kBlock) void k_validate_csr(const int64_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                                                         int64_t nv, int64_t ne, int32_t* __restrict__ bad,
                                                         unsigned long long* __restrict__ census) {
  __shared__ uint32_t tally[32];
  if (threadIdx.x < 32) tally[threadIdx.x] = 0;
  __syncthreads();
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  bool b = false;
  for (int64_t v = i; v < nv; v += stride) {
    const int64_t d = indptr[v + 1] - indptr[v];
    b |= d < 0;
    if (d > 0) {
      const int k = 63 - __builtin_clzll((unsigned long long)d);
      atomicAdd(&tally[k < 31 ? k : 31], 1u);
    }
  }
  for (int64_t e = i; e < ne; e += stride) b |= (uint32_t)indices[e] >= (uint64_t)nv;
  if (i == 0) b |= indptr[0] != 0 || indptr[nv] != ne;
  if (b) atomicOr(bad, 1);
  __syncthreads();
  if (threadIdx.x < 32 && tally[threadIdx.x] != 0) atomicAdd(&census[threadIdx.x], (unsigned long long)tally[threadIdx.x]);
}

// COOP_SYMMETRIC: checks that the lists are strictly ascending and that every edge t in N(s) has its reverse s in N(t),
// and records where: rev[e] = position of s in t's list, for the edge at position e of the indices array (bisection).
// Also adds up the entries of the lists longer than kLongListDegree: LABOR-0 works from the neighbours' side only on
// graphs where such lists hold a good part of the edges.
__global__ __launch_bounds__(kBlock) void k_build_reverse(const int64_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                                                          int64_t nv, uint32_t* __restrict__ rev, int32_t* bad,
                                                          unsigned long long* long_mass) {
  // one wave per vertex at a time, lanes over its list
  if (*bad != 0) return;  // (a malformed CSR was reported by the kernel before this one: its offsets cannot be trusted)
  const int64_t n_waves = ((int64_t)gridDim.x * kBlock) >> 6;
  bool b = false;
  for (int64_t s = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6; s < nv; s += n_waves) {
    const int64_t beg = indptr[s], end = indptr[s + 1];
    if (lane_id() == 0 && end - beg > kLongListDegree) atomicAdd(long_mass, (unsigned long long)(end - beg));
    for (int64_t e = beg + lane_id(); e < end; e += kWave) {
      const int32_t t = indices[e];
      if (e > beg && indices[e - 1] >= t) b = true;
      const int64_t tb = indptr[t];
      const int64_t td = indptr[t + 1] - tb;
      int64_t lo = 0, hi = td;
      while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (indices[tb + mid] < (int32_t)s) lo = mid + 1; else hi = mid;
      }
      if (lo >= td || indices[tb + lo] != (int32_t)s) { b = true; lo = 0; }
      rev[e] = (uint32_t)lo;
    }
  }
  if (b) atomicOr(bad, 1);
}

}  // namespace coop

using namespace coop;

extern "C" {

const char* coop_strerror(int code) {
  switch (code) {
    case COOP_OK: return "ok";
    case COOP_E_NULL: return "null pointer argument";
    case COOP_E_RANGE: return "vertex id out of range";
    case COOP_E_DUPSEED: return "duplicate seed vertex";
    case COOP_E_ARG: return "invalid argument";
    case COOP_E_NOMEM: return "allocator returned no memory";
    case COOP_E_CAPACITY: return "workspace capacity exceeded";
    case COOP_E_HIP: return "HIP runtime error";
    case COOP_E_GRAPH: return "malformed CSR graph";
    default: return "unknown error";
  }
}

int coop_version(void) { return 2; }

void* coop_arena_alloc(void* arena, size_t bytes, int tag) {
  (void)tag;
  coop_arena* a = (coop_arena*)arena;
  if (!a || !a->base) return nullptr;
  const size_t need = (bytes + 255) & ~(size_t)255;
  if (a->used + need > a->bytes) return nullptr;
  void* p = (char*)a->base + a->used;
  a->used += need;
  return p;
}

int coop_graph_load_with(const int64_t* indptr, const int32_t* indices, int64_t n_vertices, int64_t n_edges, int flags,
                         coop_alloc_fn alloc, void* alloc_ctx, void* stream, coop_graph** out) {
  if (!out) return COOP_E_NULL;
  *out = nullptr;
  if (!indptr || (!indices && n_edges > 0)) return COOP_E_NULL;
  if (n_vertices < 0 || n_vertices >= ((int64_t)1 << 31) || n_edges < 0 || (flags & ~(COOP_VALIDATE | COOP_SYMMETRIC))) return COOP_E_ARG;
  uint32_t* rev = nullptr;
  bool own_rev = false;  // the reverse index came from hipMalloc (no allocator given): coop_graph_free releases it
  int64_t long_mass = 0;
  bool have_census = false;
  int64_t census[32] = {};
  if (flags & (COOP_VALIDATE | COOP_SYMMETRIC)) {  // (the reverse index is built from offsets and ids that have been checked)
    hipStream_t s = (hipStream_t)stream;
    struct Check { int32_t bad, pad; unsigned long long long_mass; unsigned long long census[32]; };
    Check* d_chk = nullptr;
    if (alloc) {
      d_chk = (Check*)alloc(alloc_ctx, (sizeof(Check) + 255) & ~(size_t)255, COOP_TAG_SCRATCH);
      if (!d_chk) return COOP_E_NOMEM;
      if ((flags & COOP_SYMMETRIC) && n_edges > 0) {
        rev = (uint32_t*)alloc(alloc_ctx, (((size_t)n_edges * sizeof(uint32_t)) + 255) & ~(size_t)255, COOP_TAG_GRAPH);
        if (!rev) return COOP_E_NOMEM;
      }
    } else {
      COOP_HIP_TRY(hipMalloc((void**)&d_chk, sizeof(Check)));
      if ((flags & COOP_SYMMETRIC) && n_edges > 0) {
        if (hipMalloc((void**)&rev, (size_t)n_edges * sizeof(uint32_t)) != hipSuccess) {
          (void)hipFree(d_chk);
          return COOP_E_NOMEM;
        }
        own_rev = true;
      }
    }
    Check h_chk{};
    hipError_t e = hipMemcpyAsync(d_chk, &h_chk, sizeof(Check), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
      COOP_LAUNCH(K_VALIDATE, k_validate_csr, dim3(256 * 16), dim3(kBlock), 0, s, indptr, indices, n_vertices, n_edges, &d_chk->bad,
                  d_chk->census);
      if ((flags & COOP_SYMMETRIC) && n_vertices > 0 && n_edges > 0) {
        // (a grid holds fewer than 2^32 threads: the waves stride over the vertices)
        const int64_t want = (n_vertices * kWave + kBlock - 1) / kBlock;
        COOP_LAUNCH(K_VALIDATE, k_build_reverse, dim3((unsigned)(want < (1 << 22) ? want : (1 << 22))), dim3(kBlock), 0, s, indptr, indices,
                    n_vertices, rev, &d_chk->bad, &d_chk->long_mass);
      }
      e = hipGetLastError();
      if (e == hipSuccess) e = hipMemcpyAsync(&h_chk, d_chk, sizeof(Check), hipMemcpyDeviceToHost, s);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (!alloc) (void)hipFree(d_chk);
    if (e != hipSuccess || h_chk.bad) {
      if (own_rev) (void)hipFree(rev);
      return e != hipSuccess ? COOP_E_HIP : COOP_E_GRAPH;
    }
    long_mass = (int64_t)h_chk.long_mass;
    have_census = true;
    for (int k = 0; k < 32; ++k) census[k] = (int64_t)h_chk.census[k];
  }
  coop_graph* g = new (std::nothrow) coop_graph{indptr, indices, n_vertices, n_edges, (flags & COOP_SYMMETRIC) != 0 && n_edges > 0, rev, long_mass, own_rev};
  if (!g) {
    if (own_rev) (void)hipFree(rev);
    return COOP_E_NOMEM;
  }
  g->have_census = have_census;
  for (int k = 0; k < 32; ++k) g->census[k] = census[k];
  *out = g;
  return COOP_OK;
}

int coop_graph_load(const int64_t* indptr, const int32_t* indices, int64_t n_vertices, int64_t n_edges, int flags,
                    void* stream, coop_graph** out) {
  return coop_graph_load_with(indptr, indices, n_vertices, n_edges, flags, nullptr, nullptr, stream, out);
}

int coop_graph_free(coop_graph* g) {
  if (g && g->rev_pos && g->own_rev) (void)hipFree(g->rev_pos);
  delete g;
  return COOP_OK;
}

int coop_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (!on) collect_locked();
  g_prof.on = on != 0;
  return COOP_OK;
}

int coop_profile_filter(int id) {
  if (id >= K_COUNT_) return COOP_E_ARG;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.only = id < 0 ? -1 : id;
  return COOP_OK;
}

int coop_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  collect_locked();
  for (int i = 0; i < K_COUNT_; ++i) { g_prof.ms[i] = 0; g_prof.launches[i] = 0; }
  return COOP_OK;
}

int coop_profile_kernels(void) { return K_COUNT_; }

const char* coop_profile_name(int id) { return (id >= 0 && id < K_COUNT_) ? kKernelNames[id] : nullptr; }

int coop_profile_read(int id, double* total_ms, int64_t* launches) {
  if (id < 0 || id >= K_COUNT_) return COOP_E_ARG;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  collect_locked();
  if (total_ms) *total_ms = g_prof.ms[id];
  if (launches) *launches = g_prof.launches[id];
  return COOP_OK;
}

}  // extern "C"
