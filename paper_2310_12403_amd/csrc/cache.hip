// On-GPU LRU vertex cache in front of a feature table that lives in pinned host memory (or anywhere the device can
// read): the cached variant of Algorithm 1's feature-loading step (Sec. 4.2 measures its miss rate under kappa).
//
// Semantics (exact): a textbook LRU fed, per batch of distinct ids, first the ids that are cached when the batch
// starts, then the ids that are not, each group in batch order.  Equivalently: every access gets a stamp from a
// global counter (hits first, then misses); after the batch the cache holds the `capacity` entries with the largest
// stamps.  So, with H hits and M misses and `size` entries before the batch,
//     inserted misses  = the last min(M, capacity) misses,
//     evicted entries  = the E = max(0, size + min(M, capacity) - capacity) smallest stamps among current entries
//                        (hits were just re-stamped, so they go last).
// The E-th smallest stamp is found exactly by a most-significant-digit radix select over the stamp array (up to 8
// bits per pass, the bits of the live range split evenly over the passes; all live stamps lie in [previous eviction
// threshold, clock), so three passes are typical; each pass is one kernel, whose last block picks the digit).
//
// Data layout: slot_of[n_vertices] (int32, -1 = not cached), vertex_of[capacity], stamp[capacity] (0 = free),
// rows[capacity][row_bytes], free_list[capacity] (stack of free slots).  Which free slot a miss lands in is
// unspecified; contents, stamps and outputs are deterministic.
#include <new>

#include "coop_internal.h"
#include "device_utils.h"

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

namespace coop {

constexpr int kSelBits = 8;  // most bits per radix-select pass: 256 counters, so that merging the blocks' counts into the
constexpr int kSelBins = 1 << kSelBits;  // global ones takes at most 256 atomics per block
constexpr int kSelBlock = 1024;    // threads of a select block
constexpr int kSelMaxBlocks = 256; // one per compute unit
constexpr int kRowUnroll = 4;  // rows per thread in flight (as in the plain gather)

struct CacheCtl {
  uint64_t prefix;     // radix select: digits chosen so far; after the last pass, the E-th smallest (stamp - base)
  uint64_t remaining;  // radix select: rank still to be located inside the current prefix
  int64_t n_hit;
  int32_t n_push;      // slots pushed on the free list by the current eviction
  int32_t err_range;
  uint32_t sel_done;   // radix select: blocks of the current pass that have merged their counts (back to 0 after each pass)
  uint32_t pad;
};

// ---- lookup ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_cache_lookup(const int32_t* __restrict__ ids, int64_t n_ids, int64_t n_vertices,
                                                         const int32_t* __restrict__ slot_of, int32_t* __restrict__ slot_i,
                                                         uint64_t* __restrict__ hit_bits, CacheCtl* ctl) {
  // (several ids per thread do not make this faster: the scattered reads of slot_of, a table of one word per vertex of
  // the graph, are what it waits for, not their latency)
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  bool hit = false;
  if (i < n_ids) {
    const int32_t v = ids[i];
    int32_t slot = -1;
    if ((uint64_t)(uint32_t)v < (uint64_t)n_vertices) slot = slot_of[v];
    else atomicOr(&ctl->err_range, 1);
    slot_i[i] = slot;
    hit = slot >= 0;
  }
  const uint64_t b = ballot64(hit);
  if (lane_id() == 0 && (i & ~(int64_t)63) < n_ids) hit_bits[i >> 6] = b;
}

// order[r] = the r-th hit for r < n_hit; order[n_ids - 1 - q] = the q-th miss: the row movers then run over dense lists
// of hits and of misses instead of idling through the other kind.  An entry holds the id's index in the batch and what
// its mover reads from (the cache slot of a hit, the vertex of a miss), so that a mover reaches its row with one
// dependent load.  An id's rank among the hits is the scanned bit count of the 64-id words in front of its word plus the
// bits below it in its own word (the scan runs over n_ids / 64 words, not over n_ids flags).
struct OrderEntry {
  int32_t i;     // index in the batch: row i of `out`
  int32_t from;  // hit: cache slot; miss: vertex id
};
__global__ __launch_bounds__(kBlock) void k_cache_split(const uint64_t* __restrict__ hit_bits, const uint32_t* __restrict__ word_rank,
                                                        const int32_t* __restrict__ ids, const int32_t* __restrict__ slot_i,
                                                        int64_t n_ids, OrderEntry* __restrict__ order) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_ids) return;
  const uint64_t word = hit_bits[i >> 6];
  const int64_t h = (int64_t)word_rank[i >> 6] + __popcll(word & ((1ull << (i & 63)) - 1ull));
  if ((word >> (i & 63)) & 1ull) order[h] = OrderEntry{(int32_t)i, slot_i[i]};
  else order[n_ids - 1 - (i - h)] = OrderEntry{(int32_t)i, ids[i]};
}

// ---- row movers -----------------------------------------------------------------------------------------------
// Rows are moved by lpr = 2^lpr_log2 adjacent lanes, V-sized vectors, kRowUnroll rows per thread in flight.
template <typename V>
__global__ __launch_bounds__(kBlock) void k_cache_hits(const V* __restrict__ rows, int32_t vecs, int lpr_log2,
                                                       const OrderEntry* __restrict__ order,
                                                       const CacheCtl* __restrict__ ctl, V* __restrict__ out,
                                                       uint64_t* __restrict__ stamp, uint64_t clock) {
  const int64_t n_hit = ctl->n_hit;  // known on the device before the host has read it
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kBlock >> lpr_log2;
  const int sub = threadIdx.x & (lpr - 1);
  const int64_t row0 = ((int64_t)blockIdx.x * kRowUnroll) * rows_per_block + (threadIdx.x >> lpr_log2);
  if ((int64_t)blockIdx.x * kRowUnroll * rows_per_block >= n_hit) return;
  int64_t src[kRowUnroll], dst[kRowUnroll];
#pragma unroll
  for (int u = 0; u < kRowUnroll; ++u) {
    const int64_t r = row0 + (int64_t)u * rows_per_block;  // r-th hit
    src[u] = -1;
    dst[u] = 0;
    if (r < n_hit) {
      const OrderEntry e = order[r];
      src[u] = e.from;
      dst[u] = e.i;
    }
  }
  for (int32_t v = sub; v < vecs; v += lpr) {
    V x[kRowUnroll];
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u)
      if (src[u] >= 0) x[u] = __builtin_nontemporal_load(rows + src[u] * vecs + v);  // (a cached row is read at most once per call)
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u)
      if (src[u] >= 0) __builtin_nontemporal_store(x[u], out + dst[u] * vecs + v);
  }
  // the new stamps go out behind the rows: memory operations complete in the order in which they were sent, and the row
  // loads must not wait for these scattered stores
  if (sub == 0) {
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u)
      if (src[u] >= 0) stamp[src[u]] = clock + (uint64_t)(row0 + (int64_t)u * rows_per_block);
  }
}

template <typename V>
__global__ __launch_bounds__(kBlock) void k_cache_misses(const V* __restrict__ table, int32_t vecs, int lpr_log2,
                                                         const OrderEntry* __restrict__ order,
                                                         int64_t n_ids, V* __restrict__ out, V* __restrict__ rows,
                                                         int32_t* __restrict__ slot_of, int32_t* __restrict__ vertex_of,
                                                         uint64_t* __restrict__ stamp, const int32_t* __restrict__ free_list,
                                                         int64_t n_free, int64_t n_miss, int64_t n_ins, uint64_t clock_miss,
                                                         int64_t table_rows) {
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kBlock >> lpr_log2;
  const int sub = threadIdx.x & (lpr - 1);
  const int64_t row0 = ((int64_t)blockIdx.x * kRowUnroll) * rows_per_block + (threadIdx.x >> lpr_log2);
  int64_t src[kRowUnroll], dst[kRowUnroll], dst_slot[kRowUnroll];
  int32_t src_id[kRowUnroll];  // the vertex itself (src is its row in the table, which may be aliased)
#pragma unroll
  for (int u = 0; u < kRowUnroll; ++u) {
    const int64_t rank_m = row0 + (int64_t)u * rows_per_block;  // rank_m-th miss
    src[u] = -1;
    dst[u] = 0;
    dst_slot[u] = -1;
    src_id[u] = 0;
    if (rank_m < n_miss) {
      const OrderEntry e = order[n_ids - 1 - rank_m];
      const int32_t i = e.i, id = e.from;
      if (id >= 0) {  // ids out of range were reported by the lookup; negative ones are skipped here
        src[u] = id < table_rows ? id : id % table_rows;
        src_id[u] = id;
        dst[u] = i;
        const int64_t q = rank_m - (n_miss - n_ins);  // the last n_ins misses enter the cache
        if (q >= 0) dst_slot[u] = free_list[n_free - 1 - q];
      }
    }
  }
  for (int32_t v = sub; v < vecs; v += lpr) {
    V x[kRowUnroll];
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u)
      if (src[u] >= 0) x[u] = __builtin_nontemporal_load(table + src[u] * vecs + v);
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u) {
      if (src[u] >= 0) {
        __builtin_nontemporal_store(x[u], out + dst[u] * vecs + v);
        if (dst_slot[u] >= 0) __builtin_nontemporal_store(x[u], rows + dst_slot[u] * vecs + v);  // (not read again before a later call)
      }
    }
  }
  // the books of the rows that entered the cache, behind the row traffic as well (a kernel of its own for these three
  // stores costs more than it takes off this one)
  if (sub == 0) {
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u)
      if (dst_slot[u] >= 0) {
        slot_of[src_id[u]] = (int32_t)dst_slot[u];
        vertex_of[dst_slot[u]] = src_id[u];
        stamp[dst_slot[u]] = clock_miss + (uint64_t)(row0 + (int64_t)u * rows_per_block);
      }
  }
}

// ---- eviction: radix select of the E-th smallest stamp, then sweep -----------------------------------------------
// One pass of the select: counts, per value of the next `bits` bits, the live entries whose leading digits equal the
// prefix found so far; the block that merges its counts last (a counter in the control block; nobody waits) finds the
// digit that holds the `remaining`-th entry, extends the prefix and clears the counters for the next pass.
__global__ __launch_bounds__(kSelBlock) void k_cache_sel_pass(const uint64_t* __restrict__ stamp, int64_t capacity, uint64_t base,
                                                              int shift, int bits, int prev_shift, CacheCtl* ctl,
                                                              uint32_t* __restrict__ hist) {
  __shared__ uint32_t lh[kSelBins];
  __shared__ uint32_t wave_tot[kSelBins / kWave];
  __shared__ uint32_t s_last;
  if (threadIdx.x < kSelBins) lh[threadIdx.x] = 0;
  __syncthreads();
  const uint64_t prefix = ctl->prefix;
  const uint32_t digit_mask = (1u << bits) - 1u;
  const int64_t stride = (int64_t)gridDim.x * kSelBlock;
  constexpr int U = 4;  // stamps per thread in flight
  for (int64_t first = (int64_t)blockIdx.x * kSelBlock + threadIdx.x; first < capacity; first += U * stride) {
    uint64_t st[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = first + u * stride;
      st[u] = i < capacity ? stamp[i] : 0;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t x = st[u] - base;
      const bool in = st[u] != 0 && (prev_shift < 0 || (x >> prev_shift) == prefix);
      const uint32_t digit = (uint32_t)(x >> shift) & digit_mask;
      // neighbouring slots were mostly filled by the same call and share a digit: one add for the wave then
      const uint64_t m = ballot64(in);
      if (m == 0) continue;
      const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, __builtin_ctzll(m));
      if (ballot64(in && digit == d0) == m) {
        if ((uint32_t)lane_id() == (uint32_t)__builtin_ctzll(m)) atomicAdd(&lh[d0], (uint32_t)__popcll(m));
      } else if (in) {
        atomicAdd(&lh[digit], 1u);
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < kSelBins) {
    const uint32_t c = lh[threadIdx.x];
    if (c) atomicAdd(&hist[threadIdx.x], c);
  }
  __syncthreads();  // the block's adds have been performed (each wave waits for its own before the barrier)
  if (threadIdx.x == 0) {
    __threadfence();  // ... and are ordered before the block counts as done
    s_last = atomicAdd(&ctl->sel_done, 1u) == gridDim.x - 1 ? 1u : 0u;
    __threadfence();  // every other block merged its counts before it counted itself
  }
  __syncthreads();
  if (s_last == 0) return;
  const bool has = threadIdx.x < kSelBins;  // (the first kSelBins / 64 waves, whole)
  const uint32_t v = has ? __hip_atomic_load(&hist[threadIdx.x % kSelBins], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
  uint32_t incl = wave_incl_scan(v);
  if (has && lane_id() == kWave - 1) wave_tot[threadIdx.x / kWave] = incl;
  __syncthreads();
  if (!has) return;
  for (int w = 0; w < (int)threadIdx.x / kWave; ++w) incl += wave_tot[w];
  uint32_t total = 0;
  for (int w = 0; w < kSelBins / kWave; ++w) total += wave_tot[w];
  const uint64_t remaining = ctl->remaining;
  const uint64_t before = (uint64_t)(incl - v);
  // the digit that holds the remaining-th entry; if the counts fall short of it (they do not), the last digit
  const bool mine = remaining > (uint64_t)total ? threadIdx.x == digit_mask : (before < remaining && remaining <= (uint64_t)incl);
  if (mine) {
    ctl->prefix = (prefix << bits) | (uint64_t)threadIdx.x;
    ctl->remaining = remaining - before;
    ctl->sel_done = 0;
  }
  __hip_atomic_store(&hist[threadIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Evicts every entry with stamp - base <= threshold (or every entry, if evict_all) and pushes the freed slots on the
// free list.  Each block owns a contiguous chunk of slots: it first counts its evictions, reserves that many free-list
// places with ONE atomic, then sweeps the chunk again handing out the places by ballot and a running offset.
__global__ __launch_bounds__(kBlock) void k_cache_evict(uint64_t* __restrict__ stamp, int32_t* __restrict__ vertex_of,
                                                        int32_t* __restrict__ slot_of, int32_t* __restrict__ free_list,
                                                        int64_t capacity, int64_t chunk, uint64_t base, bool evict_all,
                                                        int64_t n_free, CacheCtl* ctl) {
  __shared__ int32_t wave_cnt[kWavesPerBlock];
  __shared__ int32_t block_base;
  const uint64_t thr = ctl->prefix;
  const int64_t lo = (int64_t)blockIdx.x * chunk;
  const int64_t hi = lo + chunk < capacity ? lo + chunk : capacity;
  const int lane = lane_id(), wib = wave_in_block();
  auto is_out = [&](int64_t i) {
    if (i >= hi) return false;
    const uint64_t st = stamp[i];
    return st != 0 && (evict_all || st - base <= thr);
  };
  // pass 1: how many
  int32_t mine = 0;
  for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) mine += is_out(i);
  mine = (int32_t)wave_sum_i64(mine);
  if (lane == 0) wave_cnt[wib] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    int32_t total = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) total += wave_cnt[w];
    block_base = total ? atomicAdd(&ctl->n_push, total) : 0;
  }
  __syncthreads();
  int64_t run = n_free + block_base;
  // pass 2: hand out the places (chunk is a multiple of the block size, so every thread runs every round)
  for (int64_t r = lo; r < hi; r += kBlock) {
    const int64_t i = r + threadIdx.x;
    const bool out = is_out(i);
    const uint64_t mask = ballot64(out);
    __syncthreads();
    if (lane == 0) wave_cnt[wib] = (int32_t)__popcll(mask);
    __syncthreads();
    int32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
      const int32_t cw = wave_cnt[w];
      if (w < wib) before += cw;
      total += cw;
    }
    if (out) {
      const int32_t v = vertex_of[i];
      slot_of[v] = -1;
      vertex_of[i] = -1;
      stamp[i] = 0;
      const int64_t p = run + before + (int64_t)lanes_below(mask);
      if (p < capacity) free_list[p] = (int32_t)i;  // always true: exactly n_evict entries qualify
    }
    run += total;
  }
}

__global__ void k_cache_ctl_set(CacheCtl* ctl, uint64_t remaining) {
  ctl->prefix = 0; ctl->remaining = remaining; ctl->n_push = 0; ctl->sel_done = 0;
}

__global__ void k_cache_clear_err(CacheCtl* ctl) { ctl->err_range = 0; }

// Landing pad in mapped pinned host memory.  The counts of a call reach the host by a one-thread kernel that stores the
// control block and then a ticket, which the host polls: quicker than an asynchronous copy and a wait for it.
struct CachePad {
  CacheCtl ctl;          // counts of the call under way; must stay the first member
  uint64_t ticket;       // written by the device after ctl
  uint64_t next_ticket;  // host side only
  CacheCtl threshold;    // control block after the last eviction (copied, read one call late)
};
__global__ void k_cache_publish(const CacheCtl* __restrict__ ctl, CachePad* pad, uint64_t ticket) {
  pad->ctl = *ctl;
  __threadfence_system();
  __hip_atomic_store(&pad->ticket, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(kBlock) void k_fill_i32(int32_t* __restrict__ p, int64_t n, int32_t v, bool iota) {
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (; i < n; i += stride) p[i] = iota ? (int32_t)i : v;
}

}  // namespace coop

using namespace coop;

struct coop_cache {
  int64_t capacity, n_vertices, max_ids, row_bytes;
  int vec_bytes;          // 16 / 8 / 4 / 2: widest vector that divides the row and the buffers' alignment
  int32_t* slot_of;
  int32_t* vertex_of;
  uint64_t* stamp;
  void* rows;
  int32_t* free_list;
  // per-call scratch, sized for max_ids
  int32_t* slot_i;
  uint64_t* hit_bits;
  uint32_t* rank_h;
  OrderEntry* order;      // hits from the front, misses from the back
  void* scan_tmp;
  uint32_t* hist;
  CacheCtl* d_ctl;
  CachePad* pad;          // mapped pinned
  hipEvent_t ev_threshold;  // threshold of the last eviction has landed in pad->threshold
  bool base_pending;      // ... and has not been added to base yet
  // host-side state
  int64_t size;           // entries held
  uint64_t clock;         // next stamp
  uint64_t base;          // every live stamp is >= base (last eviction threshold + 1)
};

// Pinned memory and event of a cache; whatever was created is released.
static void release_host_side(coop_cache* c) {
  if (c->ev_threshold) { (void)hipEventSynchronize(c->ev_threshold); (void)hipEventDestroy(c->ev_threshold); }
  if (c->pad) (void)hipHostFree(c->pad);
}

// The threshold of the last eviction, once it has arrived: everything at or below it is gone.
static int settle_base(coop_cache* c) {
  if (!c->base_pending) return COOP_OK;
  COOP_HIP_TRY(hipEventSynchronize(c->ev_threshold));
  c->base += c->pad->threshold.prefix + 1;
  c->base_pending = false;
  return COOP_OK;
}

static unsigned grid_for(int64_t n) {
  int64_t b = (n + kBlock - 1) / kBlock;
  if (b > 256 * 32) b = 256 * 32;
  return (unsigned)(b > 0 ? b : 1);
}

extern "C" int coop_cache_create(int64_t capacity_rows, int64_t n_vertices, int32_t dim, int dtype, int64_t max_ids,
                                 coop_alloc_fn alloc_fn, void* alloc_ctx, void* stream, coop_cache** out) {
  if (!out) return COOP_E_NULL;
  *out = nullptr;
  if (!alloc_fn) return COOP_E_NULL;
  if (dtype != COOP_F32 && dtype != COOP_F16) return COOP_E_ARG;
  if (capacity_rows < 0 || capacity_rows >= ((int64_t)1 << 31) || n_vertices < 0 || n_vertices >= ((int64_t)1 << 31) ||
      dim < 1 || max_ids < 0 || max_ids >= ((int64_t)1 << 31))
    return COOP_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  coop_cache* c = new (std::nothrow) coop_cache{};
  if (!c) return COOP_E_NOMEM;
  c->capacity = capacity_rows; c->n_vertices = n_vertices; c->max_ids = max_ids;
  c->row_bytes = (int64_t)dim * (dtype == COOP_F32 ? 4 : 2);
  Alloc alloc{alloc_fn, alloc_ctx};
  c->slot_of = alloc.get<int32_t>(n_vertices, COOP_TAG_OUTPUT);
  c->vertex_of = alloc.get<int32_t>(capacity_rows, COOP_TAG_OUTPUT);
  c->stamp = alloc.get<uint64_t>(capacity_rows, COOP_TAG_OUTPUT);
  c->rows = alloc.get<char>(capacity_rows * c->row_bytes, COOP_TAG_OUTPUT);
  c->free_list = alloc.get<int32_t>(capacity_rows, COOP_TAG_OUTPUT);
  c->slot_i = alloc.get<int32_t>(max_ids, COOP_TAG_OUTPUT);
  c->hit_bits = alloc.get<uint64_t>((max_ids + 63) / 64, COOP_TAG_OUTPUT);
  c->rank_h = alloc.get<uint32_t>(max_ids, COOP_TAG_OUTPUT);
  c->order = alloc.get<OrderEntry>(max_ids, COOP_TAG_OUTPUT);
  c->scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(max_ids), COOP_TAG_OUTPUT);
  c->hist = alloc.get<uint32_t>(kSelBins, COOP_TAG_OUTPUT);
  c->d_ctl = alloc.get<CacheCtl>(1, COOP_TAG_OUTPUT);
  if (alloc.failed) { delete c; return COOP_E_NOMEM; }
  if (hipHostMalloc((void**)&c->pad, sizeof(CachePad), hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_threshold, hipEventDisableTiming) != hipSuccess) {
    release_host_side(c);
    delete c;
    return COOP_E_HIP;
  }
  *c->pad = CachePad{};
  c->size = 0; c->clock = 1; c->base = 1;
  if (n_vertices > 0) COOP_LAUNCH(K_FILL, k_fill_i32, dim3(grid_for(n_vertices)), dim3(kBlock), 0, s, c->slot_of, n_vertices, -1, false);
  if (capacity_rows > 0) {
    COOP_LAUNCH(K_FILL, k_fill_i32, dim3(grid_for(capacity_rows)), dim3(kBlock), 0, s, c->vertex_of, capacity_rows, -1, false);
    COOP_LAUNCH(K_FILL, k_fill_i32, dim3(grid_for(capacity_rows)), dim3(kBlock), 0, s, c->free_list, capacity_rows, 0, true);
    fill_u64(c->stamp, capacity_rows, 0, s);
  }
  fill_u64((uint64_t*)c->hist, kSelBins / 2, 0, s);
  COOP_LAUNCH(K_FILL, k_cache_ctl_set, dim3(1), dim3(1), 0, s, c->d_ctl, (uint64_t)0);
  COOP_LAUNCH(K_FILL, k_cache_clear_err, dim3(1), dim3(1), 0, s, c->d_ctl);
  if (hipStreamSynchronize(s) != hipSuccess) { release_host_side(c); delete c; return COOP_E_HIP; }
  *out = c;
  return COOP_OK;
}

extern "C" int coop_cache_free(coop_cache* c) {
  if (!c) return COOP_OK;
  release_host_side(c);
  delete c;
  return COOP_OK;
}

// ---- export / import (checkpoint and resume) --------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_cache_export(const int32_t* __restrict__ vertex_of, const uint64_t* __restrict__ stamp,
                                                         int64_t capacity, int32_t* __restrict__ vertices_out,
                                                         uint64_t* __restrict__ stamps_out, CacheCtl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const bool live = i < capacity && stamp[i] != 0;
  const uint64_t mask = ballot64(live);
  if (mask == 0) return;
  int32_t first = 0;
  if (lane_id() == 0) first = atomicAdd(&ctl->n_push, (int32_t)__popcll(mask));
  first = __builtin_amdgcn_readfirstlane(first);
  if (live) {
    const int64_t p = first + (int64_t)lanes_below(mask);
    vertices_out[p] = vertex_of[i];
    stamps_out[p] = stamp[i];
  }
}

// entry i of the exported lists goes to slot i; its row is read again from the backing table
template <typename V>
__global__ __launch_bounds__(kBlock) void k_cache_import(const V* __restrict__ table, int64_t table_rows, int32_t vecs, int lpr_log2,
                                                         const int32_t* __restrict__ vertices, const uint64_t* __restrict__ stamps,
                                                         int64_t n, int64_t n_vertices, V* __restrict__ rows,
                                                         int32_t* __restrict__ slot_of, int32_t* __restrict__ vertex_of,
                                                         uint64_t* __restrict__ stamp, CacheCtl* ctl) {
  const int lpr = 1 << lpr_log2;
  const int sub = threadIdx.x & (lpr - 1);
  const int64_t i = (int64_t)blockIdx.x * (kBlock >> lpr_log2) + (threadIdx.x >> lpr_log2);
  if (i >= n) return;
  const int32_t v = vertices[i];
  if ((uint64_t)(uint32_t)v >= (uint64_t)n_vertices || stamps[i] == 0) {
    if (sub == 0) atomicOr(&ctl->err_range, 1);
    return;
  }
  if (sub == 0) {
    slot_of[v] = (int32_t)i;
    vertex_of[i] = v;
    stamp[i] = stamps[i];
  }
  const int64_t src = v < table_rows ? v : v % table_rows;
  for (int32_t c = sub; c < vecs; c += lpr) rows[i * vecs + c] = table[src * vecs + c];
}

// every listed vertex must own its slot: a vertex listed twice owns only one of the two
__global__ __launch_bounds__(kBlock) void k_cache_import_check(const int32_t* __restrict__ slot_of, const int32_t* __restrict__ vertex_of,
                                                               int64_t n, CacheCtl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const int32_t v = vertex_of[i];
  if (v < 0 || slot_of[v] != (int32_t)i) atomicOr(&ctl->err_range, 1);
}

__global__ __launch_bounds__(kBlock) void k_cache_free_tail(int32_t* __restrict__ free_list, int64_t n_live, int64_t capacity) {
  // free slots are n_live .. capacity-1; the stack pops from its top, any order will do
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < capacity - n_live) free_list[i] = (int32_t)(n_live + i);
}

extern "C" int coop_cache_export(coop_cache* c, int32_t* vertices_out, uint64_t* stamps_out, coop_cache_state* state_out, void* stream) {
  if (!c || !state_out || (c->capacity > 0 && (!vertices_out || !stamps_out))) return COOP_E_NULL;
  hipStream_t s = (hipStream_t)stream;
  COOP_LAUNCH(K_FILL, k_cache_ctl_set, dim3(1), dim3(1), 0, s, c->d_ctl, (uint64_t)0);
  if (c->capacity > 0)
    COOP_LAUNCH(K_CACHE_LOOKUP, k_cache_export, dim3((unsigned)((c->capacity + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, c->vertex_of,
                c->stamp, c->capacity, vertices_out, stamps_out, c->d_ctl);
  COOP_HIP_TRY(hipStreamSynchronize(s));
  if (int rc = settle_base(c)) return rc;
  state_out->size = c->size;
  state_out->clock = c->clock;
  state_out->base = c->base;
  return COOP_OK;
}

extern "C" int coop_cache_import(coop_cache* c, const void* table, int64_t table_rows, const int32_t* vertices, const uint64_t* stamps,
                                 const coop_cache_state* state, void* stream) {
  if (!c || !state) return COOP_E_NULL;
  if (state->size < 0 || state->size > c->capacity || table_rows < 1 || state->clock == 0 || state->base == 0) return COOP_E_ARG;
  if (state->size > 0 && (!table || !vertices || !stamps)) return COOP_E_NULL;
  hipStream_t s = (hipStream_t)stream;
  if (int rc = settle_base(c)) return rc;
  // back to the empty state (n_live slots reserved at the front), then the listed entries into slots 0 .. size-1
  auto reset = [&](int64_t n_live) {
    if (c->n_vertices > 0) COOP_LAUNCH(K_FILL, k_fill_i32, dim3(grid_for(c->n_vertices)), dim3(kBlock), 0, s, c->slot_of, c->n_vertices, -1, false);
    if (c->capacity > 0) {
      COOP_LAUNCH(K_FILL, k_fill_i32, dim3(grid_for(c->capacity)), dim3(kBlock), 0, s, c->vertex_of, c->capacity, -1, false);
      fill_u64(c->stamp, c->capacity, 0, s);
      COOP_LAUNCH(K_FILL, k_cache_free_tail, dim3(grid_for(c->capacity)), dim3(kBlock), 0, s, c->free_list, n_live, c->capacity);
    }
    COOP_LAUNCH(K_FILL, k_cache_clear_err, dim3(1), dim3(1), 0, s, c->d_ctl);
  };
  reset(state->size);
  if (state->size > 0) {
    const uintptr_t align = (uintptr_t)table | (uintptr_t)c->rows | (uintptr_t)c->row_bytes;
    const int vb = align % 16 == 0 ? 16 : align % 8 == 0 ? 8 : align % 4 == 0 ? 4 : 2;
    const int32_t vecs = (int32_t)(c->row_bytes / vb);
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < vecs && lpr_log2 < 8) ++lpr_log2;
    const unsigned grid = (unsigned)((state->size + (kBlock >> lpr_log2) - 1) / (kBlock >> lpr_log2));
#define COOP_IMPORT(V) COOP_LAUNCH(K_CACHE_UPDATE, k_cache_import<V>, dim3(grid), dim3(kBlock), 0, s, (const V*)table, table_rows, vecs, \
                                   lpr_log2, vertices, stamps, state->size, c->n_vertices, (V*)c->rows, c->slot_of, c->vertex_of,     \
                                   c->stamp, c->d_ctl)
    if (vb == 16) COOP_IMPORT(u32x4);
    else if (vb == 8) COOP_IMPORT(u32x2);
    else if (vb == 4) COOP_IMPORT(uint32_t);
    else COOP_IMPORT(uint16_t);
#undef COOP_IMPORT
    COOP_LAUNCH(K_CACHE_LOOKUP, k_cache_import_check, dim3(grid_for(state->size)), dim3(kBlock), 0, s, c->slot_of, c->vertex_of, state->size,
                c->d_ctl);
  }
  COOP_HIP_TRY(hipMemcpyAsync(&c->pad->ctl, c->d_ctl, sizeof(CacheCtl), hipMemcpyDeviceToHost, s));
  COOP_HIP_TRY(hipStreamSynchronize(s));
  if (c->pad->ctl.err_range) {  // a bad list (vertex out of range or listed twice, zero stamp): leave an empty cache
    reset(0);
    COOP_HIP_TRY(hipStreamSynchronize(s));
    c->size = 0; c->clock = 1; c->base = 1;
    return COOP_E_RANGE;
  }
  c->size = state->size;
  c->clock = state->clock;
  c->base = state->base;
  return COOP_OK;
}

extern "C" int coop_map_host_pointer(const void* host, void** device_out) {
  if (!host || !device_out) return COOP_E_NULL;
  void* d = nullptr;
  if (hipHostGetDevicePointer(&d, const_cast<void*>(host), 0) != hipSuccess || !d) {
    (void)hipGetLastError();
    return COOP_E_ARG;
  }
  *device_out = d;
  return COOP_OK;
}

extern "C" int coop_cache_vertices(const coop_cache* c, const int32_t** vertex_of_out, int64_t* size_out) {
  if (!c) return COOP_E_NULL;
  if (vertex_of_out) *vertex_of_out = c->vertex_of;
  if (size_out) *size_out = c->size;
  return COOP_OK;
}

namespace {
template <typename V>
void launch_rows(coop_cache* c, const void* table, int64_t table_rows, const int32_t* ids, int64_t n_ids, void* out, int64_t n_free,
                 int64_t n_miss, int64_t n_ins, int64_t n_hit, bool hits, hipStream_t s) {
  const int32_t vecs = (int32_t)(c->row_bytes / (int64_t)sizeof(V));
  int lpr_log2 = 0;
  while ((1 << lpr_log2) < vecs && lpr_log2 < 8) ++lpr_log2;
  const int64_t rows_per_launch_block = (int64_t)(kBlock >> lpr_log2) * kRowUnroll;
  const unsigned grid = (unsigned)((n_ids + rows_per_launch_block - 1) / rows_per_launch_block);
  if (hits) {
    COOP_LAUNCH(K_CACHE_GATHER, k_cache_hits<V>, dim3(grid), dim3(kBlock), 0, s, (const V*)c->rows, vecs, lpr_log2, (const OrderEntry*)c->order,
                c->d_ctl, (V*)out, c->stamp, c->clock);
  } else {
    const unsigned grid_m = (unsigned)((n_miss + rows_per_launch_block - 1) / rows_per_launch_block);
    COOP_LAUNCH(K_CACHE_UPDATE, k_cache_misses<V>, dim3(grid_m), dim3(kBlock), 0, s, (const V*)table, vecs, lpr_log2, (const OrderEntry*)c->order, n_ids,
                (V*)out, (V*)c->rows, c->slot_of, c->vertex_of, c->stamp, c->free_list, n_free, n_miss, n_ins,
                c->clock + (uint64_t)n_hit, table_rows);
  }
}

void dispatch_rows(coop_cache* c, int vec_bytes, const void* table, int64_t table_rows, const int32_t* ids, int64_t n_ids, void* out,
                   int64_t n_free, int64_t n_miss, int64_t n_ins, int64_t n_hit, bool hits, hipStream_t s) {
  switch (vec_bytes) {
    case 16: launch_rows<u32x4>(c, table, table_rows, ids, n_ids, out, n_free, n_miss, n_ins, n_hit, hits, s); break;
    case 8: launch_rows<u32x2>(c, table, table_rows, ids, n_ids, out, n_free, n_miss, n_ins, n_hit, hits, s); break;
    case 4: launch_rows<uint32_t>(c, table, table_rows, ids, n_ids, out, n_free, n_miss, n_ins, n_hit, hits, s); break;
    default: launch_rows<uint16_t>(c, table, table_rows, ids, n_ids, out, n_free, n_miss, n_ins, n_hit, hits, s); break;
  }
}
}  // namespace

extern "C" int coop_cache_gather(coop_cache* c, const void* table, int64_t table_rows, const int32_t* ids, int64_t n_ids, void* out,
                                 int64_t* n_miss_out, void* stream) {
  if (!c) return COOP_E_NULL;
  if (table_rows < 1) return COOP_E_ARG;
  if (n_ids < 0 || n_ids > c->max_ids) return COOP_E_CAPACITY;
  if (n_miss_out) *n_miss_out = 0;
  if (n_ids == 0) return COOP_OK;
  if (!table || !ids || !out) return COOP_E_NULL;
  hipStream_t s = (hipStream_t)stream;
  const uintptr_t align = (uintptr_t)table | (uintptr_t)out | (uintptr_t)c->rows | (uintptr_t)c->row_bytes;
  const int vec_bytes = align % 16 == 0 ? 16 : align % 8 == 0 ? 8 : align % 4 == 0 ? 4 : 2;
  if (align % 2 != 0) return COOP_E_ARG;

  // (a call on another stream than the last one's: the threshold of that one is still to be copied out of the control block)
  if (c->base_pending) COOP_HIP_TRY(hipStreamWaitEvent(s, c->ev_threshold, 0));
  // 1. lookup, hit ranks
  COOP_LAUNCH(K_FILL, k_cache_ctl_set, dim3(1), dim3(1), 0, s, c->d_ctl, (uint64_t)0);
  COOP_LAUNCH(K_CACHE_LOOKUP, k_cache_lookup, dim3((unsigned)((n_ids + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, ids, n_ids,
              c->n_vertices, c->slot_of, c->slot_i, c->hit_bits, c->d_ctl);
  scan_popc_to_u32(c->hit_bits, (n_ids + 63) / 64, c->rank_h, &c->d_ctl->n_hit, c->scan_tmp, s);
  const uint64_t ticket = ++c->pad->next_ticket;  // the counts are known from here on: on their way while the split runs
  COOP_LAUNCH(K_FILL, k_cache_publish, dim3(1), dim3(1), 0, s, (const CacheCtl*)c->d_ctl, c->pad, ticket);
  COOP_LAUNCH(K_CACHE_LOOKUP, k_cache_split, dim3((unsigned)((n_ids + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, (const uint64_t*)c->hit_bits,
              (const uint32_t*)c->rank_h, ids, (const int32_t*)c->slot_i, n_ids, c->order);
  // 2. hits: rows out of the cache, new stamps (runs while the host waits for the counts and queues the rest)
  dispatch_rows(c, vec_bytes, table, table_rows, ids, n_ids, out, 0, 0, 0, 0, true, s);
  {  // the wait is bounded: after a while, or once the stream has run dry, the host synchronises instead
    bool seen = false;
    for (int64_t spin = 0; spin < ((int64_t)1 << 26); ++spin) {
      if (__atomic_load_n(&c->pad->ticket, __ATOMIC_ACQUIRE) == ticket) { seen = true; break; }
      if ((spin & 0xFFFF) == 0xFFFF && hipStreamQuery(s) == hipSuccess) break;
      __builtin_ia32_pause();
    }
    if (!seen) {
      COOP_HIP_TRY(hipStreamSynchronize(s));
      if (__atomic_load_n(&c->pad->ticket, __ATOMIC_ACQUIRE) != ticket) return COOP_E_HIP;
    }
  }
  if (int rc = settle_base(c)) return rc;
  if (c->pad->ctl.err_range) {
    // the cached ids of this call were already served and re-stamped: keep the stamps unique, insert nothing
    COOP_LAUNCH(K_FILL, k_cache_clear_err, dim3(1), dim3(1), 0, s, c->d_ctl);
    c->clock += (uint64_t)n_ids;
    (void)hipStreamSynchronize(s);
    return COOP_E_RANGE;
  }
  const int64_t n_hit = c->pad->ctl.n_hit;
  const int64_t n_miss = n_ids - n_hit;
  const int64_t n_ins = n_miss < c->capacity ? n_miss : c->capacity;
  int64_t n_evict = c->size + n_ins - c->capacity;
  if (n_evict < 0) n_evict = 0;
  int64_t n_free = c->capacity - c->size;

  // 3. eviction
  const uint64_t clock_after = c->clock + (uint64_t)n_ids;
  bool threshold_known = false;
  if (n_evict > 0) {
    const bool evict_all = n_evict >= c->size;
    if (!evict_all) {
      uint64_t range = clock_after - c->base;  // live stamps minus base lie in [0, range)
      int nbits = 1;
      while (nbits < 64 && (range >> nbits) != 0) ++nbits;
      const int passes = (nbits + kSelBits - 1) / kSelBits;
      COOP_LAUNCH(K_FILL, k_cache_ctl_set, dim3(1), dim3(1), 0, s, c->d_ctl, (uint64_t)n_evict);
      // the bits of the range are split evenly over the passes
      int prev_shift = -1, shift = nbits;
      for (int p = 0; p < passes; ++p) {
        const int bits = (shift + (passes - p) - 1) / (passes - p);
        shift -= bits;
        int64_t blocks = (c->capacity + kSelBlock * 4 - 1) / (kSelBlock * 4);
        if (blocks > kSelMaxBlocks) blocks = kSelMaxBlocks;
        COOP_LAUNCH(K_CACHE_SELECT, k_cache_sel_pass, dim3((unsigned)(blocks > 0 ? blocks : 1)), dim3(kSelBlock), 0, s, c->stamp, c->capacity,
                    c->base, shift, bits, prev_shift, c->d_ctl, c->hist);
        prev_shift = shift;
      }
      threshold_known = true;
    }
    {
      // at most 1,024 blocks: every block reserves its places with an atomic on one counter, which takes them one after
      // the other (some 20 ns each), and the longer runs of neighbouring slots that a block hands out make the rows that
      // the miss mover writes next lie closer together (with 2,048 blocks the sweep takes 0.086 instead of 0.077 ms and
      // the mover 0.38 instead of 0.34 to 0.36; with 256 the sweep itself takes 0.117)
      int64_t blocks = (c->capacity + kBlock - 1) / kBlock;
      if (blocks > 1024) blocks = 1024;
      int64_t chunk = (c->capacity + blocks - 1) / blocks;
      chunk = (chunk + kBlock - 1) / kBlock * kBlock;
      blocks = (c->capacity + chunk - 1) / chunk;
      COOP_LAUNCH(K_CACHE_EVICT, k_cache_evict, dim3((unsigned)blocks), dim3(kBlock), 0, s, c->stamp, c->vertex_of, c->slot_of,
                  c->free_list, c->capacity, chunk, c->base, evict_all, n_free, c->d_ctl);
    }
    n_free += n_evict;
    c->size -= n_evict;
  }

  // 4. misses: rows from the backing table to `out`, the last n_ins of them also into free slots
  if (n_miss > 0) dispatch_rows(c, vec_bytes, table, table_rows, ids, n_ids, out, n_free, n_miss, n_ins, n_hit, false, s);
  c->size += n_ins;
  c->clock = clock_after;

  if (threshold_known) {  // read when it is next needed: the call does not wait for its own row copies
    COOP_HIP_TRY(hipMemcpyAsync(&c->pad->threshold, c->d_ctl, sizeof(CacheCtl), hipMemcpyDeviceToHost, s));
    COOP_HIP_TRY(hipEventRecord(c->ev_threshold, s));
    c->base_pending = true;
  }
  if (n_miss_out) *n_miss_out = n_miss;
  return COOP_OK;
}
