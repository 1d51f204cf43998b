// Frontier dedup and relabelling (Eq. 2: S^{l+1} = S^l ∪ sampled sources): every edge's source vertex gets the FIRST
// position of that vertex in the list [S^l ; col_global], through hash tables in LDS after a partition of the list into
// buckets (long lists, further down) or through one open-addressing hash table in HBM (short lists, and the fallback).
//
// The table in HBM: the list is inserted into a table of 8-byte slots (key << 32 | position in that list).  A slot is
// claimed with atomicCAS; every further occurrence of the key lowers the slot's position with atomicMin, so after
// the insert kernel each slot holds the FIRST position of its key, whichever thread won the race.  A vertex is
// "new" exactly at the edge whose position equals that first position (and is not a seed position).  The new-flags
// are kept as a bit per edge; a device-wide scan over the words' bit counts plus a bit count inside the word gives each
// new vertex its rank, hence its place n_dst + rank in S^{l+1}: the order is "S^l, then first appearance in
// col_global", independent of scheduling.
#include "coop_internal.h"
#include "device_utils.h"

namespace coop {

constexpr uint64_t kEmptySlot = ~0ull;

// multiplicative (Fibonacci) hashing of the key to 32 bits, then multiply-high range reduction onto [0, cap)
__device__ __forceinline__ uint64_t slot_of_key(uint32_t key, uint64_t cap) {
  const uint32_t h = (uint32_t)(((uint64_t)key * 0x9E3779B97F4A7C15ull) >> 32);
  return ((uint64_t)h * cap) >> 32;
}

// (m_dev, optional: the exact number of edges, on the device; m is then the capacity of col)
__global__ __launch_bounds__(kBlock) void k_uniq_insert(const int32_t* __restrict__ dst, int64_t n_dst,
                                                        const int32_t* __restrict__ col, int64_t m, const int64_t* __restrict__ m_dev,
                                                        unsigned long long* __restrict__ table, uint64_t cap, Ctl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (m_dev != nullptr && *m_dev < m) m = *m_dev;
  if (i >= n_dst + m) return;
  const uint32_t key = (uint32_t)(i < n_dst ? dst[i] : col[i - n_dst]);
  const unsigned long long mine = ((unsigned long long)key << 32) | (uint32_t)i;
  uint64_t h = slot_of_key(key, cap);
  for (;;) {
    unsigned long long cur = __hip_atomic_load(&table[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (cur == kEmptySlot) {
      cur = atomicCAS(&table[h], (unsigned long long)kEmptySlot, mine);
      if (cur == kEmptySlot) return;  // claimed
    }
    if ((uint32_t)(cur >> 32) == key) {
      // an edge position above the one already recorded cannot lower it: no atomic needed (this is what keeps a
      // hub that shows up in thousands of lists from serialising thousands of atomics on one slot)
      if (i >= n_dst && cur < mine) return;
      const unsigned long long old = atomicMin(&table[h], mine);
      // two positions below n_dst with one key: the destination list holds a vertex twice
      if (i < n_dst && (int64_t)(uint32_t)old < n_dst) atomicOr(&ctl->err_dup, 1);
      return;
    }
    if (++h == cap) h = 0;  // the table is at most half full, so an empty slot or the key is always reached
  }
}

__device__ __forceinline__ uint32_t first_position(const unsigned long long* __restrict__ table, uint64_t cap, uint32_t key) {
  uint64_t h = slot_of_key(key, cap);
  for (;;) {
    const unsigned long long cur = table[h];
    if ((uint32_t)(cur >> 32) == key) return (uint32_t)cur;
    if (cur == kEmptySlot) return 0xFFFFFFFFu;  // not reachable for inserted keys
    if (++h == cap) h = 0;
  }
}

// first[e] = first position of col[e] in [S^l ; col]; bit e of `bits` = that position is this very edge
__global__ __launch_bounds__(kBlock) void k_uniq_flag(const int32_t* __restrict__ col, int64_t m, const int64_t* __restrict__ m_dev,
                                                      int64_t n_dst, const unsigned long long* __restrict__ table, uint64_t cap,
                                                      uint32_t* __restrict__ first, uint64_t* __restrict__ bits) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (m_dev != nullptr && *m_dev < m) m = *m_dev;
  bool is_new = false;
  if (e < m) {
    const uint32_t f = first_position(table, cap, (uint32_t)col[e]);
    first[e] = f;
    is_new = (int64_t)f == n_dst + e;
  }
  const uint64_t b = ballot64(is_new);
  if (lane_id() == 0 && (e & ~(int64_t)63) < m) bits[e >> 6] = b;
}

// col_local and the tail of src_ids; the threads of the first n_dst positions also copy S^l to the front of src_ids
// (m_dev, optional: the exact number of edges, on the device; m is then the capacity of col.  The kernel may be
// launched before the host has seen the dedup's error and overflow flags, on a `first` that a failed dedup left
// partly unwritten: positions outside [0, n_dst + m) are skipped, so that every access stays inside the arrays whatever
// `first` holds; the caller discards the result in that case.)
__global__ __launch_bounds__(kBlock) void k_uniq_relabel(const int32_t* __restrict__ dst, const int32_t* __restrict__ col, int64_t m,
                                                         const int64_t* __restrict__ m_dev, int64_t n_dst,
                                                         const uint32_t* __restrict__ first, const uint64_t* __restrict__ bits,
                                                         TiledScan<uint32_t> word_rank, int32_t* __restrict__ src,
                                                         int32_t* __restrict__ col_local) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (m_dev != nullptr && *m_dev < m) m = *m_dev;
  if (e < n_dst) src[e] = dst[e];
  if (e >= m) return;
  const int64_t f = first[e];
  if (f >= n_dst + m) return;
  int64_t local = f;
  if (f >= n_dst) {
    const int64_t at = f - n_dst;  // the edge at which this vertex first appears
    const uint64_t below = bits[at >> 6] & ((1ull << (at & 63)) - 1ull);
    local = n_dst + word_rank.at(at >> 6) + __popcll(below);
    if (at == e) src[local] = col[e];
  }
  col_local[e] = (int32_t)local;
}

// ---- first positions by partition ------------------------------------------------------------------------------
// For long lists the table in HBM costs two dependent random accesses per entry (insert, then look-up), each an
// atomic or a miss of every cache.  The partitioned form touches HBM in streams only: the (key, position) pairs are
// distributed over buckets by the high bits of the key's hash (count, scan, scatter: the classic three-step
// partition, with a counter matrix [bucket][block] so that no atomic leaves a block and every pair has its place
// before it is moved), and a bucket, about kPartPairs pairs, is deduplicated by one block in a table in LDS.
// All occurrences of a key share a bucket, so the minimum position found there is the global first position.  The
// results are the same `first` and `bits` arrays that the table in HBM produces.
constexpr int kPartBlock = 1024;        // threads of a counting / scattering block
constexpr int kPartMaxBlocks = 512;     // blocks of those two kernels (two per compute unit)
constexpr int kPartPairs = 4096;        // mean pairs of a bucket
constexpr uint32_t kPartMaxBuckets = 8192;  // counters of a block in LDS: 32 KB
constexpr int kFirstBlock = 1024;       // threads of a bucket's block
constexpr uint32_t kPartSlots = 8192;   // slots of a bucket's table in LDS (64 KB): at most half full when every pair of a
                                        // mean bucket is distinct, a quarter or less with the usual share of repeats
constexpr uint32_t kPartFull = kPartSlots / 4 * 3;  // distinct keys at which a bucket gives up
static_assert(kPartFull + 1 + kFirstBlock < kPartSlots, "a probe must always reach an empty slot");

__device__ __forceinline__ uint32_t hash_of_key(uint32_t key) { return (uint32_t)(((uint64_t)key * 0x9E3779B97F4A7C15ull) >> 32); }
__device__ __forceinline__ uint32_t bucket_of_hash(uint32_t h, uint32_t n_buckets) { return (uint32_t)(((uint64_t)h * n_buckets) >> 32); }
// a bucket's hashes share their high bits: the table slot comes from the low ones, stirred
__device__ __forceinline__ uint32_t table_slot_of_hash(uint32_t h) {
  uint32_t x = h ^ (h >> 16);
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  return x & (kPartSlots - 1);
}

// The stretch of [S^l ; col] that block `block` of `n_blocks` counts and scatters.
__device__ __forceinline__ void part_stretch(int64_t n_all, uint32_t n_blocks, uint32_t block, int64_t* lo, int64_t* hi) {
  int64_t stretch = (n_all + n_blocks - 1) / n_blocks;
  stretch = (stretch + kPartBlock - 1) / kPartBlock * kPartBlock;
  *lo = (int64_t)block * stretch;
  *hi = *lo + stretch < n_all ? *lo + stretch : n_all;
  if (*lo > n_all) *lo = n_all;
}
// A bucket's pairs are laid out by column, one column per block.  Consecutive blocks run on different XCDs (round
// robin over 8), so the blocks of one XCD take neighbouring columns: a cache line of pairs is then put together in
// one XCD's L2.  (gridDim.x is a multiple of 8.)
__device__ __forceinline__ uint32_t part_column() { return (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3); }

// counts[b * gridDim.x + column] = pairs of this block's stretch that fall into bucket b
__global__ __launch_bounds__(kPartBlock) void k_part_count(const int32_t* __restrict__ dst, int64_t n_dst, const int32_t* __restrict__ col,
                                                           int64_t m, const int64_t* __restrict__ m_dev, uint32_t n_buckets,
                                                           uint32_t* __restrict__ counts) {
  extern __shared__ uint32_t tally[];  // [n_buckets]
  if (m_dev != nullptr && *m_dev < m) m = *m_dev;
  int64_t lo, hi;
  part_stretch(n_dst + m, gridDim.x, blockIdx.x, &lo, &hi);
  for (uint32_t b = threadIdx.x; b < n_buckets; b += kPartBlock) tally[b] = 0u;
  __syncthreads();
  constexpr int U = 4;  // independent loads in flight per thread
  for (int64_t base = lo + threadIdx.x; base < hi; base += (int64_t)U * kPartBlock) {
    uint32_t key[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = base + (int64_t)u * kPartBlock;
      key[u] = i < hi ? (uint32_t)(i < n_dst ? dst[i] : col[i - n_dst]) : 0u;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (base + (int64_t)u * kPartBlock < hi) atomicAdd(&tally[bucket_of_hash(hash_of_key(key[u]), n_buckets)], 1u);
  }
  __syncthreads();
  const uint32_t column = part_column();
  for (uint32_t b = threadIdx.x; b < n_buckets; b += kPartBlock) counts[(size_t)b * gridDim.x + column] = tally[b];
}

// The same stretch again: its pairs go to pairs[], bucket b's from place[b * gridDim.x + column] on (place = exclusive
// scan of counts).  A round of kTilePairs pairs is first ordered by bucket in LDS, so that the pairs of a round that
// share a bucket leave as one contiguous run written by neighbouring lanes, not as single 8-byte stores.
constexpr int kTilePairs = 8 * kPartBlock;
__global__ __launch_bounds__(kPartBlock) void k_part_scatter(const int32_t* __restrict__ dst, int64_t n_dst, const int32_t* __restrict__ col,
                                                             int64_t m, const int64_t* __restrict__ m_dev, uint32_t n_buckets,
                                                             TiledScan<uint32_t> place, unsigned long long* __restrict__ pairs) {
  __shared__ unsigned long long staged[kTilePairs];  // the round's pairs, by bucket
  extern __shared__ uint32_t cursor[];               // [n_buckets] next free place of the bucket's column
  uint32_t* off = cursor + n_buckets;                // [n_buckets] the round's tallies, then run starts
  __shared__ uint32_t wave_total[kPartBlock / kWave];
  if (m_dev != nullptr && *m_dev < m) m = *m_dev;
  int64_t lo, hi;
  part_stretch(n_dst + m, gridDim.x, blockIdx.x, &lo, &hi);
  const uint32_t column = part_column();
  for (uint32_t b = threadIdx.x; b < n_buckets; b += kPartBlock) cursor[b] = place.at((int64_t)b * gridDim.x + column);
  const uint32_t per = (n_buckets + kPartBlock - 1) / kPartBlock;  // tallies that a thread scans (at most 8)
  const int lane = lane_id(), wave = wave_in_block();
  for (int64_t tile = lo; tile < hi; tile += kTilePairs) {
    const uint32_t tile_n = (uint32_t)(hi - tile < kTilePairs ? hi - tile : kTilePairs);
    for (uint32_t b = threadIdx.x; b < n_buckets; b += kPartBlock) off[b] = 0u;
    __syncthreads();
    constexpr int U = kTilePairs / kPartBlock;
    uint32_t key[U], bucket[U], rank[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = tile + u * kPartBlock + threadIdx.x;
      key[u] = i < hi ? (uint32_t)(i < n_dst ? dst[i] : col[i - n_dst]) : 0u;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (tile + u * kPartBlock + threadIdx.x >= hi) continue;
      bucket[u] = bucket_of_hash(hash_of_key(key[u]), n_buckets);
      rank[u] = atomicAdd(&off[bucket[u]], 1u);
    }
    __syncthreads();
    {  // tallies -> run starts (exclusive scan over the buckets)
      uint32_t c[8], sum = 0;
#pragma unroll
      for (uint32_t q = 0; q < 8; ++q) {
        const uint32_t b = threadIdx.x * per + q;
        c[q] = q < per && b < n_buckets ? off[b] : 0u;
        sum += c[q];
      }
      uint32_t incl = sum;
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += o;
      }
      if (lane == kWave - 1) wave_total[wave] = incl;
      __syncthreads();
      uint32_t run = incl - sum;
      for (int w = 0; w < wave; ++w) run += wave_total[w];
#pragma unroll
      for (uint32_t q = 0; q < 8; ++q) {
        const uint32_t b = threadIdx.x * per + q;
        if (q < per && b < n_buckets) off[b] = run;
        run += c[q];
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = tile + u * kPartBlock + threadIdx.x;
      if (i < hi) staged[off[bucket[u]] + rank[u]] = ((unsigned long long)key[u] << 32) | (uint32_t)i;
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < tile_n; j += kPartBlock) {
      const unsigned long long pr = staged[j];
      const uint32_t b = bucket_of_hash(hash_of_key((uint32_t)(pr >> 32)), n_buckets);
      pairs[cursor[b] + (j - off[b])] = pr;
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < n_buckets; b += kPartBlock) cursor[b] += (b + 1 < n_buckets ? off[b + 1] : tile_n) - off[b];
    __syncthreads();
  }
}

// One bucket per block: first positions of the bucket's keys through a table in LDS, then first[] of the bucket's edges.
__global__ __launch_bounds__(kFirstBlock) void k_part_first(const unsigned long long* __restrict__ pairs, TiledScan<uint32_t> place,
                                                            uint32_t G, int64_t n_dst, int64_t n_all, uint32_t* __restrict__ first,
                                                            Ctl* ctl) {
  __shared__ unsigned long long table[kPartSlots];
  __shared__ uint32_t n_claimed, full;
  uint32_t lo = place.at((int64_t)blockIdx.x * G), hi = place.at((int64_t)(blockIdx.x + 1) * G);
  if ((int64_t)hi > n_all) hi = (uint32_t)n_all;  // (holds by construction; keeps every access inside the arrays regardless)
  if (lo > hi) lo = hi;
  for (uint32_t i = threadIdx.x; i < kPartSlots; i += kFirstBlock) table[i] = kEmptySlot;
  if (threadIdx.x == 0) { n_claimed = 0; full = 0; }
  __syncthreads();
  constexpr int U = 4;  // pairs per thread and round, loaded together
  unsigned long long first_round[U];  // the pairs of the first round, kept for the look-up phase
#pragma unroll
  for (int u = 0; u < U; ++u) first_round[u] = kEmptySlot;
  for (uint32_t base = lo; base < hi; base += U * kFirstBlock) {
    if (*(volatile uint32_t*)&full) break;
    unsigned long long mine[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = base + u * kFirstBlock + threadIdx.x;
      mine[u] = i < hi ? pairs[i] : kEmptySlot;
      if (base == lo) first_round[u] = mine[u];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (mine[u] == kEmptySlot || *(volatile uint32_t*)&full) continue;
      const uint32_t key = (uint32_t)(mine[u] >> 32);
      const bool seed_pos = (int64_t)(uint32_t)mine[u] < n_dst;
      uint32_t h = table_slot_of_hash(hash_of_key(key));
      for (;;) {  // ends: at most kPartFull + 1 + kFirstBlock < kPartSlots slots are ever claimed
        unsigned long long cur = *(volatile unsigned long long*)&table[h];
        if (cur == kEmptySlot) {
          cur = atomicCAS(&table[h], (unsigned long long)kEmptySlot, mine[u]);
          if (cur == kEmptySlot) {
            if (atomicAdd(&n_claimed, 1u) >= kPartFull) full = 1;
            break;
          }
        }
        if ((uint32_t)(cur >> 32) == key) {
          if (!seed_pos && cur < mine[u]) break;
          const unsigned long long old = atomicMin(&table[h], mine[u]);
          if (seed_pos && (int64_t)(uint32_t)old < n_dst) atomicOr(&ctl->err_dup, 1);  // S^l holds a vertex twice
          break;
        }
        h = (h + 1) & (kPartSlots - 1);
      }
    }
  }
  __syncthreads();
  if (full) {  // more distinct keys than the table serves: the caller falls back to the table in HBM
    if (threadIdx.x == 0) atomicOr(&ctl->uniq_overflow, 1);
    return;
  }
  const bool one_round = hi - lo <= (uint32_t)(U * kFirstBlock);  // (the usual bucket: its pairs are still in the registers)
  for (uint32_t base = lo; base < hi; base += U * kFirstBlock) {
    unsigned long long mine[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = base + u * kFirstBlock + threadIdx.x;
      mine[u] = one_round ? first_round[u] : (i < hi ? pairs[i] : kEmptySlot);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t pos = (uint32_t)mine[u];
      if (mine[u] == kEmptySlot || pos < n_dst || pos >= n_all) continue;
      const uint32_t key = (uint32_t)(mine[u] >> 32);
      uint32_t h = table_slot_of_hash(hash_of_key(key));
      unsigned long long cur;
      for (;;) {  // (every key of the bucket was inserted above; an empty slot ends the search regardless)
        cur = table[h];
        if ((uint32_t)(cur >> 32) == key || cur == kEmptySlot) break;
        h = (h + 1) & (kPartSlots - 1);
      }
      const int64_t e = pos - n_dst;
      first[e] = (uint32_t)cur;
    }
  }
}

// bit e of `bits` = edge e is the first occurrence of its vertex (its first position is its own)
__global__ __launch_bounds__(kBlock) void k_flag_from_first(const uint32_t* __restrict__ first, int64_t m, const int64_t* __restrict__ m_dev,
                                                            int64_t n_dst, uint64_t* __restrict__ bits) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (m_dev != nullptr && *m_dev < m) m = *m_dev;
  const bool is_new = e < m && (int64_t)first[e] == n_dst + e;
  const uint64_t b = ballot64(is_new);
  if (lane_id() == 0 && (e & ~(int64_t)63) < m) bits[e >> 6] = b;
}

__global__ void k_clear_uniq_overflow(Ctl* ctl) { ctl->uniq_overflow = 0; }

static inline unsigned nblocks(int64_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

int g_unique_mode = 0;  // COOP_TUNE_UNIQUE: 0 automatic, 1 table in HBM, 2 partition whenever it applies, 3 as 2 with buckets 16 times too large

// launches the dedup's kernels up to the scan that ranks the new vertices and sends the control block to the host
static int unique_launch(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, UniqueWork* w,
                         bool by_partition, Alloc& alloc, Ctl* d_ctl, Ctl* h_ctl, hipStream_t s) {
  const int64_t n_all = n_dst + m;
  const int64_t n_words = (m + 63) / 64;
  if (by_partition) {
    const int64_t n_buckets = w->n_buckets;
    const int64_t by_size = (n_all + 4 * kPartBlock - 1) / (4 * kPartBlock);
    const uint32_t G = (uint32_t)(by_size < kPartMaxBlocks ? (by_size + 7) / 8 * 8 : kPartMaxBlocks);  // a multiple of 8
    const int64_t n_counts = n_buckets * G;
    uint32_t* counts = alloc.get<uint32_t>(n_counts, COOP_TAG_SCRATCH);
    uint32_t* place = alloc.get<uint32_t>(n_counts + 1, COOP_TAG_SCRATCH);
    unsigned long long* pairs = alloc.get<unsigned long long>(n_all, COOP_TAG_SCRATCH);
    void* tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_counts), COOP_TAG_SCRATCH);
    if (alloc.failed) return COOP_E_NOMEM;
    const size_t lds = (size_t)n_buckets * sizeof(uint32_t);
    COOP_LAUNCH(K_PART_COUNT, k_part_count, dim3(G), dim3(kPartBlock), lds, s, dst, n_dst, col_global, m, m_dev, (uint32_t)n_buckets, counts);
    const TiledScan<uint32_t> places = scan_u32_tiled(counts, n_counts, place, tmp, &d_ctl->scan_done, s);
    COOP_LAUNCH(K_PART_SCATTER, k_part_scatter, dim3(G), dim3(kPartBlock), 2 * lds, s, dst, n_dst, col_global, m, m_dev, (uint32_t)n_buckets,
                places, pairs);
    COOP_LAUNCH(K_PART_FIRST, k_part_first, dim3((unsigned)n_buckets), dim3(kFirstBlock), 0, s, pairs, places, G, n_dst, n_all, w->first, d_ctl);
    if (hipGetLastError() != hipSuccess) return COOP_E_HIP;  // (a launch that did not happen would leave `first` unwritten)
    COOP_LAUNCH(K_UNIQ_FLAG, k_flag_from_first, dim3(nblocks(m)), dim3(kBlock), 0, s, w->first, m, m_dev, n_dst, w->bits);
  } else {
    // at most half full; an even number of slots (the clear uses 16-byte stores)
    const int64_t cap = 2 * n_all + 1024;
    unsigned long long* table = alloc.get<unsigned long long>(cap, COOP_TAG_SCRATCH);
    if (alloc.failed) return COOP_E_NOMEM;
    if (n_all > 0) {
      fill_u64((uint64_t*)table, cap, kEmptySlot, s);
      COOP_LAUNCH(K_UNIQ_INSERT, k_uniq_insert, dim3(nblocks(n_all)), dim3(kBlock), 0, s, dst, n_dst, col_global, m, m_dev, table, (uint64_t)cap,
                  d_ctl);
    }
    if (m > 0)
      COOP_LAUNCH(K_UNIQ_FLAG, k_uniq_flag, dim3(nblocks(m)), dim3(kBlock), 0, s, col_global, m, m_dev, n_dst, table, (uint64_t)cap, w->first,
                  w->bits);
  }
  // sizes (and the duplicate / range flags) back to the host, sent by the scan's last thread when there is a scan
  w->pub = begin_publish(d_ctl, h_ctl);
  if (m > 0) w->rank = scan_popc_tiled(w->bits, n_words, w->word_rank, &d_ctl->total_new, w->scan_tmp, &d_ctl->scan_done, s, &w->pub, m_dev);
  else if (launch_publish(w->pub, s) != COOP_OK) return COOP_E_HIP;
  w->by_partition = by_partition;
  return COOP_OK;
}

int unique_front_launch(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, UniqueWork* w,
                        Alloc& alloc, Ctl* d_ctl, Ctl* h_ctl, hipStream_t s) {
  const int64_t n_all = n_dst + m;
  w->first = alloc.get<uint32_t>(m, COOP_TAG_SCRATCH);
  const int64_t n_words = (m + 63) / 64;
  w->word_rank = alloc.get<uint32_t>(n_words + 1, COOP_TAG_SCRATCH);
  w->bits = alloc.get<uint64_t>(n_words, COOP_TAG_SCRATCH);
  w->scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_words), COOP_TAG_SCRATCH);
  if (alloc.failed) return COOP_E_NOMEM;
  // by partition from a few hundred thousand entries on (below that its five launches cost more than the table's
  // three), as long as a block's counters fit LDS
  const int64_t pairs_per_bucket = g_unique_mode == 3 ? 16 * kPartPairs : kPartPairs;
  w->n_buckets = (n_all + pairs_per_bucket - 1) / pairs_per_bucket;
  const bool by_partition = m > 0 && w->n_buckets <= kPartMaxBuckets && g_unique_mode != 1 && (g_unique_mode >= 2 || n_all >= 262144);
  return unique_launch(dst, n_dst, col_global, m, m_dev, w, by_partition, alloc, d_ctl, h_ctl, s);
}

int unique_front_finish(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, UniqueWork* w,
                        Alloc& alloc, Ctl* d_ctl, Ctl* h_ctl, hipStream_t s, bool* redone) {
  *redone = false;
  int rc = wait_ctl(w->pub, h_ctl, s);
  if (rc != COOP_OK) return rc;
  if (w->by_partition && h_ctl->uniq_overflow != 0) {  // a bucket's table overflowed: once more through the table in HBM
    hipLaunchKernelGGL(k_clear_uniq_overflow, dim3(1), dim3(1), 0, s, d_ctl);
    rc = unique_launch(dst, n_dst, col_global, m, m_dev, w, false, alloc, d_ctl, h_ctl, s);
    if (rc != COOP_OK) return rc;
    rc = wait_ctl(w->pub, h_ctl, s);
    if (rc != COOP_OK) return rc;
    *redone = true;
  }
  w->n_new = m > 0 ? h_ctl->total_new : 0;
  return COOP_OK;
}

int unique_back(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, const UniqueWork& w,
                int32_t* col_local, int32_t* src, hipStream_t s) {
  const int64_t n_threads = m > n_dst ? m : n_dst;
  if (n_threads > 0)
    COOP_LAUNCH(K_UNIQ_RELABEL, k_uniq_relabel, dim3(nblocks(n_threads)), dim3(kBlock), 0, s, dst, col_global, m, m_dev, n_dst, w.first, w.bits,
                w.rank, src, col_local);
  return COOP_OK;
}

}  // namespace coop
