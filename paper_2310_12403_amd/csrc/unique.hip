// Frontier dedup and relabelling (Eq. 2: S^{l+1} = S^l ∪ sampled sources) with an open-addressing hash table in HBM.
//
// The list [S^l ; col_global] is inserted into a table of 8-byte slots (key << 32 | position in that list).  A slot is
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
__global__ __launch_bounds__(kBlock) void k_uniq_relabel(const int32_t* __restrict__ dst, const int32_t* __restrict__ col, int64_t m,
                                                         int64_t n_dst, const uint32_t* __restrict__ first,
                                                         const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_rank,
                                                         int32_t* __restrict__ src, int32_t* __restrict__ col_local) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e < n_dst) src[e] = dst[e];
  if (e >= m) return;
  const int64_t f = first[e];
  int64_t local = f;
  if (f >= n_dst) {
    const int64_t at = f - n_dst;  // the edge at which this vertex first appears
    const uint64_t below = bits[at >> 6] & ((1ull << (at & 63)) - 1ull);
    local = n_dst + word_rank[at >> 6] + __popcll(below);
    if (at == e) src[local] = col[e];
  }
  col_local[e] = (int32_t)local;
}

static inline unsigned nblocks(int64_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

int unique_front(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const int64_t* m_dev, UniqueWork* w, Alloc& alloc,
                 Ctl* d_ctl, Ctl* h_ctl, hipStream_t s) {
  const int64_t n_all = n_dst + m;
  // at most half full; an even number of slots (the clear uses 16-byte stores)
  int64_t cap = 2 * n_all + 1024;

  unsigned long long* table = alloc.get<unsigned long long>(cap, COOP_TAG_SCRATCH);
  w->first = alloc.get<uint32_t>(m, COOP_TAG_SCRATCH);
  const int64_t n_words = (m + 63) / 64;
  w->word_rank = alloc.get<uint32_t>(n_words, COOP_TAG_SCRATCH);
  w->bits = alloc.get<uint64_t>(n_words, COOP_TAG_SCRATCH);
  void* scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_words), COOP_TAG_SCRATCH);
  if (alloc.failed) return COOP_E_NOMEM;

  if (n_all > 0) {
    fill_u64((uint64_t*)table, cap, kEmptySlot, s);
    COOP_LAUNCH(K_UNIQ_INSERT, k_uniq_insert, dim3(nblocks(n_all)), dim3(kBlock), 0, s, dst, n_dst, col_global, m, m_dev, table,
                (uint64_t)cap, d_ctl);
  }
  if (m > 0) {
    COOP_LAUNCH(K_UNIQ_FLAG, k_uniq_flag, dim3(nblocks(m)), dim3(kBlock), 0, s, col_global, m, m_dev, n_dst, table, (uint64_t)cap,
                w->first, w->bits);
  }
  // sizes (and the duplicate / range flags) back to the host, sent by the scan's last thread when there is a scan
  const Publish pub = begin_publish(d_ctl, h_ctl);
  if (m > 0) scan_popc_to_u32(w->bits, n_words, w->word_rank, &d_ctl->total_new, scan_tmp, s, &pub, m_dev);
  else if (launch_publish(pub, s) != COOP_OK) return COOP_E_HIP;
  const int rc = wait_ctl(pub, h_ctl, s);
  if (rc != COOP_OK) return rc;
  w->n_new = m > 0 ? h_ctl->total_new : 0;
  return COOP_OK;
}

int unique_back(const int32_t* dst, int64_t n_dst, const int32_t* col_global, int64_t m, const UniqueWork& w, int32_t* col_local,
                int32_t** src_out, int64_t* n_src_out, Alloc& alloc, hipStream_t s) {
  const int64_t n_src = n_dst + w.n_new;
  int32_t* src = alloc.get<int32_t>(n_src, COOP_TAG_OUTPUT);
  if (alloc.failed) return COOP_E_NOMEM;
  const int64_t n_threads = m > n_dst ? m : n_dst;
  if (n_threads > 0)
    COOP_LAUNCH(K_UNIQ_RELABEL, k_uniq_relabel, dim3(nblocks(n_threads)), dim3(kBlock), 0, s, dst, col_global, m, n_dst, w.first, w.bits,
                w.word_rank, src, col_local);
  *src_out = src;
  *n_src_out = n_src;
  return COOP_OK;
}

}  // namespace coop
