// LABOR-0 layers (App. A.1.2): edge (t -> s) is kept iff r_t <= k / d_s, i.e. R_t * d_s <= k * 2^32 in integers,
// which for d_s > k is R_t <= floor(k * 2^32 / d_s).  Kept edges leave in (destination order, adjacency order).
//
// Every neighbour list is read ONCE per minibatch.  S^l is a prefix of S^{l+1} (Eq. 2), so a vertex that becomes a
// destination at layer l is a destination at every later layer too, with the same list and a different key: the scan
// pass of layer l therefore covers only the vertices new at layer l and evaluates, for each neighbour, the keep tests
// of layers l .. L-1 at once (one mixer evaluation per layer, one read of the entry).  The kept (vertex, position)
// pairs are parked in small per-destination staging rows, one row set per covered layer; building layer l' later is
// a scan over the kept-edge counts and a copy of the rows.  A row that overflows is rare; those lists are scanned a
// second time, in order, straight into the edge arrays.
#include "device_utils.h"
#include "blend_filters.h"
#include "sample_internal.h"

namespace coop {

typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kAllThr = 0xFFFFFFFFu;  // threshold of a list no longer than the fanout: everything is kept
constexpr int kScanGroups = 4;             // 16-byte groups per lane and step of the fast scan (4 KiB per wave and step)

struct ScanOut {
  StageEntry* stage[kMaxFuse];
  int32_t* cnt[kMaxFuse];
};

struct FusedKeys {
  LayerKeys K[kMaxFuse];
  double cw, sw;
};

// The pieces of one layer's destinations, by the pass that scanned them.
struct LayerChunks {
  const Segment* seg[kMaxFuse];
  const uint32_t* thr[kMaxFuse];
  const StageEntry* stage[kMaxFuse];
  int64_t start[kMaxFuse];
  int n_chunks;
  __device__ __forceinline__ int find(int64_t w) const {
    int p = 0;
#pragma unroll
    for (int q = 1; q < kMaxFuse; ++q)
      if (q < n_chunks && w >= start[q]) p = q;
    return p;
  }
};

// ---- LABOR-0 from the other side (c = 0, symmetric graph) ----------------------------------------------------------
// R_t = mix(t ^ K0) ^ K1 is a bijection of the 32-bit integers, so the vertices with R_t <= u_max can be listed without
// looking at the graph: t = unmix(u ^ K1) ^ K0 for u = 0 .. u_max, kept if t < |V|.  A destination s with a list longer
// than D keeps exactly the neighbours with R_t <= floor(k 2^32 / d_s) < k 2^32 / D: all of them are among the
// |V| k / D vertices listed for u_max = floor(k 2^32 / (D + 1)).  On a symmetric graph "t is a neighbour of s" can be
// decided from t's side: the kernel walks the (mostly short) lists of the listed vertices, looks every entry s up in the
// table of long destinations, and where R_t is within that destination's threshold it has found a kept edge, whose
// position in the destination's own list comes from the graph handle's index of reverse positions.  The long lists,
// most of the entries that a scan would have to read, are never read.
__device__ __forceinline__ uint32_t long_slot(uint32_t s) { return (uint32_t)(((uint64_t)s * 0x9E3779B97F4A7C15ull) >> 32); }
// a slot of the table of long destinations: key = vertex + 1 (0: empty), its list index, its thresholds; one 32-byte
// sector.  Open addressing, and no key lies further than kLongProbes slots from its home: a table too full for that
// makes the pass fall back to the ordinary scan.
struct alignas(32) LongSlot { uint32_t key, list, thr[kMaxFuse], pad[2]; };
constexpr uint32_t kLongProbes = 64;
// In front of the table, a bit per hash value says whether any long destination has it: the walk keeps these bits in
// LDS, and goes to the table (in L2) only for the entries that pass, the long destinations' own and a few per cent more.
constexpr uint32_t kLongBits = 1u << 18;  // 32 KB
constexpr int kWalkBlock = 512;           // three blocks per CU, each with the bits in LDS
__device__ __forceinline__ uint32_t long_bit(uint32_t s) { return long_slot(s) >> 14; }

struct EnumItem { int64_t beg; uint32_t len, t, u, pad; };  // up to kEnumItem entries of listed vertex t's list; u = R_t
constexpr uint32_t kEnumItem = 64;         // entries per item: 16 lanes walk it, 4 entries each, loaded together
constexpr int kListBlock = 256;            // threads per block of k_enum_list
constexpr uint32_t kEnumListSpan = 8192;   // variates per block of k_enum_list
constexpr uint32_t kEnumListStep = 1024;   // variates per step of a block (4 per thread), between two barriers
constexpr uint32_t kEnumListBuf = 2048;    // vertices a block collects before it writes their items out

struct EnumOut {
  EnumItem* item[kMaxFuse];    // [item_cap[f]] per covered layer
  uint32_t* n_item[kMaxFuse];  // one counter each
  uint32_t item_cap[kMaxFuse];
};

// blockIdx.y = covered layer f: lists the vertices with R_t <= u_max[f].  A block takes kEnumListSpan consecutive
// variates, collects the vertices they belong to in LDS, fetches their list bounds, and writes their lists, cut into
// items, to the layer's item list: one reservation (a same-address atomic) per flush (one in 40 of the variates of a
// papers100M-sized graph gives a vertex).
__global__ __launch_bounds__(kListBlock) void k_enum_list(FusedKeys keys, uint32_t um0, uint32_t um1, uint32_t um2, uint32_t um3,
                                                      int64_t n_vertices, const int64_t* __restrict__ g_indptr, EnumOut eo, Ctl* ctl,
                                                      uint32_t todo /* bit f: layer f is to be listed (the others have their lists) */) {
  __shared__ uint2 buf[kEnumListBuf];     // (t, u)
  __shared__ uint32_t s_d[kEnumListBuf], s_at[kEnumListBuf];
  __shared__ uint16_t s_long[kEnumListBuf];  // the collected vertices that give more than one item
  __shared__ uint32_t n_buf, n_local, n_long, base;
  const int f = blockIdx.y;
  const uint32_t u_max = f == 0 ? um0 : f == 1 ? um1 : f == 2 ? um2 : um3;
  const uint32_t K0 = keys.K[f].Ka[0], K1 = keys.K[f].Ka[1];
  const uint64_t first = (uint64_t)blockIdx.x * kEnumListSpan;
  if (first > u_max || ((todo >> f) & 1u) == 0) return;  // block-uniform
  EnumItem* __restrict__ item_f = f == 0 ? eo.item[0] : f == 1 ? eo.item[1] : f == 2 ? eo.item[2] : eo.item[3];
  uint32_t* n_item_f = f == 0 ? eo.n_item[0] : f == 1 ? eo.n_item[1] : f == 2 ? eo.n_item[2] : eo.n_item[3];
  const uint32_t item_cap_f = f == 0 ? eo.item_cap[0] : f == 1 ? eo.item_cap[1] : f == 2 ? eo.item_cap[2] : eo.item_cap[3];
  if (threadIdx.x == 0) { n_buf = 0; n_local = 0; n_long = 0; }
  __syncthreads();
  auto flush = [&]() {  // block-uniform call, after a barrier
    const uint32_t nb = n_buf;  // <= kEnumListBuf: a step adds at most kEnumListStep and is taken only when that many fit
    for (uint32_t i = threadIdx.x; i < nb; i += kListBlock) {
      const uint32_t t = buf[i].x;
      const int64_t beg = g_indptr[t];
      const uint32_t d = (uint32_t)(g_indptr[t + 1] - beg);  // (0: a vertex without neighbours is nobody's neighbour)
      s_d[i] = d;
      if (d != 0) s_at[i] = atomicAdd(&n_local, (d + kEnumItem - 1) / kEnumItem);
      if (d > kEnumItem) s_long[atomicAdd(&n_long, 1u)] = (uint16_t)i;
    }
    __syncthreads();
    if (threadIdx.x == 0) base = n_local ? atomicAdd(n_item_f, n_local) : 0u;
    __syncthreads();
    if (base + n_local > item_cap_f) {
      if (threadIdx.x == 0) atomicOr(&ctl->cand_overflow, 1);  // (the pass is redone without this shortcut)
    } else {
      for (uint32_t i = threadIdx.x; i < nb; i += kListBlock) {  // a thread per vertex with one item
        const uint32_t d = s_d[i];
        if (d != 0 && d <= kEnumItem) item_f[base + s_at[i]] = EnumItem{g_indptr[buf[i].x], d, buf[i].x, buf[i].y, 0u};
      }
      for (uint32_t v = 0; v < n_long; ++v) {                // the block together for each of the others
        const uint32_t i = s_long[v];
        const uint32_t d = s_d[i];
        const uint2 tu = buf[i];
        const int64_t beg = g_indptr[tu.x];
        EnumItem* to = item_f + base + s_at[i];
        for (uint32_t q = threadIdx.x; q * kEnumItem < d; q += kListBlock) {
          const uint32_t off = q * kEnumItem;
          to[q] = EnumItem{beg + off, d - off < kEnumItem ? d - off : kEnumItem, tu.x, tu.y, 0u};
        }
      }
    }
    __syncthreads();
    if (threadIdx.x == 0) { n_buf = 0; n_local = 0; n_long = 0; }
    __syncthreads();
  };
  for (uint32_t step = 0; step < kEnumListSpan; step += kEnumListStep) {
#pragma unroll
    for (uint32_t q = 0; q < kEnumListStep; q += kListBlock) {
      const uint64_t u = first + step + q + threadIdx.x;
      const uint32_t t = unmix32((uint32_t)u ^ K1) ^ K0;
      if (u <= u_max && (uint64_t)t < (uint64_t)n_vertices) buf[atomicAdd(&n_buf, 1u)] = make_uint2(t, (uint32_t)u);
    }
    __syncthreads();
    const bool nearly_full = n_buf > kEnumListBuf - kEnumListStep;  // read by everyone before anyone adds again
    __syncthreads();
    if (nearly_full) flush();
  }
  flush();
}

// blockIdx.y = covered layer f: 16 lanes per item; a lane's four entries are requested together, and so are the table
// slots of those that pass the bit test.
// A kept edge costs a chain of three dependent memory operations (its reverse position, a returning atomic on its
// destination's counter, the store into the staging row), and a step of 256 entries finds only a handful: committed on
// the spot they would make the wave wait out that chain in every step with a few lanes at work.  So the kept edges of a
// wave wait in a queue in LDS and are committed 64 at a time, every lane with a chain of its own, and once more when the
// wave is through its items.
struct WalkQueue {
  uint32_t n;  // entries waiting (below 128; the same for every lane of the wave)
  uint32_t list[2 * kWave];
  int32_t t[2 * kWave];
  uint32_t pos_lo[2 * kWave], pos_hi[2 * kWave];  // position of the entry in the graph's indices
};
__global__ __launch_bounds__(kWalkBlock, 6) void k_enum_walk(const int32_t* __restrict__ g_indices, const uint32_t* __restrict__ rev_pos,
                                                          const uint32_t* __restrict__ long_bits, const LongSlot* __restrict__ long_tab,
                                                          uint32_t long_mask, uint32_t stage_cap, ScanOut out, EnumOut eo, Ctl* ctl) {
  __shared__ uint32_t bits[kLongBits / 32];
  __shared__ WalkQueue queues[kWalkBlock / kWave];
  const int f = blockIdx.y;
  if (ctl->cand_overflow != 0) return;  // (some items were not written, or some destinations not entered: the pass is redone)
  WalkQueue& wq = queues[threadIdx.x / kWave];
  if ((threadIdx.x & (kWave - 1)) == 0) wq.n = 0;
  for (uint32_t i = threadIdx.x; i < kLongBits / 128; i += kWalkBlock)
    reinterpret_cast<uint4*>(bits)[i] = reinterpret_cast<const uint4*>(long_bits)[i];
  __syncthreads();
  uint32_t total = *(f == 0 ? eo.n_item[0] : f == 1 ? eo.n_item[1] : f == 2 ? eo.n_item[2] : eo.n_item[3]);
  const uint32_t item_cap_f = f == 0 ? eo.item_cap[0] : f == 1 ? eo.item_cap[1] : f == 2 ? eo.item_cap[2] : eo.item_cap[3];
  if (total > item_cap_f) total = item_cap_f;
  const EnumItem* __restrict__ item_f = f == 0 ? eo.item[0] : f == 1 ? eo.item[1] : f == 2 ? eo.item[2] : eo.item[3];
  int32_t* __restrict__ cnt_f = f == 0 ? out.cnt[0] : f == 1 ? out.cnt[1] : f == 2 ? out.cnt[2] : out.cnt[3];
  StageEntry* __restrict__ stage_f = f == 0 ? out.stage[0] : f == 1 ? out.stage[1] : f == 2 ? out.stage[2] : out.stage[3];
  const uint32_t sub = threadIdx.x & 15u;
  const uint32_t groups = (gridDim.x * kWalkBlock) >> 4;
  // The first `n` queued edges (n <= 64), shared out among the lanes that are still here (the 16-lane groups of a wave
  // run out of items at different times): reverse position, place in the row, store.
  auto commit = [&](uint32_t n) {
    const uint64_t here = ballot64(true);
    const uint32_t n_here = (uint32_t)__popcll(here);
    for (uint32_t i = lanes_below(here); i < n; i += n_here) {
      const uint32_t list = wq.list[i];
      const uint32_t j = rev_pos[((uint64_t)wq.pos_hi[i] << 32) | wq.pos_lo[i]];
      const uint32_t at = (uint32_t)atomicAdd(&cnt_f[list], 1);
      if (at < stage_cap) stage_f[(size_t)list * stage_cap + at] = StageEntry{wq.t[i], j};
      else if (at == stage_cap) atomicAdd(&ctl->n_overflow, 1);  // exactly one entry sees the row fill up
    }
  };
  // (two items ahead: while the table slots of the current item are in flight, so are the entries of the next one and the
  // record of the one after it)
  uint32_t c = (blockIdx.x * kWalkBlock + threadIdx.x) >> 4;
  if (c >= total) return;
  EnumItem it = item_f[c];
  EnumItem it_next = it;
  if (c + groups < total) it_next = item_f[c + groups];
  uint32_t s4[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t j = (uint32_t)e * 16u + sub;
    s4[e] = (uint32_t)g_indices[it.beg + (j < it.len ? j : it.len - 1)];  // (len >= 1; a lane past the end repeats the last entry)
  }
  for (;;) {
    const bool more = c + groups < total;
    uint32_t h4[4];
    bool maybe[4];
    uint4 head4[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t b = long_bit(s4[e]);
      maybe[e] = (uint32_t)e * 16u + sub < it.len && ((bits[b >> 5] >> (b & 31u)) & 1u) != 0;
      h4[e] = long_slot(s4[e]) & long_mask;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (maybe[e]) head4[e] = *reinterpret_cast<const uint4*>(&long_tab[h4[e]]);
    // The requests for the next rounds go out behind the table slots, not in front of them: loads come back in the
    // order in which they were sent, and the slots (in L2) must not wait for these (in HBM).
    asm volatile("" ::: "memory");
    EnumItem it_next2 = it_next;
    if ((uint64_t)c + 2ull * groups < total) it_next2 = item_f[c + 2u * groups];
    uint32_t s4_next[4] = {0, 0, 0, 0};
    if (more) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t j = (uint32_t)e * 16u + sub;
        s4_next[e] = (uint32_t)g_indices[it_next.beg + (j < it_next.len ? j : it_next.len - 1)];
      }
    }
    asm volatile("" ::: "memory");
    // Which entries are long destinations of this pass (the key in a slot is the vertex + 1, 0 an empty slot), and is
    // R_t within their threshold?  An entry whose home slot holds another key moves on to the next slot; the entries
    // of a lane do so together, a round of requests at a time.
    uint32_t list4[4];
    bool open4[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) open4[e] = maybe[e];
    for (uint32_t probe = 1;; ++probe) {
      bool again = false;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (open4[e]) {
          if (head4[e].x == s4[e] + 1) {
            open4[e] = false;
            list4[e] = head4[e].y;
            maybe[e] = it.u <= (f == 0 ? head4[e].z : f == 1 ? head4[e].w : long_tab[h4[e]].thr[f]);
          } else if (head4[e].x == 0 || probe >= kLongProbes) {
            open4[e] = false;
            maybe[e] = false;
          } else {
            h4[e] = (h4[e] + 1) & long_mask;
            again = true;
          }
        }
      if (!again) break;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (open4[e]) head4[e] = *reinterpret_cast<const uint4*>(&long_tab[h4[e]]);
    }
    // kept edges t -> s join the wave's queue; a full wave of them is committed at once
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint64_t mask = ballot64(maybe[e]);
      if (mask == 0) continue;
      uint32_t nq = wq.n;  // (below 64 here)
      if (maybe[e]) {
        const uint32_t at = nq + lanes_below(mask);
        const uint64_t pos = (uint64_t)it.beg + (uint32_t)e * 16u + sub;
        wq.list[at] = list4[e];
        wq.t[at] = (int32_t)it.t;
        wq.pos_lo[at] = (uint32_t)pos;
        wq.pos_hi[at] = (uint32_t)(pos >> 32);
      }
      nq += (uint32_t)__popcll(mask);
      __builtin_amdgcn_wave_barrier();
      if (nq >= (uint32_t)kWave) {
        commit(kWave);
        __builtin_amdgcn_wave_barrier();
        const uint32_t rest = nq - kWave;  // fewer than 64: to the front
        const uint64_t here = ballot64(true);
        const uint32_t n_here = (uint32_t)__popcll(here);
        // (in rounds of the lanes that are here, each round read before it is written: a round only writes below what it read)
        for (uint32_t first = 0; first < rest; first += n_here) {
          const uint32_t i = first + lanes_below(here);
          uint32_t ml = 0, mlo = 0, mhi = 0;
          int32_t mt = 0;
          if (i < rest) { ml = wq.list[kWave + i]; mt = wq.t[kWave + i]; mlo = wq.pos_lo[kWave + i]; mhi = wq.pos_hi[kWave + i]; }
          __builtin_amdgcn_wave_barrier();
          if (i < rest) { wq.list[i] = ml; wq.t[i] = mt; wq.pos_lo[i] = mlo; wq.pos_hi[i] = mhi; }
          __builtin_amdgcn_wave_barrier();
        }
        nq = rest;
      }
      if (lanes_below(ballot64(true)) == 0) wq.n = nq;
      __builtin_amdgcn_wave_barrier();
    }
    if (!more) break;
    c += groups;
    it = it_next;
    it_next = it_next2;
#pragma unroll
    for (int e = 0; e < 4; ++e) s4[e] = s4_next[e];
  }
  // what still waits, fewer than 64 (every lane that had an item arrives here, whenever its group ran out)
  __builtin_amdgcn_wave_barrier();
  commit(wq.n);
}

// list records of the destinations scanned in this pass, and their keep thresholds for the nf covered layers
// (pthr, lim2: the blended path's first and second filter thresholds, null when c = 0)
constexpr int kSegBlock = 1024;  // large blocks: one queue reservation (a same-address atomic) per 1024 destinations
__global__ __launch_bounds__(kSegBlock) void k_segments(const int64_t* __restrict__ g_indptr, int64_t n_vertices,
                                                     const int32_t* __restrict__ dst, int64_t n, int nf,
                                                     uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3, Segment* __restrict__ seg,
                                                     uint32_t* __restrict__ thr, PreThr* __restrict__ pthr, float* __restrict__ lim2,
                                                     double cw, double sw, int queued, Ctl* ctl,
                                                     uint32_t piece_len, uint32_t split_min, Piece* __restrict__ pieces, uint32_t piece_cap,
                                                     uint32_t* __restrict__ piece_count, ScanOut out, uint32_t enum_degree,
                                                     uint32_t* __restrict__ long_bits, LongSlot* __restrict__ long_tab, uint32_t long_mask) {
  __shared__ uint32_t s_wave_at[kSegBlock / kWave];
  __shared__ uint32_t s_base, s_total;
  const int64_t i = (int64_t)blockIdx.x * kSegBlock + threadIdx.x;
  const bool live = i < n;
  Segment g{0, 0, 0};
  bool sampled = live;  // every covered layer keeps a proper subset (d > k)
  uint32_t thr_mine[kMaxFuse] = {0, 0, 0, 0};
  if (live) {
    const int32_t s = dst[i];
    if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
      atomicOr(&ctl->err_range, 1);
    } else {
      g.beg = g_indptr[s];
      g.d = (uint32_t)(g_indptr[s + 1] - g.beg);
    }
    const uint32_t ks[kMaxFuse] = {k0, k1, k2, k3};
#pragma unroll
    for (int f = 0; f < kMaxFuse; ++f)
      if (f < nf) {
        const uint32_t t = g.d > ks[f] ? (uint32_t)(((uint64_t)ks[f] << 32) / (uint64_t)g.d) : kAllThr;
        sampled &= t != kAllThr;
        thr[(int64_t)f * n + i] = t;
        thr_mine[f] = t;
        if (pthr) {
          PreThr pt = blend_first_thresholds(t, cw, sw);
          pt.keep2 = blend_keep_threshold(t, cw + sw);
          pthr[(int64_t)f * n + i] = pt;
          lim2[(int64_t)f * n + i] = blend_second_threshold(t, cw + sw);
        }
        if (queued) out.cnt[f][i] = 0;  // kept edges are counted by atomics
      }
  }
  // A list longer than enum_degree (when that is not 0) is not scanned at all: its kept neighbours are found from the
  // other side (k_enum_*).  The destination is entered in the table that maps such vertices to their list.
  const bool from_other_side = enum_degree != 0 && sampled && g.d > enum_degree;
  if (from_other_side) {
    g.split = 1;  // (the scan leaves it alone, like a list cut into pieces)
#pragma unroll
    for (int f = 0; f < kMaxFuse; ++f)
      if (f < nf) out.cnt[f][i] = 0;  // kept edges are counted by atomics
    const unsigned long long mine = ((unsigned long long)(uint32_t)i << 32) | ((uint32_t)dst[i] + 1u);  // (key, list)
    uint32_t h = long_slot((uint32_t)dst[i]) & long_mask;
    bool entered = false;
    for (uint32_t probe = 0; probe < kLongProbes && !entered; ++probe) {
      if (atomicCAS(reinterpret_cast<unsigned long long*>(&long_tab[h]), 0ull, mine) == 0ull) {
        entered = true;
#pragma unroll
        for (int f = 0; f < kMaxFuse; ++f)
          if (f < nf) long_tab[h].thr[f] = thr_mine[f];
      }
      h = (h + 1) & long_mask;
    }
    if (!entered) atomicOr(&ctl->cand_overflow, 1);  // (the pass is redone without this shortcut)
    const uint32_t b = long_bit((uint32_t)dst[i]);
    atomicOr(&long_bits[b >> 5], 1u << (b & 31u));
    sampled = false;  // no pieces
  }
  if (piece_len == 0) {  // wave-uniform
    if (live) seg[i] = g;
    return;
  }
  // A long list is cut into pieces of about piece_len entries (equal lengths, multiples of 4), each scanned by a wave
  // of its own: the waves of the scan then all have about the same amount of work whatever the degree distribution.
  // The block reserves queue slots for all its long lists with one atomic; each wave then writes its pieces together.
  uint32_t np = sampled && g.d > split_min ? (g.d + piece_len - 1) / piece_len : 0u;
  if (np > (1u << 20)) np = 0;  // keeps the block's sum below 2^30 (only lists of 2^28 entries and more, at the smallest piece length)
  const uint32_t incl = wave_incl_scan(np);
  const uint32_t lane = (uint32_t)lane_id();
  const int wv = uniform_wave_in_block();
  if (lane == kWave - 1) s_wave_at[wv] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t sum = 0;
    for (int q = 0; q < kSegBlock / kWave; ++q) { const uint32_t t = s_wave_at[q]; s_wave_at[q] = sum; sum += t; }
    s_total = sum;
    s_base = sum != 0 ? atomicAdd(piece_count, sum) : 0u;
  }
  __syncthreads();
  const uint32_t total = s_total;
  if (total != 0) {  // block-uniform
    const uint32_t block_base = s_base;
    // room always suffices for distinct destinations (the queue holds a piece for every piece_len edges of the graph);
    // a seed list with duplicates may run out: its lists then stay whole and what was reserved becomes empty slots
    const bool fits = block_base <= piece_cap && total <= piece_cap - block_base;
    const uint32_t base = block_base + s_wave_at[wv];
    uint64_t todo = ballot64(np != 0);
    while (todo != 0) {
      const int src = __builtin_ctzll(todo);
      todo &= todo - 1;
      const uint32_t np_s = (uint32_t)__builtin_amdgcn_readlane((int)np, src);
      const uint32_t at = base + (uint32_t)__builtin_amdgcn_readlane((int)incl, src) - np_s;
      const uint32_t list = (uint32_t)((int64_t)blockIdx.x * kSegBlock + (threadIdx.x & ~(kWave - 1)) + src);
      for (uint32_t q = lane; q < np_s; q += kWave)
        if (at + q < piece_cap) pieces[at + q] = fits ? Piece{list, q} : Piece{kNoPiece, 0u};
    }
    if (fits && np != 0) {
      g.split = 1;
#pragma unroll
      for (int f = 0; f < kMaxFuse; ++f)
        if (f < nf) out.cnt[f][i] = 0;  // the pieces add their counts
    }
  }
  if (live) seg[i] = g;
}

// Ordered visit of the neighbour list [beg, beg + d) of one destination by the whole wave, one entry per lane and
// step: calls emit(rank, t, j) for every kept neighbour t at list position j, rank counting kept neighbours in
// adjacency order.  Returns the number kept (same value in every lane).  Used for short lists, for an indices array
// that is not 16-byte aligned, and for the overflow pass.
template <bool BLEND, typename Emit>
__device__ __forceinline__ uint32_t labor_scan_ordered(const int32_t* __restrict__ g_indices, int64_t beg, uint32_t d, uint32_t thr,
                                                       const LayerKeys& K, double cw, double sw, Emit emit) {
  const int lane = lane_id();
  const bool all = thr == kAllThr;
  uint32_t count = 0;
  for (uint32_t base = 0; base < d; base += kWave) {
    const uint32_t j = base + lane;
    bool kp = j < d;
    int32_t t = 0;
    if (kp) {
      t = g_indices[beg + j];
      if (!all) kp = variate<false, BLEND>(K, cw, sw, (uint32_t)t, 0u, 0u) <= thr;
    }
    const uint64_t m = ballot64(kp);
    if (kp) emit(count + lanes_below(m), t, j);
    count += (uint32_t)__popcll(m);
  }
  return count;
}

// Kept entries of one list and one layer, parked in registers: lane q holds the q-th kept entry.
struct KeptRegs {
  int32_t ent_t = 0, ent_j = 0;
  uint32_t count = 0;  // wave-uniform
  __device__ __forceinline__ void push(uint32_t lane, int32_t t, int32_t j) {
    if (lane == (count & 63u)) { ent_t = t; ent_j = j; }
    ++count;
  }
};

// Where the fast scan puts the kept entries of a list.  take(l, mm, f, t, j): in this wave step the lanes of mask mm
// (f = this lane is one of them) keep entry t at list position j for layer l.
//
// RegSink parks them in registers, one entry per lane (for the pieces of a cut list: a piece learns its place in the
// destination's staging row only when it knows how many entries it keeps).
template <int NF>
struct RegSink {
  KeptRegs kept[NF];
  __device__ __forceinline__ void take(int l, uint64_t mm, bool, int32_t t, int32_t j, uint32_t lane) {
    while (mm != 0) {
      const int src_lane = __builtin_ctzll(mm);
      mm &= mm - 1;
      kept[l].push(lane, __builtin_amdgcn_readlane(t, src_lane), __builtin_amdgcn_readlane(j, src_lane));
    }
  }
};
// RowSink writes them straight to the destination's staging row, each lane its own entry at the next free slots
// (running count plus the lane's rank in the mask): no loop over the entries, and no particular order in the row
// (the fill pass ranks such rows by list position).  Entries beyond the row's capacity are counted, not stored.
template <int NF>
struct RowSink {
  StageEntry* row[NF];
  uint32_t count[NF];  // wave-uniform
  uint32_t cap;
  __device__ __forceinline__ void take(int l, uint64_t mm, bool f, int32_t t, int32_t j, uint32_t) {
    const uint32_t slot = count[l] + lanes_below(mm);
    if (f && slot < cap) row[l][slot] = StageEntry{t, (uint32_t)j};
    count[l] += (uint32_t)__popcll(mm);
  }
};

// Fast scan of a long list (d > 64) for NF layers at once.  The list is read as 16-byte aligned groups of four
// entries, kScanGroups groups per lane and step, all requested before the first is hashed.  Only groups that lie
// wholly inside the list go through the main loop, so validity is one compare per group, not per entry; the up to
// three entries in front of the first whole group and behind the last one are handled by one extra step.  Per entry
// and layer the hot loop is the mixer and one compare; one ballot per group tells whether any lane kept anything for
// any layer.  Only then are the (few) kept entries picked off per-entry ballot masks by a wave-uniform loop and
// parked in registers, in no particular order (they are ranked when the list is done).
template <bool BLEND, int NF, typename Sink>
__device__ __forceinline__ void labor_scan_fast(const int32_t* __restrict__ g_indices, int64_t beg, uint32_t d, uint32_t j0,
                                                const uint32_t (&thr)[NF], const FusedKeys& keys, Sink& sink) {
  constexpr uint32_t kStep = kWave * 4 * kScanGroups;
  const int64_t abeg = beg & ~(int64_t)3;        // first aligned group
  const uint32_t head = (uint32_t)(beg - abeg);  // entries of that group that precede the list
  const uint32_t total = head + d;               // list end, relative to abeg
  const uint32_t vec_end = total & ~3u;          // whole groups end here
  const uint32_t vec_beg = head ? 4u : 0u;       // whole groups start here
  const int32_t* __restrict__ p = g_indices + abeg;
  const uint32_t lane = (uint32_t)lane_id();
  const int32_t j_lane = (int32_t)(lane * 4 + j0) - (int32_t)head;  // list position of this lane's first entry at r0 = 0

  // The loads of the next step are issued before this step's entries are hashed.  A lane whose group lies behind the
  // list loads the last whole group instead (in bounds, and cheaper than switching lanes off); `ok` discards it.
  i32x4 nbuf[kScanGroups];
  auto fetch = [&](uint32_t at) {
#pragma unroll
    for (int gq = 0; gq < kScanGroups; ++gq) {
      if (at + (uint32_t)(gq * kWave * 4) >= vec_end) break;  // wave-uniform: the whole slot lies behind the list
      uint32_t r = at + (uint32_t)(gq * kWave * 4) + lane * 4;
      r = r < vec_end - 4 ? r : vec_end - 4;
      nbuf[gq] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(p + r));
    }
  };
#pragma unroll
  for (int gq = 0; gq < kScanGroups; ++gq) nbuf[gq] = i32x4{0, 0, 0, 0};
  if (vec_beg < vec_end) fetch(vec_beg);
  // The ragged ends (lanes 0..2: the entries in front of the first whole group; lanes 3..5: those behind the last one)
  // are requested right behind the first step, not when the whole groups are done: a list of one or two steps, and
  // most lists are, then waits for memory once, not twice.
  const uint32_t end_pos = lane < 3 ? head + lane : vec_end + (lane - 3);
  const bool end_valid = lane < 3 ? (head != 0 && end_pos < 4 && end_pos < total) : (lane < 6 && end_pos < total && vec_end >= vec_beg);
  int32_t end_t = 0;
  if (end_valid) end_t = p[end_pos];
  for (uint32_t base = vec_beg; base < vec_end; base += kStep) {
    i32x4 buf[kScanGroups];
    bool ok[kScanGroups];
#pragma unroll
    for (int gq = 0; gq < kScanGroups; ++gq) {
      buf[gq] = nbuf[gq];
      ok[gq] = base + (uint32_t)(gq * kWave * 4) + lane * 4 < vec_end;
    }
    if (base + kStep < vec_end) fetch(base + kStep);
#pragma unroll
    for (int gq = 0; gq < kScanGroups; ++gq) {
      const uint32_t r0 = base + (uint32_t)(gq * kWave * 4);  // wave-uniform
      if (r0 >= vec_end) break;                                // the rest of this step lies behind the list
      bool f[NF][4];
      bool any = false;
#pragma unroll
      for (int l = 0; l < NF; ++l) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          f[l][e] = ok[gq] & (variate<false, BLEND>(keys.K[l], keys.cw, keys.sw, (uint32_t)buf[gq][e], 0u, 0u) <= thr[l]);
          any |= f[l][e];
        }
      }
      if (ballot64(any) != 0) {
#pragma unroll
        for (int l = 0; l < NF; ++l) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint64_t mm = ballot64(f[l][e]);
            if (mm != 0) sink.take(l, mm, f[l][e], buf[gq][e], j_lane + (int32_t)(r0 + e), lane);
          }
        }
      }
    }
  }
#pragma unroll
  for (int l = 0; l < NF; ++l) {  // the ragged ends
    const bool fl = end_valid && variate<false, BLEND>(keys.K[l], keys.cw, keys.sw, (uint32_t)end_t, 0u, 0u) <= thr[l];
    const uint64_t mm = ballot64(fl);
    if (mm != 0) sink.take(l, mm, fl, end_t, (int32_t)(end_pos - head + j0), lane);
  }
}

// ---- blended variates (c > 0) -------------------------------------------------------------------------------------
// The exact blend (two Phi^-1 and a Phi in binary64) costs about a hundred times the integer path and needs four
// times the registers of the traversal, so it is reached in three stages:
//   1. integer bounds on min(U1, U2) and max(U1, U2) (per list and layer; in the traversal loop);
//   2. the blend in fp32, for a full wave of stage-1 passers at a time, taken from a per-wave queue in LDS that lives
//      across the wave's lists: an estimate safely above the keep threshold is dropped, one safely below is a kept
//      edge, and only the narrow band in between (a few percent of the kept edges) is left undecided;
//   3. the exact blend for the undecided, in a kernel of its own (k_labor_exact) over a buffer in device memory that
//      the scan kernel appended them to: the scan kernel keeps the occupancy of a streaming kernel, the exact stage
//      runs with every lane busy.
// A kept edge takes the next free slot of its destination's staging row with an atomic on the row's counter; rows
// filled this way are unordered and the fill pass ranks them by list position.
constexpr int kQueueCap = 2 * kWave;

// A candidate for the exact blend.
struct Cand {
  int32_t t;       // neighbour
  uint32_t j;      // its position in the destination's list
  uint32_t list;   // destination, index within the pass
  uint32_t layer;  // covered layer, 0 .. NF-1
};
// The buffer is split into kCandSub sub-buffers with a counter each (a block appends to sub-buffer blockIdx mod
// kCandSub): appending costs an atomic with a returned value, and a single counter would serialise them.
constexpr int kCandSub = 256;
struct CandOut {
  Cand* buf;          // [kCandSub][cap_each]
  uint32_t* count;    // [kCandSub] entries appended so far (may run past cap_each: the excess is dropped, the pass redone)
  uint32_t cap_each;
};

// Stage-1 queue: one per covered layer, three words per candidate: the neighbour, its list position, and which of
// the wave's lists it belongs to (everything else is recomputed from t or looked up per list at stage 2).
struct FirstQueue {
  int32_t t[kMaxFuse][kQueueCap];
  uint32_t j[kMaxFuse][kQueueCap];
  uint32_t slot[kMaxFuse][kQueueCap];
};

struct BlendState {
  FirstQueue* q1;  // passed stage 1 (any list of this wave)
  CandOut cand;    // where the stage-2 survivors go
  uint32_t n1[kMaxFuse] = {0, 0, 0, 0};  // wave-uniform fill levels (each below 64 between calls)
};

// What stage 2 needs to know about the wave's lists: lane i holds the thresholds of list first + i.
template <int NF>
struct ListBlend {
  uint32_t first;
  float lim2[NF];
  float keep2[NF];
};

// stage 2 on entries [first, first + n) of layer l's stage-1 queue (n <= 64): the two uniforms again, the blend in
// fp32.  An estimate safely below the threshold is a kept edge (it takes the next free slot of its destination's
// staging row); one safely above is dropped; the few in between are appended to the candidate buffer of the exact
// stage (one atomic per call).
template <int NF>
__device__ __forceinline__ void blend_second(BlendState& st, int l, uint32_t first, uint32_t n, const ListBlend<NF>& lb, const FusedKeys& keys,
                                             float cwf, float swf, uint32_t stage_cap, const ScanOut& out, Ctl* ctl) {
  const uint32_t lane = (uint32_t)lane_id();
  Cand e{};
  uint32_t slot = 0;
  if (lane < n) {
    e.t = st.q1->t[l][first + lane];
    e.j = st.q1->j[l][first + lane];
    slot = st.q1->slot[l][first + lane];
  }
  // thresholds of the candidate's list: from the lane that holds them (every lane takes part in the exchange)
  const float lim2 = __shfl(lb.lim2[l], (int)slot, kWave);
  const float keep2 = __shfl(lb.keep2[l], (int)slot, kWave);
  bool keep = false, maybe = false;
  if (lane < n) {
    const uint32_t u1 = keyed_uniform<false>(keys.K[l].Ka, (uint32_t)e.t, 0u);
    const uint32_t u2 = keyed_uniform<false>(keys.K[l].Kb, (uint32_t)e.t, 0u);
    e.list = lb.first + slot;
    e.layer = (uint32_t)l;
    const float est = __builtin_fmaf(cwf, approx_phi_inv_f32(u1), swf * approx_phi_inv_f32(u2));
    keep = est <= keep2;
    maybe = !keep && est <= lim2;
  }
  if (keep) {
    const uint32_t at = (uint32_t)atomicAdd(&out.cnt[l][e.list], 1);
    if (at < stage_cap) out.stage[l][(size_t)e.list * stage_cap + at] = StageEntry{e.t, e.j};
    else if (at == stage_cap) atomicAdd(&ctl->n_overflow, 1);  // exactly one entry sees the row fill up
  }
  const uint64_t mask = ballot64(maybe);
  if (mask == 0) return;
  const uint32_t sub = blockIdx.x & (kCandSub - 1);
  uint32_t at = 0;
  if (lane == 0) at = atomicAdd(&st.cand.count[sub], (uint32_t)__popcll(mask));
  at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at) + lanes_below(mask);
  if (maybe) {
    if (at < st.cand.cap_each) st.cand.buf[(size_t)sub * st.cand.cap_each + at] = e;
    else atomicOr(&ctl->cand_overflow, 1);
  }
}

// stage-1 passers of layer l join its queue; a full wave of them goes through stage 2 at once
template <int NF>
__device__ __forceinline__ void blend_first(BlendState& st, int l, bool pre, int32_t t, uint32_t j, uint32_t slot, const ListBlend<NF>& lb,
                                            const FusedKeys& keys, float cwf, float swf, uint32_t stage_cap, const ScanOut& out, Ctl* ctl) {
  const uint64_t mask = ballot64(pre);
  if (mask == 0) return;
  if (pre) {
    const uint32_t at = st.n1[l] + lanes_below(mask);  // below 128
    st.q1->t[l][at] = t;
    st.q1->j[l][at] = j;
    st.q1->slot[l][at] = slot;
  }
  st.n1[l] += (uint32_t)__popcll(mask);
  __builtin_amdgcn_wave_barrier();
  if (st.n1[l] >= (uint32_t)kWave) {
    blend_second<NF>(st, l, 0u, kWave, lb, keys, cwf, swf, stage_cap, out, ctl);
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t rest = st.n1[l] - kWave;  // fewer than 64: to the front
    int32_t mt = 0;
    uint32_t mj = 0, ms = 0;
    if (lane < rest) { mt = st.q1->t[l][kWave + lane]; mj = st.q1->j[l][kWave + lane]; ms = st.q1->slot[l][kWave + lane]; }
    __builtin_amdgcn_wave_barrier();
    if (lane < rest) { st.q1->t[l][lane] = mt; st.q1->j[l][lane] = mj; st.q1->slot[l][lane] = ms; }
    st.n1[l] = rest;
    __builtin_amdgcn_wave_barrier();
  }
}

// what still waits in the stage-1 queues goes through stage 2
template <int NF>
__device__ __forceinline__ void blend_flush_first(BlendState& st, const ListBlend<NF>& lb, const FusedKeys& keys, uint32_t stage_cap,
                                                  const ScanOut& out, Ctl* ctl) {
  const float cwf = (float)keys.cw, swf = (float)keys.sw;
#pragma unroll
  for (int l = 0; l < NF; ++l)
    if (st.n1[l] != 0) {
      blend_second<NF>(st, l, 0u, st.n1[l], lb, keys, cwf, swf, stage_cap, out, ctl);
      st.n1[l] = 0;
      __builtin_amdgcn_wave_barrier();
    }
}

// Blended scan of entries [beg, beg + d) of the wave's list number `slot` (a whole list, or the piece that starts at
// list position j0): same traversal as labor_scan_fast; per entry and layer two mixer evaluations and the stage-1
// compare against pthr.  Candidates may still wait in the stage-1 queues on return.
template <int NF>
__device__ __forceinline__ void labor_scan_blend(const int32_t* __restrict__ g_indices, int64_t beg, uint32_t d, uint32_t j0, uint32_t slot,
                                                 const PreThr (&pthr)[NF], const ListBlend<NF>& lb, const FusedKeys& keys, BlendState& st,
                                                 uint32_t stage_cap, const ScanOut& out, Ctl* ctl) {
  constexpr uint32_t kStep = kWave * 4 * kScanGroups;
  const int64_t abeg = beg & ~(int64_t)3;
  const uint32_t head = (uint32_t)(beg - abeg);
  const uint32_t total = head + d;
  const uint32_t vec_end = total & ~3u;
  const uint32_t vec_beg = head ? 4u : 0u;
  const int32_t* __restrict__ p = g_indices + abeg;
  const uint32_t lane = (uint32_t)lane_id();
  const float cwf = (float)keys.cw, swf = (float)keys.sw;
  // the ragged ends (lanes 0..2: the entries in front of the first whole group; lanes 3..5: those behind the last one) are
  // requested now, so that a short list waits for memory once
  const uint32_t end_pos = lane < 3 ? head + lane : vec_end + (lane - 3);
  const bool end_valid = lane < 3 ? (head != 0 && end_pos < 4 && end_pos < total) : (lane < 6 && end_pos < total && vec_end >= vec_beg);
  int32_t end_t = 0;
  if (end_valid) end_t = p[end_pos];

  for (uint32_t base = vec_beg; base < vec_end; base += kStep) {
    i32x4 buf[kScanGroups];
    bool ok[kScanGroups];
#pragma unroll
    for (int gq = 0; gq < kScanGroups; ++gq) {
      const uint32_t r = base + (uint32_t)(gq * kWave * 4) + lane * 4;
      ok[gq] = r < vec_end;
      buf[gq] = i32x4{0, 0, 0, 0};
      if (ok[gq]) buf[gq] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(p + r));
    }
#pragma unroll
    for (int gq = 0; gq < kScanGroups; ++gq) {
      if (base + (uint32_t)(gq * kWave * 4) >= vec_end) break;  // wave-uniform: the rest of this step lies behind the list
      const uint32_t r = base + (uint32_t)(gq * kWave * 4) + lane * 4;
      bool pre[NF][4];
      bool any = false;
#pragma unroll
      for (int l = 0; l < NF; ++l) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t u1 = keyed_uniform<false>(keys.K[l].Ka, (uint32_t)buf[gq][e], 0u);
          const uint32_t u2 = keyed_uniform<false>(keys.K[l].Kb, (uint32_t)buf[gq][e], 0u);
          const uint32_t lo = u1 < u2 ? u1 : u2, hi = u1 < u2 ? u2 : u1;
          pre[l][e] = ok[gq] & ((lo <= pthr[l].a1) | ((lo <= pthr[l].a2) & (hi <= pthr[l].b2)));
          any |= pre[l][e];
        }
      }
      if (ballot64(any) != 0) {
#pragma unroll
        for (int l = 0; l < NF; ++l) {
#pragma unroll
          for (int e = 0; e < 4; ++e) blend_first<NF>(st, l, pre[l][e], buf[gq][e], r + e - head + j0, slot, lb, keys, cwf, swf, stage_cap, out, ctl);
        }
      }
    }
  }
#pragma unroll
  for (int l = 0; l < NF; ++l) {  // the ragged ends
    const uint32_t a = keyed_uniform<false>(keys.K[l].Ka, (uint32_t)end_t, 0u);
    const uint32_t b = keyed_uniform<false>(keys.K[l].Kb, (uint32_t)end_t, 0u);
    const uint32_t lo = a < b ? a : b, hi = a < b ? b : a;
    blend_first<NF>(st, l, end_valid && (lo <= pthr[l].a1 || (lo <= pthr[l].a2 && hi <= pthr[l].b2)), end_t, end_pos - head + j0, slot, lb, keys,
                    cwf, swf, stage_cap, out, ctl);
  }
}

// The first `piece_blocks` blocks of the grid take the pieces of the long lists (wave w takes pieces w, w + W, ... of
// the queue, W = their number of waves; the queue length is read from device memory, so every wave ends after a
// bounded number of steps).  A piece adds its kept-edge counts to the list's counters and puts its entries wherever
// that leaves them in the staging row; the fill pass sorts the rows of cut lists by list position.
template <bool BLEND, int VEC, int NF>
__global__ __launch_bounds__(kBlock) void k_labor_scan(const int32_t* __restrict__ g_indices, const Segment* __restrict__ seg,
                                                       const uint32_t* __restrict__ thr_all, const PreThr* __restrict__ pthr_all,
                                                       const float* __restrict__ lim2_all, int64_t n, int lists_per_wave, FusedKeys keys,
                                                       uint32_t stage_cap, ScanOut out,
                                                       Ctl* ctl, int piece_blocks, const Piece* __restrict__ pieces,
                                                       const uint32_t* __restrict__ piece_count, uint32_t piece_cap, uint32_t piece_len,
                                                       CandOut cand) {
  constexpr bool kQueued = BLEND && VEC == 4;  // blended variates through the staged filters
  extern __shared__ __align__(16) uint32_t scan_lds[];  // with kQueued: a FirstQueue per wave of the block
  BlendState bst{};
  if constexpr (kQueued) {
    bst.q1 = reinterpret_cast<FirstQueue*>(scan_lds) + uniform_wave_in_block();
    bst.cand = cand;
  }
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t wpb = blockDim.x / kWave;  // waves per block (at most kWavesPerBlock)
  if constexpr (VEC == 4) {
    if ((int)blockIdx.x < piece_blocks) {
      uint32_t n_pieces = *piece_count;
      if (n_pieces > piece_cap) n_pieces = piece_cap;
      const uint32_t n_waves = (uint32_t)piece_blocks * wpb;
      for (uint32_t p = blockIdx.x * wpb + (uint32_t)uniform_wave_in_block(); p < n_pieces; p += n_waves) {
        const Piece pc = pieces[p];
        const uint32_t list = (uint32_t)__builtin_amdgcn_readfirstlane((int)pc.list);
        if (list == kNoPiece) continue;
        const uint32_t q = (uint32_t)__builtin_amdgcn_readfirstlane((int)pc.q);
        const Segment g = seg[list];
        const int64_t beg = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)((uint64_t)g.beg >> 32)) << 32) |
                                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)g.beg));
        const uint32_t d = (uint32_t)__builtin_amdgcn_readfirstlane((int)g.d);
        const uint32_t np = (d + piece_len - 1) / piece_len;  // as in k_segments
        const uint32_t plen = ((d + np - 1) / np + 3u) & ~3u;
        const uint64_t j0_64 = (uint64_t)q * plen;
        if (j0_64 >= d) continue;  // rounding the piece length up can leave the last slots of a very long list empty
        const uint32_t j0 = (uint32_t)j0_64;
        const uint32_t len = d - j0 < plen ? d - j0 : plen;
        uint32_t thr[NF];
#pragma unroll
        for (int l = 0; l < NF; ++l) thr[l] = (uint32_t)__builtin_amdgcn_readfirstlane((int)thr_all[(int64_t)l * n + list]);
        if constexpr (kQueued) {
          PreThr pthr[NF];
          ListBlend<NF> lb;
          lb.first = list;  // every lane holds this list's thresholds: slot 0
#pragma unroll
          for (int l = 0; l < NF; ++l) {
            const PreThr pt = pthr_all[(int64_t)l * n + list];
            pthr[l].a2 = (uint32_t)__builtin_amdgcn_readfirstlane((int)pt.a2);
            pthr[l].a1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)pt.a1);
            pthr[l].b2 = (uint32_t)__builtin_amdgcn_readfirstlane((int)pt.b2);
            pthr[l].keep2 = pt.keep2;
            lb.keep2[l] = pt.keep2;
            lb.lim2[l] = lim2_all[(int64_t)l * n + list];
          }
          labor_scan_blend<NF>(g_indices, beg + j0, len, j0, 0u, pthr, lb, keys, bst, stage_cap, out, ctl);
          blend_flush_first<NF>(bst, lb, keys, stage_cap, out, ctl);
          continue;
        }
        RegSink<NF> sink;
        KeptRegs (&kept)[NF] = sink.kept;
        labor_scan_fast<BLEND, NF>(g_indices, beg + j0, len, j0, thr, keys, sink);
#pragma unroll
        for (int l = 0; l < NF; ++l) {
          const uint32_t c = kept[l].count;
          if (c == 0) continue;
          uint32_t at = 0;
          if (lane == 0) at = (uint32_t)atomicAdd(&out.cnt[l][list], (int32_t)c);
          at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
          if (at + c <= stage_cap) {  // c <= stage_cap <= 64: every entry is still in its register
            if (lane < c) out.stage[l][(size_t)list * stage_cap + at + lane] = StageEntry{kept[l].ent_t, (uint32_t)kept[l].ent_j};
          } else if (at <= stage_cap && lane == 0) {
            atomicAdd(&ctl->n_overflow, 1);  // the one piece that takes the row over its capacity reports the list
          }
        }
      }
      return;
    }
  }
  const int64_t wave = ((int64_t)blockIdx.x - piece_blocks) * wpb + uniform_wave_in_block();
  const int64_t first = wave * lists_per_wave;
  if (first >= n) return;
  const int64_t mine = first + lane;
  const bool has = (int)lane < lists_per_wave && mine < n;
  Segment g{0, 0, 0};
  uint32_t my_thr[NF];
  PreThr my_pthr[NF];
  float my_lim2[NF];
#pragma unroll
  for (int l = 0; l < NF; ++l) { my_thr[l] = kAllThr; my_pthr[l] = PreThr{kAllThr, kAllThr, kAllThr, 0.0f}; my_lim2[l] = 0.0f; }
  if (has) {
    g = seg[mine];
#pragma unroll
    for (int l = 0; l < NF; ++l) {
      my_thr[l] = thr_all[(int64_t)l * n + mine];
      if constexpr (kQueued) { my_pthr[l] = pthr_all[(int64_t)l * n + mine]; my_lim2[l] = lim2_all[(int64_t)l * n + mine]; }
    }
  }
  const uint32_t beg_lo = (uint32_t)g.beg, beg_hi = (uint32_t)((uint64_t)g.beg >> 32);
  uint32_t my_count[NF];
#pragma unroll
  for (int l = 0; l < NF; ++l) my_count[l] = 0;
  ListBlend<NF> lbw;  // lane i: thresholds of list first + i
  lbw.first = (uint32_t)first;
#pragma unroll
  for (int l = 0; l < NF; ++l) { lbw.lim2[l] = my_lim2[l]; lbw.keep2[l] = my_pthr[l].keep2; }
  const int n_lists = (int)(n - first < lists_per_wave ? n - first : lists_per_wave);
  for (int i = 0; i < n_lists; ++i) {
    const int64_t beg = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)beg_hi, i) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane((int)beg_lo, i));
    const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)g.d, i);
    if (__builtin_amdgcn_readlane((int)g.split, i) != 0) continue;  // cut into pieces, scanned by other waves
    uint32_t thr[NF];
    bool any_all = false;
#pragma unroll
    for (int l = 0; l < NF; ++l) {
      thr[l] = (uint32_t)__builtin_amdgcn_readlane((int)my_thr[l], i);
      any_all |= thr[l] == kAllThr;
    }
    if constexpr (kQueued) {  // every list, whatever its length: kept edges reach the rows through the queues
      PreThr pthr[NF];
#pragma unroll
      for (int l = 0; l < NF; ++l) {
        pthr[l].a2 = (uint32_t)__builtin_amdgcn_readlane((int)my_pthr[l].a2, i);
        pthr[l].a1 = (uint32_t)__builtin_amdgcn_readlane((int)my_pthr[l].a1, i);
        pthr[l].b2 = (uint32_t)__builtin_amdgcn_readlane((int)my_pthr[l].b2, i);
        pthr[l].keep2 = 0.0f;  // (stage 2 takes it from the lane that holds the list)
      }
      if (d != 0) labor_scan_blend<NF>(g_indices, beg, d, 0u, (uint32_t)i, pthr, lbw, keys, bst, stage_cap, out, ctl);
      continue;
    }
    if (VEC == 4 && !any_all && d > (uint32_t)kWave) {
      RowSink<NF> sink;
      sink.cap = stage_cap;
#pragma unroll
      for (int l = 0; l < NF; ++l) { sink.row[l] = out.stage[l] + (size_t)(first + i) * stage_cap; sink.count[l] = 0; }
      labor_scan_fast<BLEND, NF>(g_indices, beg, d, 0u, thr, keys, sink);
#pragma unroll
      for (int l = 0; l < NF; ++l)
        if ((int)lane == i) my_count[l] = sink.count[l];
    } else {
#pragma unroll
      for (int l = 0; l < NF; ++l) {
        StageEntry* row = out.stage[l] + (size_t)(first + i) * stage_cap;
        const uint32_t c = labor_scan_ordered<BLEND>(g_indices, beg, d, thr[l], keys.K[l], keys.cw, keys.sw,
                                                     [&](uint32_t rank, int32_t t, uint32_t j) {
                                                       if (rank < stage_cap) row[rank] = StageEntry{t, j};
                                                     });
        if ((int)lane == i) my_count[l] = c;
      }
    }
  }
  if constexpr (kQueued) {
    blend_flush_first<NF>(bst, lbw, keys, stage_cap, out, ctl);
    return;  // (the counters were kept by atomics, here and in the exact stage)
  }
  if (has && g.split == 0) {  // (the pieces of a cut list add their counts themselves)
#pragma unroll
    for (int l = 0; l < NF; ++l) {
      out.cnt[l][mine] = (int32_t)my_count[l];
      if (my_count[l] > stage_cap) atomicAdd(&ctl->n_overflow, 1);
    }
  }
}

// Stage 3 of the blended path: the exact blend for every candidate the scan kernel appended, one candidate per thread
// (grid-stride; the count is read from device memory).  A kept edge takes the next free slot of its destination's
// staging row.
__global__ __launch_bounds__(kBlock) void k_labor_exact(CandOut cand, const uint32_t* __restrict__ thr_all, int64_t n, int nf, FusedKeys keys,
                                                        uint32_t stage_cap, ScanOut out, Ctl* ctl) {
  uint32_t total = cand.count[blockIdx.y];  // blockIdx.y: the sub-buffer
  if (total > cand.cap_each) total = cand.cap_each;
  const Cand* __restrict__ mine = cand.buf + (size_t)blockIdx.y * cand.cap_each;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (uint64_t)gridDim.x * kBlock) {
    const Cand e = mine[i];
    if (e.layer >= (uint32_t)nf || (int64_t)e.list >= n) continue;  // (never: the scan kernel wrote it)
    LayerKeys K = keys.K[0];
    int32_t* cnt = out.cnt[0];
    StageEntry* stage = out.stage[0];
#pragma unroll
    for (int f = 1; f < kMaxFuse; ++f)
      if (e.layer == (uint32_t)f) { K = keys.K[f]; cnt = out.cnt[f]; stage = out.stage[f]; }
    const uint32_t thr = thr_all[(int64_t)e.layer * n + e.list];
    const double n1 = kit_phi_inv_u32(keyed_uniform<false>(K.Ka, (uint32_t)e.t, 0u));
    const double n2 = kit_phi_inv_u32(keyed_uniform<false>(K.Kb, (uint32_t)e.t, 0u));
    const uint32_t R = kit_phi_to_u32(__builtin_fma(keys.cw, n1, keys.sw * n2));
    if (R <= thr) {
      const uint32_t at = (uint32_t)atomicAdd(&cnt[e.list], 1);
      if (at < stage_cap) stage[(size_t)e.list * stage_cap + at] = StageEntry{e.t, e.j};
      else if (at == stage_cap) atomicAdd(&ctl->n_overflow, 1);  // exactly one entry sees the row fill up
    }
  }
}

__global__ void k_enum_redo(Ctl* ctl, uint32_t* piece_count) {
  ctl->cand_overflow = 0;
  *piece_count = 0;
}

__global__ void k_labor_redo(Ctl* ctl, uint32_t* piece_count, uint32_t* cand_count) {  // kCandSub threads
  if (threadIdx.x == 0) {
    ctl->cand_overflow = 0;
    *piece_count = 0;
  }
  cand_count[threadIdx.x] = 0;
}

// staged rows -> the block's edge arrays: kFillLanes threads per destination, each taking every kFillLanes-th slot
constexpr int kFillLanesLog2 = 3;
// (edge_limit: entries of col_global / eid; nothing is written beyond them)
__global__ __launch_bounds__(kBlock) void k_labor_fill_staged(LayerChunks ch, int64_t n_dst, uint32_t stage_cap,
                                                              const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                              int64_t* __restrict__ eid, int64_t edge_limit) {
  __shared__ uint32_t row_j[kBlock >> kFillLanesLog2][kWave];  // list positions of one staged row per lane group
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t w = idx >> kFillLanesLog2;
  if (w >= n_dst) return;
  const int64_t o = eptr[w];
  const int64_t c = eptr[w + 1] - o;
  if (c > (int64_t)stage_cap) return;  // overflowed row: the overflow pass writes these edges
  const int p = ch.find(w);
  const int64_t local = w - ch.start[p];
  const StageEntry* __restrict__ row = ch.stage[p] + (size_t)local * stage_cap;
  const Segment g = ch.seg[p][local];
  const int sub = (int)(idx & ((1 << kFillLanesLog2) - 1));
  // A row may hold its entries in any order (the fast scan writes them as they come, the pieces of a cut list and the
  // blended passes take slots by atomics): an entry's place is its rank by list position.  The lane group (all in one
  // wave) shares the positions through LDS.  Rows that happen to be in order go the same way: two paths side by side
  // in a wave cost more than ranking a dozen entries.
  uint32_t* js = row_j[threadIdx.x >> kFillLanesLog2];
  constexpr int kPerLane = kWave >> kFillLanesLog2;
  StageEntry mine[kPerLane];
#pragma unroll
  for (int i = 0; i < kPerLane; ++i) {
    const int slot = sub + (i << kFillLanesLog2);
    mine[i] = StageEntry{0, 0xFFFFFFFFu};
    if (slot < c) { mine[i] = row[slot]; js[slot] = mine[i].j; }  // (only js[0..c) is read below)
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int i = 0; i < kPerLane; ++i) {
    const int slot = sub + (i << kFillLanesLog2);
    if (slot >= c) break;
    int64_t place = 0;
    for (int q = 0; q < (int)c; ++q) place += js[q] < mine[i].j;
    if (o + place < edge_limit) {
      col_global[o + place] = mine[i].t;
      eid[o + place] = g.beg + mine[i].j;
    }
  }
}

// second, ordered scan of the (rare) destinations whose staging row overflowed, writing straight to the edge arrays
template <bool BLEND>
__global__ __launch_bounds__(kBlock) void k_labor_fill_overflow(const int32_t* __restrict__ g_indices, LayerChunks ch, int64_t n_dst,
                                                                LayerKeys K, double cw, double sw, uint32_t stage_cap,
                                                                const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                                int64_t* __restrict__ eid) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + uniform_wave_in_block();
  if (w >= n_dst) return;
  const int64_t o = eptr[w];
  if (eptr[w + 1] - o <= (int64_t)stage_cap) return;
  const int p = ch.find(w);
  const int64_t local = w - ch.start[p];
  const Segment g = ch.seg[p][local];
  const uint32_t thr = ch.thr[p][local];
  labor_scan_ordered<BLEND>(g_indices, g.beg, g.d, thr, K, cw, sw, [&](uint32_t rank, int32_t t, uint32_t j) {
    col_global[o + rank] = t;
    eid[o + rank] = g.beg + j;
  });
}

template <bool BLEND, int VEC>
static void launch_scan(int nf, dim3 grid, dim3 block, hipStream_t s, const int32_t* indices, const Segment* seg, const uint32_t* thr, const PreThr* pthr, const float* lim2, int64_t n,
                        int lpw, const FusedKeys& keys, uint32_t cap, const ScanOut& out, Ctl* ctl, int piece_blocks, const Piece* pieces,
                        const uint32_t* piece_count, uint32_t piece_cap, uint32_t piece_len, const CandOut& cand) {
  switch (nf) {
    case 1: COOP_LAUNCH(K_LABOR_COUNT, (k_labor_scan<BLEND, VEC, 1>), grid, block, (BLEND && VEC == 4) ? (size_t)(block.x / kWave) * sizeof(FirstQueue) : 0, s, indices, seg, thr, pthr, lim2, n, lpw, keys, cap, out, ctl, piece_blocks, pieces, piece_count, piece_cap, piece_len, cand); break;
    case 2: COOP_LAUNCH(K_LABOR_COUNT, (k_labor_scan<BLEND, VEC, 2>), grid, block, (BLEND && VEC == 4) ? (size_t)(block.x / kWave) * sizeof(FirstQueue) : 0, s, indices, seg, thr, pthr, lim2, n, lpw, keys, cap, out, ctl, piece_blocks, pieces, piece_count, piece_cap, piece_len, cand); break;
    case 3: COOP_LAUNCH(K_LABOR_COUNT, (k_labor_scan<BLEND, VEC, 3>), grid, block, (BLEND && VEC == 4) ? (size_t)(block.x / kWave) * sizeof(FirstQueue) : 0, s, indices, seg, thr, pthr, lim2, n, lpw, keys, cap, out, ctl, piece_blocks, pieces, piece_count, piece_cap, piece_len, cand); break;
    default: COOP_LAUNCH(K_LABOR_COUNT, (k_labor_scan<BLEND, VEC, 4>), grid, block, (BLEND && VEC == 4) ? (size_t)(block.x / kWave) * sizeof(FirstQueue) : 0, s, indices, seg, thr, pthr, lim2, n, lpw, keys, cap, out, ctl, piece_blocks, pieces, piece_count, piece_cap, piece_len, cand); break;
  }
}

int labor_layer(LaborState& st, const SampleCtx& cx, int l, const int32_t* dst, int64_t n_dst, coop_block* blk, int64_t edge_cap) {
  const bool defer = edge_cap > 0;
  hipStream_t s = cx.s;
  Alloc& alloc = *cx.alloc;
  if (l == 0) {
    // fuse when every remaining layer fits one scan (GNNs have 2-3 layers); otherwise scan layer by layer
    st.fuse = cx.L <= kMaxFuse && g_fuse_layers != 0;
    uint32_t kmax = 0;
    for (int i = 0; i < cx.L; ++i) kmax = (uint32_t)cx.fanouts[i] > kmax ? (uint32_t)cx.fanouts[i] : kmax;
    // staging rows: room for 2k + 16 kept edges (a row overflows with probability < 1e-8 at k = 10), 32 or 64 entries
    // (what one wave parks in a register pair); a row that overflows is redone by the overflow pass
    st.stage_cap = 2 * (uint64_t)kmax + 16 > 32 ? 64 : 32;
    if (g_stage_cap_override) st.stage_cap = (uint32_t)g_stage_cap_override;
    st.n_pass = 0;
    st.covered = 0;
  }
  const uint32_t cap = st.stage_cap;

  // ---- scan pass over the destinations not covered yet ------------------------------------------------------------
  // Normally the pass evaluates every remaining layer and is recorded.  A pass over only a few lists (the seeds'
  // hop) is not worth a many-layer kernel: it evaluates this layer alone and leaves its destinations to the next pass.
  constexpr int64_t kFuseMinLists = 32768;
  const bool record = st.fuse && (n_dst - st.covered >= kFuseMinLists || l == cx.L - 1 || g_fuse_layers == 2);
  LaborPass local;
  LaborPass& ps = record ? st.pass[st.n_pass] : local;
  ps.first_layer = l;
  ps.start = st.covered;
  ps.n_new = n_dst - ps.start;
  ps.nf = record ? cx.L - l : 1;
  const int64_t n_new = ps.n_new;
  ps.seg = alloc.get<Segment>(n_new, COOP_TAG_SCRATCH);
  ps.thr = alloc.get<uint32_t>(n_new * ps.nf, COOP_TAG_SCRATCH);
  PreThr* pthr = cx.blend ? alloc.get<PreThr>(n_new * ps.nf, COOP_TAG_SCRATCH) : nullptr;
  float* lim2 = cx.blend ? alloc.get<float>(n_new * ps.nf, COOP_TAG_SCRATCH) : nullptr;
  for (int f = 0; f < ps.nf; ++f) {
    ps.stage[f] = alloc.get<StageEntry>(n_new * (int64_t)cap, COOP_TAG_SCRATCH);
    ps.cnt[f] = alloc.get<int32_t>(n_new, COOP_TAG_SCRATCH);
  }
  blk->indptr = alloc.get<int64_t>(n_dst + 1, COOP_TAG_OUTPUT);
  void* scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_dst), COOP_TAG_SCRATCH);
  if (alloc.failed) return COOP_E_NOMEM;

  FusedKeys keys{};
  keys.cw = cx.cw;
  keys.sw = cx.sw;
  uint32_t ks[kMaxFuse] = {1, 1, 1, 1};
  for (int f = 0; f < ps.nf; ++f) {
    layer_keys(cx.seed, COOP_LABOR0, l + f, cx.group, keys.K[f].Ka);
    layer_keys(cx.seed, COOP_LABOR0, l + f, cx.group + 1, keys.K[f].Kb);
    ks[f] = (uint32_t)cx.fanouts[l + f];
  }
  // long lists are cut into pieces (k_segments queues them); room for every piece the graph's edges could make
  const uint32_t piece_len = cx.vec4 ? (uint32_t)g_piece_len : 0u;
  // Lists longer than split_min go to the piece waves, which come first in the grid.  With independent variates that is
  // for the lists worth cutting (twice the piece length).  The blended scan costs three times as much per entry, and a
  // wave that meets a few lists of several thousand entries late in the kernel keeps it waiting: there every list above
  // 2,048 entries goes first, whole if it is shorter than two pieces (papers100M-shaped, kappa 16: scan 1.44 -> 1.32 ms;
  // no difference with independent variates).
  const uint32_t split_min = g_split_min != 0 ? (uint32_t)g_split_min : (cx.blend && piece_len >= 2048u ? 2048u : 2u * piece_len);
  uint32_t piece_cap = 0;
  Piece* pieces = nullptr;
  if (piece_len != 0 && n_new > 0) {
    const int64_t by_edges = cx.g->n_edges / piece_len;
    const int64_t long_lists = cx.g->n_edges / (int64_t)split_min + 1;
    const int64_t cap64 = by_edges + (n_new < long_lists ? n_new : long_lists) + 1;
    piece_cap = (uint32_t)(cap64 < ((int64_t)1 << 30) ? cap64 : ((int64_t)1 << 30));
    pieces = alloc.get<Piece>(piece_cap, COOP_TAG_SCRATCH);
    if (alloc.failed) return COOP_E_NOMEM;
  }
  // blended variates: stage 3 works from a buffer of the candidates that the fp32 blend left undecided, a few percent
  // of the k kept edges per destination and layer; k / 2 each is ample (a pass that overflows it is redone with more)
  const bool queued = cx.blend && cx.vec4 && n_new > 0;
  int64_t cand_cap = 0;
  uint32_t* cand_count = nullptr;
  if (queued) {
    uint32_t kpass = 1;
    for (int f = 0; f < ps.nf; ++f) kpass = ks[f] > kpass ? ks[f] : kpass;
    cand_cap = g_blend_candidates ? g_blend_candidates : (int64_t)kpass * n_new * ps.nf / 2 + 65536;
    if (cand_cap > ((int64_t)1 << 30)) cand_cap = (int64_t)1 << 30;
    cand_count = alloc.get<uint32_t>(kCandSub, COOP_TAG_SCRATCH);
    if (alloc.failed) return COOP_E_NOMEM;
    fill_u64((uint64_t*)cand_count, kCandSub / 2, 0, s);
  }
  // ---- this layer's destinations, piece by piece: a recorded pass covered it as its (l - first_layer)-th layer ------
  if (record) { st.n_pass += 1; st.covered = n_dst; }
  LayerChunks ch{};
  ChunkedI32 counts{};
  int nc = 0;
  auto add_chunk = [&](const LaborPass& q) {
    if (q.n_new == 0) return;  // a pass that scanned nothing (a layer that added no vertex) contributes no piece
    const int f = l - q.first_layer;
    ch.seg[nc] = q.seg;
    ch.thr[nc] = q.thr + (int64_t)f * q.n_new;
    ch.stage[nc] = q.stage[f];
    ch.start[nc] = counts.start[nc] = q.start;
    counts.ptr[nc] = q.cnt[f];
    ++nc;
  };
  for (int p = 0; p < st.n_pass; ++p) add_chunk(st.pass[p]);
  if (!record) add_chunk(local);
  if (nc == 0) { ch.seg[0] = ps.seg; ch.thr[0] = ps.thr; ch.stage[0] = ps.stage[0]; counts.ptr[0] = ps.cnt[0]; nc = 1; }  // n_dst == 0
  ch.n_chunks = counts.n_chunks = nc;

  bool no_enum = false, used_enum = false;
  for (;;) {
    used_enum = false;
    if (n_new > 0) {
      ScanOut out{};
      for (int f = 0; f < ps.nf; ++f) { out.stage[f] = ps.stage[f]; out.cnt[f] = ps.cnt[f]; }
      CandOut cand{};
      if (queued) {
        cand.cap_each = (uint32_t)((cand_cap + kCandSub - 1) / kCandSub);
        cand.buf = alloc.get<Cand>((int64_t)cand.cap_each * kCandSub, COOP_TAG_SCRATCH);
        cand.count = cand_count;
        if (alloc.failed) return COOP_E_NOMEM;
      }
      // ---- the longest lists from the other side (see k_enum_list) ---------------------------------------------------
      uint32_t kmax_pass = 0;
      for (int f = 0; f < ps.nf; ++f) kmax_pass = ks[f] > kmax_pass ? ks[f] : kmax_pass;
      // (listing and walking cost the same whatever the number of destinations and the shape of the graph: it pays only
      // for a pass over many lists of a graph whose long lists hold a good part (an eighth, here) of the edges; a knob
      // value below the default is for tests and applies always)
      const bool enough = g_enum_degree < kLongListDegree || (n_new >= 65536 && cx.g->long_mass * 8 >= cx.g->n_edges);
      const uint32_t enum_degree = cx.g->symmetric && !cx.blend && !no_enum && kmax_pass <= 64 && enough ? (uint32_t)g_enum_degree : 0u;
      used_enum = enum_degree != 0;
      LongSlot* long_tab = nullptr;
      uint32_t* long_bits = nullptr;
      uint32_t long_mask = 0;
      EnumOut eo{};
      uint32_t u_max[kMaxFuse] = {0, 0, 0, 0}, um_most = 0, list_todo = 0;
      if (enum_degree != 0) {
        // the table of long destinations: twice the number there can be (|E| / D lists are that long, at most), but no
        // more than 65536 slots or a quarter of the destinations, whichever is more: the table then stays in L2, and a
        // pass with more long lists than that is redone the ordinary way
        int64_t most = cx.g->n_edges / enum_degree + 1;
        if (most > n_new) most = n_new;
        const int64_t ceiling = n_new / 4 > 65536 ? n_new / 4 : 65536;
        uint32_t slots = 1024;
        while ((int64_t)slots < 2 * most && (int64_t)slots * 2 <= ceiling) slots <<= 1;
        long_mask = slots - 1;
        constexpr int64_t kBitSlots = kLongBits / 8 / sizeof(LongSlot);
        uint32_t* zeroed = (uint32_t*)alloc.get<LongSlot>(1 + kBitSlots + (int64_t)slots, COOP_TAG_SCRATCH);  // counters, bits, table
        long_bits = (uint32_t*)((LongSlot*)zeroed + 1);
        long_tab = (LongSlot*)zeroed + 1 + kBitSlots;
        // The vertices listed for a layer depend on the layer's keys and fanout only: a later pass that covers the same
        // layer (the pass at layer 2 after the pass at layer 1 that covered layers 1 and 2) walks the same items.
        for (int f = 0; f < ps.nf; ++f) {
          u_max[f] = (uint32_t)(((uint64_t)ks[f] << 32) / ((uint64_t)enum_degree + 1));
          LaborState::Listed* had = l + f < LaborState::kMaxListed ? &st.listed[l + f] : nullptr;
          if (had != nullptr && had->item != nullptr && had->u_max == u_max[f]) {
            eo.item[f] = had->item;
            eo.n_item[f] = had->n;
            eo.item_cap[f] = had->cap;
            continue;
          }
          // items: a listed vertex gives d / kEnumItem + 1 of them; the listed vertices' lists hold |E| u_max / 2^32
          // entries in expectation, and four times that is allowed for (a pass that needs more, because some huge hub is
          // listed, is redone the ordinary way)
          const double expect = (double)cx.g->n_vertices * ((double)u_max[f] + 1.0) / 4294967296.0;  // listed vertices
          const double entries = (double)cx.g->n_edges * ((double)u_max[f] + 1.0) / 4294967296.0;
          const double items = expect + 8.0 * sqrt(expect) + 1024.0 + 4.0 * entries / kEnumItem;
          eo.item_cap[f] = (uint32_t)(items < 268435456.0 ? items : 268435456.0);
          eo.item[f] = alloc.get<EnumItem>(eo.item_cap[f], COOP_TAG_SCRATCH);
          eo.n_item[f] = zeroed + f;
          list_todo |= 1u << f;
          um_most = u_max[f] > um_most ? u_max[f] : um_most;
          if (had != nullptr) *had = LaborState::Listed{eo.item[f], eo.n_item[f], eo.item_cap[f], u_max[f]};
        }
        for (int f = ps.nf; f < kMaxFuse; ++f) { eo.item[f] = eo.item[0]; eo.n_item[f] = eo.n_item[0]; eo.item_cap[f] = 0; }
        if (alloc.failed) return COOP_E_NOMEM;
        fill_u64((uint64_t*)zeroed, (1 + kLongBits / 8 / sizeof(LongSlot) + (int64_t)slots) * (sizeof(LongSlot) / 8), 0, s);
      }
      COOP_LAUNCH(K_SEGMENTS, k_segments, dim3(blocks_for(n_new, kSegBlock)), dim3(kSegBlock), 0, s, cx.g->indptr, cx.g->n_vertices,
                  dst + ps.start, n_new, ps.nf, ks[0], ks[1], ks[2], ks[3], ps.seg, ps.thr, pthr, lim2, cx.cw, cx.sw,
                  cx.blend && cx.vec4 ? 1 : 0, cx.d_ctl,
                  piece_len, split_min, pieces, piece_cap, cx.d_piece_count + l, out, enum_degree, long_bits, long_tab, long_mask);
      if (enum_degree != 0) {
        if (list_todo != 0) {
          const unsigned list_blocks = blocks_for((int64_t)um_most + 1, kEnumListSpan);
          COOP_LAUNCH(K_ENUM_LIST, k_enum_list, dim3(list_blocks, ps.nf), dim3(kListBlock), 0, s, keys, u_max[0], u_max[1], u_max[2], u_max[3],
                      cx.g->n_vertices, cx.g->indptr, eo, cx.d_ctl, list_todo);
        }
        // (three blocks fit a CU: one round of resident blocks strides over the items)
        uint32_t cap_most = 0;
        for (int f = 0; f < ps.nf; ++f) cap_most = eo.item_cap[f] > cap_most ? eo.item_cap[f] : cap_most;
        const int64_t walk_blocks = blocks_for((int64_t)cap_most * 16, kWalkBlock);
        COOP_LAUNCH(K_ENUM_WALK, k_enum_walk, dim3((unsigned)(walk_blocks < 768 ? walk_blocks : 768), ps.nf), dim3(kWalkBlock), 0, s,
                    cx.g->indices, (const uint32_t*)cx.g->rev_pos, (const uint32_t*)long_bits, (const LongSlot*)long_tab, long_mask, cap, out,
                    eo, cx.d_ctl);
      }
      // lists per wave: a few amortise the record fetch once there are plenty of lists (the knob overrides)
      int lpw = g_lists_per_wave;
      if (lpw == 0) lpw = n_new >= 65536 ? (cx.blend && cx.vec4 ? 8 : 4) : 1;  // blended: fuller waves at the fp32 stage
      const int64_t n_waves = (n_new + lpw - 1) / lpw;
      // the piece waves come first in the grid: one round of resident blocks, fewer if there cannot be that many pieces
      constexpr int64_t kPieceBlocks = 2048;
      // waves per block: a block leaves the CU when its slowest wave is done, and the lists differ in length by orders
      // of magnitude, so with four waves a block's slots stand empty for much of its life; two waves per block take 3 to
      // 8 % off the scan with independent variates (one: 2 to 5 %), one wave per block 2 % off the blended one, which
      // is bound by its arithmetic (its first-stage queues are dynamic LDS, one per wave of the block)
      const int wpb = cx.blend ? 1 : 2;
      const dim3 block((unsigned)(wpb * kWave));
      const int64_t piece_waves = (int64_t)piece_cap < kPieceBlocks * kWavesPerBlock ? (int64_t)piece_cap : kPieceBlocks * kWavesPerBlock;
      const int piece_blocks = (int)blocks_for(piece_waves, wpb);
      const dim3 grid(blocks_for(n_waves, wpb) + (unsigned)piece_blocks);
      const uint32_t* pcount = cx.d_piece_count + l;
      if (cx.blend) {
        if (cx.vec4) launch_scan<true, 4>(ps.nf, grid, block, s, cx.g->indices, ps.seg, ps.thr, pthr, lim2, n_new, lpw, keys, cap, out, cx.d_ctl, piece_blocks, pieces, pcount, piece_cap, piece_len, cand);
        else launch_scan<true, 1>(ps.nf, grid, block, s, cx.g->indices, ps.seg, ps.thr, pthr, lim2, n_new, lpw, keys, cap, out, cx.d_ctl, 0, pieces, pcount, 0u, 0u, cand);
      } else {
        if (cx.vec4) launch_scan<false, 4>(ps.nf, grid, block, s, cx.g->indices, ps.seg, ps.thr, pthr, lim2, n_new, lpw, keys, cap, out, cx.d_ctl, piece_blocks, pieces, pcount, piece_cap, piece_len, cand);
        else launch_scan<false, 1>(ps.nf, grid, block, s, cx.g->indices, ps.seg, ps.thr, pthr, lim2, n_new, lpw, keys, cap, out, cx.d_ctl, 0, pieces, pcount, 0u, 0u, cand);
      }
      if (queued) {  // stage 3: the exact blend for the candidates that the scan appended
        const unsigned blocks = blocks_for(cand.cap_each, kBlock) < 16 ? blocks_for(cand.cap_each, kBlock) : 16;
        COOP_LAUNCH(K_LABOR_EXACT, k_labor_exact, dim3(blocks, kCandSub), dim3(kBlock), 0, s, cand, ps.thr, n_new, ps.nf, keys, cap, out,
                    cx.d_ctl);
      }
    }

    if (defer) {  // the count stays on the device; an overflow of the candidate buffer is the caller's to notice
      scan_chunks_to_i64(counts, n_dst, blk->indptr, &cx.d_ctl->total_edges, scan_tmp, s, nullptr);
      break;
    }
    const Publish pub = begin_publish(cx.d_ctl, cx.h_ctl);  // the scan's last thread also sends the sizes to the host
    scan_chunks_to_i64(counts, n_dst, blk->indptr, &cx.d_ctl->total_edges, scan_tmp, s, &pub);  // m_l = indptr[n_dst]
    const int rc = wait_ctl(pub, cx.h_ctl, s);
    if (rc != COOP_OK) return rc;
    if (used_enum && cx.h_ctl->cand_overflow != 0) {  // the lists of the listed vertices did not fit: once more, every list scanned
      no_enum = true;
      for (auto& had : st.listed) had = LaborState::Listed{};  // (what was listed may be incomplete)
      hipLaunchKernelGGL(k_enum_redo, dim3(1), dim3(1), 0, s, cx.d_ctl, cx.d_piece_count + l);
      continue;
    }
    if (!queued || cx.h_ctl->cand_overflow == 0) break;
    // the candidate buffer of the exact stage was too small (counts are incomplete): once more with 8 times the room
    if (cand_cap >= ((int64_t)1 << 30)) return COOP_E_CAPACITY;
    cand_cap = cand_cap * 8 < ((int64_t)1 << 30) ? cand_cap * 8 : ((int64_t)1 << 30);
    hipLaunchKernelGGL(k_labor_redo, dim3(1), dim3(kCandSub), 0, s, cx.d_ctl, cx.d_piece_count + l, cand_count);
  }
  const int64_t m = defer ? edge_cap : cx.h_ctl->total_edges;  // entries of the edge arrays
  blk->n_edges = defer ? -1 : m;
  blk->col_global = alloc.get<int32_t>(m, COOP_TAG_OUTPUT);
  blk->eid = alloc.get<int64_t>(m, COOP_TAG_OUTPUT);
  blk->col_local = alloc.get<int32_t>(m, COOP_TAG_OUTPUT);
  if (alloc.failed) return COOP_E_NOMEM;

  if (m > 0 && n_dst > 0) {
    COOP_LAUNCH(K_LABOR_FILL, k_labor_fill_staged, dim3(blocks_for(n_dst << kFillLanesLog2, kBlock)), dim3(kBlock), 0, s, ch, n_dst, cap,
                blk->indptr, blk->col_global, blk->eid, m);
    if (!defer && cx.h_ctl->n_overflow > 0) {
      LayerKeys K{};
      layer_keys(cx.seed, COOP_LABOR0, l, cx.group, K.Ka);
      layer_keys(cx.seed, COOP_LABOR0, l, cx.group + 1, K.Kb);
      const dim3 grid(blocks_for(n_dst, kWavesPerBlock));
      if (cx.blend)
        COOP_LAUNCH(K_LABOR_OVERFLOW, k_labor_fill_overflow<true>, grid, dim3(kBlock), 0, s, cx.g->indices, ch, n_dst, K, cx.cw, cx.sw,
                    cap, blk->indptr, blk->col_global, blk->eid);
      else
        COOP_LAUNCH(K_LABOR_OVERFLOW, k_labor_fill_overflow<false>, grid, dim3(kBlock), 0, s, cx.g->indices, ch, n_dst, K, cx.cw, cx.sw,
                    cap, blk->indptr, blk->col_global, blk->eid);
    }
  }
  return COOP_OK;
}

}  // namespace coop
