// Random-walk sampling (App. A.1.3): from every destination s, a walks of o steps; the first step goes to a uniform
// neighbour of s, every later step to a uniform neighbour of the current vertex, or, with the restart probability p,
// of s; the k most visited vertices become the sampled neighbours of s.
//
// One wave per destination.  Lanes walk (two walks per lane at a time, so that their dependent loads overlap) and
// tally every visit in a small open-addressing table in LDS (vertex, count).  Each lane then holds its share of the
// table in registers; the k best entries by (count descending, vertex ascending), the order in which the sources
// are emitted, are found by two bisections over wave-wide ballot tallies and ranked among themselves.  The draws are keyed hashes of
// (destination, draw counter), so the result does not depend on which lane walks which walk.
#include "device_utils.h"
#include "sample_internal.h"

namespace coop {

constexpr uint32_t kRwEmpty = 0xFFFFFFFFu;
constexpr int kRwMaxSteps = 1024;  // largest walk_length * n_walks that the tally in LDS serves (beyond it: k_rw_walk_wide)

struct RwParams {
  uint32_t K[4];         // key words of (seed, sampler RW, layer, iteration)
  int32_t walk_length;   // o
  int32_t n_walks;       // a
  uint64_t restart_thr;  // restart iff draw < floor(p 2^32)
  uint32_t k_eff;        // min(fanout, o * a): slots of a staged row
};

__device__ __forceinline__ uint32_t rw_draw(const uint32_t (&K)[4], uint32_t sigma, uint32_t c) {
  return mix32(mix32(c ^ K[0]) ^ K[1] ^ sigma) ^ K[3];  // sigma = mix32(s ^ K[2])
}

// E = table slots per lane (table of 64 E slots, at most 3/4 full)
template <int E>
__global__ __launch_bounds__(kBlock) void k_rw_walk(const int64_t* __restrict__ g_indptr, const int32_t* __restrict__ g_indices,
                                                    int64_t n_vertices, const int32_t* __restrict__ dst, int64_t n_dst, RwParams rp,
                                                    int waves_per_block, StageEntry* __restrict__ rows, int32_t* __restrict__ cnt,
                                                    Ctl* ctl) {
  extern __shared__ uint32_t rw_lds[];  // per wave: 64 E vertex keys, 64 E counts
  constexpr uint32_t T = (uint32_t)kWave * E;
  const int wib = uniform_wave_in_block();
  if (wib >= waves_per_block) return;
  const int64_t w = (int64_t)blockIdx.x * waves_per_block + wib;
  if (w >= n_dst) return;
  const uint32_t lane = (uint32_t)lane_id();
  uint32_t* keys = rw_lds + (size_t)wib * 2 * T;
  uint32_t* counts = keys + T;
#pragma unroll
  for (int e = 0; e < E; ++e) { keys[e * kWave + lane] = kRwEmpty; counts[e * kWave + lane] = 0; }
  const int32_t s = dst[w];
  if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
    if (lane == 0) { atomicOr(&ctl->err_range, 1); cnt[w] = 0; }
    return;
  }
  const int64_t s_beg = g_indptr[s];
  const uint32_t s_d = (uint32_t)(g_indptr[s + 1] - s_beg);
  if (s_d == 0) {  // wave-uniform
    if (lane == 0) cnt[w] = 0;
    return;
  }
  __builtin_amdgcn_wave_barrier();
  const uint32_t sigma = mix32((uint32_t)s ^ rp.K[2]);
  const int o = rp.walk_length, a = rp.n_walks;

  for (int w0 = 0; w0 < a; w0 += 2 * kWave) {
    int walk[2] = {w0 + (int)lane, w0 + kWave + (int)lane};
    bool alive[2] = {walk[0] < a, walk[1] < a};
    uint32_t cur[2] = {(uint32_t)s, (uint32_t)s};
    for (int step = 0; step < o; ++step) {
      int64_t beg[2];
      uint32_t d[2], u[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const uint32_t c = 2u * (uint32_t)(walk[q] * o + step);
        u[q] = rw_draw(rp.K, sigma, c);
        const bool restart = step == 0 || (uint64_t)rw_draw(rp.K, sigma, c + 1u) < rp.restart_thr;
        beg[q] = s_beg;
        d[q] = s_d;
        if (alive[q] && !restart) {
          beg[q] = g_indptr[cur[q]];
          d[q] = (uint32_t)(g_indptr[cur[q] + 1] - beg[q]);
        }
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        if (d[q] == 0) alive[q] = false;  // dead end: the walk ends
        if (alive[q]) cur[q] = (uint32_t)g_indices[beg[q] + (int64_t)(((uint64_t)u[q] * (uint64_t)d[q]) >> 32)];
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        if (alive[q] && (uint64_t)cur[q] >= (uint64_t)n_vertices) {  // a neighbour id outside the graph
          atomicOr(&ctl->err_range, 1);
          alive[q] = false;
        }
        if (alive[q]) {  // tally the visit
          uint32_t h = (cur[q] * 0x9E3779B1u) >> 7 & (T - 1);
          for (;;) {
            const uint32_t old = atomicCAS(&keys[h], kRwEmpty, cur[q]);
            if (old == kRwEmpty || old == cur[q]) { atomicAdd(&counts[h], 1u); break; }
            h = (h + 1) & (T - 1);  // at most o a <= 3 T / 4 distinct vertices: an empty slot is always reached
          }
        }
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // Each lane takes its E slots of the table into registers; the k best by (count descending, vertex ascending) are
  // found without sorting: the count of the k-th best by bisection over wave-wide tallies (ballots), then, among
  // the vertices visited exactly that often, the id below which just enough of them lie, again by bisection.
  uint32_t cnt_e[E], id_e[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    id_e[e] = keys[e * kWave + lane];
    cnt_e[e] = id_e[e] != kRwEmpty ? counts[e * kWave + lane] : 0u;
  }
  __builtin_amdgcn_wave_barrier();  // the table's memory is reused below
  auto n_with_count_at_least = [&](uint32_t c) {
    uint32_t n = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) n += (uint32_t)__popcll(ballot64(cnt_e[e] >= c));
    return n;
  };
  const uint32_t k = rp.k_eff;
  uint32_t cut = 0;  // 0: fewer than k distinct vertices, all are kept
  if (n_with_count_at_least(1u) > k) {
    uint32_t lo = 1, hi = (uint32_t)(o * a);  // the largest c with at least k vertices visited c times or more
    while (lo < hi) {
      const uint32_t mid = lo + (hi - lo + 1) / 2;
      if (n_with_count_at_least(mid) >= k) lo = mid; else hi = mid - 1;
    }
    cut = lo;
  }
  bool keep[E];
  if (cut == 0) {
#pragma unroll
    for (int e = 0; e < E; ++e) keep[e] = cnt_e[e] != 0;
  } else {
    const uint32_t need = k - n_with_count_at_least(cut + 1);  // of the vertices visited exactly that often, the `need` smallest ids
    uint32_t tie[E];
#pragma unroll
    for (int e = 0; e < E; ++e) tie[e] = cnt_e[e] == cut ? id_e[e] : kRwEmpty;
    uint32_t lo = 0, hi = 0x7FFFFFFFu;  // the smallest X with at least `need` tie ids <= X (ids are distinct: exactly `need`)
    while (lo < hi) {
      const uint32_t mid = lo + (hi - lo) / 2;
      uint32_t n = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) n += (uint32_t)__popcll(ballot64(tie[e] <= mid));
      if (n >= need) hi = mid; else lo = mid + 1;
    }
#pragma unroll
    for (int e = 0; e < E; ++e) keep[e] = cnt_e[e] > cut || tie[e] <= lo;
  }
  // the kept entries, compacted into LDS as keys (count << 32 | ~vertex); an entry's place in the row is the number of
  // larger keys
  unsigned long long* kept_keys = reinterpret_cast<unsigned long long*>(keys);  // 64 E words of 8 bytes: the table's memory
  uint32_t n_kept = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const uint64_t mask = ballot64(keep[e]);
    if (keep[e]) kept_keys[n_kept + lanes_below(mask)] = ((unsigned long long)cnt_e[e] << 32) | (unsigned long long)(0xFFFFFFFFu - id_e[e]);
    n_kept += (uint32_t)__popcll(mask);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  StageEntry* row = rows + (size_t)w * rp.k_eff;
  for (uint32_t i = lane; i < n_kept; i += kWave) {
    const unsigned long long mine = kept_keys[i];
    uint32_t place = 0;
    for (uint32_t q = 0; q < n_kept; ++q) place += kept_keys[q] > mine;
    row[place] = StageEntry{(int32_t)(0xFFFFFFFFu - (uint32_t)mine), (uint32_t)(mine >> 32)};
  }
  if (lane == 0) cnt[w] = (int32_t)n_kept;
}

// ---- more than kRwMaxSteps steps per destination ---------------------------------------------------------------------
// The tally no longer fits a wave's share of LDS: it lives in device memory, one region of T slots (a power of two, at
// least twice the steps) per wave, and the waves stride over the destinations.  The same walks and the same selection,
// with passes over the table where the fast kernel has it in registers: the count of the k-th most visited vertex by
// bisection over counted passes, the id that cuts the ties likewise, the kept entries compacted into a list of their own
// and placed by rank.  A path for walk budgets in the thousands and beyond; not tuned.
__global__ __launch_bounds__(kBlock) void k_rw_walk_wide(const int64_t* __restrict__ g_indptr, const int32_t* __restrict__ g_indices,
                                                         int64_t n_vertices, const int32_t* __restrict__ dst, int64_t n_dst, RwParams rp,
                                                         uint32_t T, uint32_t* __restrict__ tables, unsigned long long* __restrict__ kept_all,
                                                         StageEntry* __restrict__ rows, int32_t* __restrict__ cnt, Ctl* ctl) {
  const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + uniform_wave_in_block();
  const uint32_t lane = (uint32_t)lane_id();
  uint32_t* keys = tables + (size_t)wave * 2u * T;
  uint32_t* counts = keys + T;
  unsigned long long* kept_keys = kept_all + (size_t)wave * rp.k_eff;
  const int o = rp.walk_length, a = rp.n_walks;
  const uint32_t k = rp.k_eff;
  for (int64_t w = wave; w < n_dst; w += n_waves) {
    for (uint32_t i = lane; i < T; i += kWave) { keys[i] = kRwEmpty; counts[i] = 0; }
    __threadfence();  // the cleared slots are in place before any lane's atomics reach them
    const int32_t s = dst[w];
    if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
      if (lane == 0) { atomicOr(&ctl->err_range, 1); cnt[w] = 0; }
      continue;
    }
    const int64_t s_beg = g_indptr[s];
    const uint32_t s_d = (uint32_t)(g_indptr[s + 1] - s_beg);
    if (s_d == 0) {  // wave-uniform
      if (lane == 0) cnt[w] = 0;
      continue;
    }
    const uint32_t sigma = mix32((uint32_t)s ^ rp.K[2]);
    for (int walk = (int)lane; walk < a; walk += kWave) {
      uint32_t cur = (uint32_t)s;
      for (int step = 0; step < o; ++step) {
        const uint32_t c = 2u * (uint32_t)(walk * o + step);
        const uint32_t u = rw_draw(rp.K, sigma, c);
        const bool restart = step == 0 || (uint64_t)rw_draw(rp.K, sigma, c + 1u) < rp.restart_thr;
        int64_t beg = s_beg;
        uint32_t d = s_d;
        if (!restart) {
          beg = g_indptr[cur];
          d = (uint32_t)(g_indptr[cur + 1] - beg);
        }
        if (d == 0) break;  // dead end: the walk ends
        cur = (uint32_t)g_indices[beg + (int64_t)(((uint64_t)u * (uint64_t)d) >> 32)];
        if ((uint64_t)cur >= (uint64_t)n_vertices) {  // a neighbour id outside the graph
          atomicOr(&ctl->err_range, 1);
          break;
        }
        uint32_t h = (cur * 0x9E3779B1u) >> 7 & (T - 1);
        for (;;) {  // at most o a <= T / 2 distinct vertices: an empty slot is always reached
          const uint32_t old = atomicCAS(&keys[h], kRwEmpty, cur);
          if (old == kRwEmpty || old == cur) { atomicAdd(&counts[h], 1u); break; }
          h = (h + 1) & (T - 1);
        }
      }
    }
    __threadfence();  // every lane's tallies are in the table before any lane reads it
    auto n_with_count_at_least = [&](uint32_t c) {
      uint32_t n = 0;
      for (uint32_t i = lane; i < T; i += kWave) n += __hip_atomic_load(&counts[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= c ? 1u : 0u;
      return (uint32_t)wave_sum_i64((int64_t)n);
    };
    uint32_t cut = 0;  // 0: at most k distinct vertices, all are kept
    if (n_with_count_at_least(1u) > k) {
      uint32_t lo = 1, hi = (uint32_t)(o * a);  // the largest c with at least k vertices visited c times or more
      while (lo < hi) {
        const uint32_t mid = lo + (hi - lo + 1) / 2;
        if (n_with_count_at_least(mid) >= k) lo = mid; else hi = mid - 1;
      }
      cut = lo;
    }
    uint32_t tie_max = 0x7FFFFFFFu;  // of the vertices visited exactly `cut` times, those with an id up to this are kept
    if (cut != 0) {
      const uint32_t need = k - n_with_count_at_least(cut + 1);
      uint32_t lo = 0, hi = 0x7FFFFFFFu;  // the smallest X with at least `need` tie ids <= X (ids are distinct: exactly `need`)
      while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        uint32_t n = 0;
        for (uint32_t i = lane; i < T; i += kWave) {
          const uint32_t c = __hip_atomic_load(&counts[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          n += (c == cut && __hip_atomic_load(&keys[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <= mid) ? 1u : 0u;
        }
        n = (uint32_t)wave_sum_i64((int64_t)n);
        if (n >= need) hi = mid; else lo = mid + 1;
      }
      tie_max = lo;
    }
    // the kept entries as keys (count << 32 | ~vertex), compacted; an entry's place in the row is the number of larger keys
    uint32_t n_kept = 0;
    for (uint32_t base = 0; base < T; base += kWave) {
      const uint32_t i = base + lane;  // (T is a multiple of 64)
      const uint32_t c = __hip_atomic_load(&counts[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t id = __hip_atomic_load(&keys[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const bool keep = c != 0 && (cut == 0 || c > cut || (c == cut && id <= tie_max));
      const uint64_t mask = ballot64(keep);
      const uint32_t at = n_kept + lanes_below(mask);
      if (keep && at < k) kept_keys[at] = ((unsigned long long)c << 32) | (unsigned long long)(0xFFFFFFFFu - id);  // (at < k always)
      n_kept += (uint32_t)__popcll(mask);
    }
    if (n_kept > k) n_kept = k;  // (holds by construction; keeps every access inside the row regardless)
    __threadfence();
    StageEntry* row = rows + (size_t)w * rp.k_eff;
    for (uint32_t i = lane; i < n_kept; i += kWave) {
      const unsigned long long mine = __hip_atomic_load(&kept_keys[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      uint32_t place = 0;
      for (uint32_t q = 0; q < n_kept; ++q) place += __hip_atomic_load(&kept_keys[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > mine;
      row[place] = StageEntry{(int32_t)(0xFFFFFFFFu - (uint32_t)mine), (uint32_t)(mine >> 32)};
    }
    if (lane == 0) cnt[w] = (int32_t)n_kept;
    __threadfence();  // the row is read out of kept_keys before the next destination writes there
  }
}

// staged rows -> the block's edge arrays; eid carries the visit count (these are edges of sum_i A^i, not of the graph)
__global__ __launch_bounds__(kBlock) void k_rw_fill(const StageEntry* __restrict__ rows, uint32_t k_eff, int64_t n_dst,
                                                    const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                    int64_t* __restrict__ eid, int64_t edge_limit) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t w = idx / k_eff;
  if (w >= n_dst) return;
  const int64_t slot = idx - w * k_eff;
  const int64_t o = eptr[w];
  if (slot >= eptr[w + 1] - o || o + slot >= edge_limit) return;
  const StageEntry e = rows[idx];
  col_global[o + slot] = e.t;
  eid[o + slot] = (int64_t)e.j;
}

int rw_layer(const SampleCtx& cx, const RwConfig& rw, int l, const int32_t* dst, int64_t n_dst, coop_block* blk, int64_t edge_cap) {
  const bool defer = edge_cap > 0;
  hipStream_t s = cx.s;
  Alloc& alloc = *cx.alloc;
  RwParams rp{};
  layer_keys(cx.seed, COOP_RW, l, cx.group, rp.K);
  rp.walk_length = rw.walk_length;
  rp.n_walks = rw.n_walks;
  rp.restart_thr = rw.restart_thr;
  const int64_t n_steps = (int64_t)rw.walk_length * rw.n_walks;
  rp.k_eff = (uint32_t)((int64_t)cx.fanouts[l] < n_steps ? cx.fanouts[l] : n_steps);

  blk->indptr = alloc.get<int64_t>(n_dst + 1, COOP_TAG_OUTPUT);
  int32_t* cnt = alloc.get<int32_t>(n_dst, COOP_TAG_SCRATCH);
  StageEntry* rows = alloc.get<StageEntry>(n_dst * (int64_t)rp.k_eff, COOP_TAG_SCRATCH);
  void* scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_dst), COOP_TAG_SCRATCH);
  if (alloc.failed) return COOP_E_NOMEM;
  if (n_dst > 0 && n_steps > kRwMaxSteps) {
    // the tally in device memory: T slots per wave, and as many waves as half a gigabyte of tables allows
    uint32_t T = 2048;
    while ((int64_t)T < 2 * n_steps) T <<= 1;
    const int64_t per_wave = 2 * (int64_t)T * 4 + (int64_t)rp.k_eff * 8;
    int64_t n_waves = ((int64_t)512 << 20) / per_wave;
    if (n_waves > 2048) n_waves = 2048;
    if (n_waves > n_dst) n_waves = n_dst;
    n_waves = (n_waves + kWavesPerBlock - 1) / kWavesPerBlock * kWavesPerBlock;  // whole blocks (at least one)
    if (n_waves < kWavesPerBlock) n_waves = kWavesPerBlock;
    uint32_t* tables = alloc.get<uint32_t>(n_waves * 2 * (int64_t)T, COOP_TAG_SCRATCH);
    unsigned long long* kept = alloc.get<unsigned long long>(n_waves * (int64_t)rp.k_eff, COOP_TAG_SCRATCH);
    if (alloc.failed) return COOP_E_NOMEM;
    COOP_LAUNCH(K_RW_WALK, k_rw_walk_wide, dim3((unsigned)(n_waves / kWavesPerBlock)), dim3(kBlock), 0, s, cx.g->indptr, cx.g->indices,
                cx.g->n_vertices, dst, n_dst, rp, T, tables, kept, rows, cnt, cx.d_ctl);
  } else if (n_dst > 0) {
    // table of 512 slots (up to 384 visits per destination, the paper's 3 x 100 included), else 2048
    if (n_steps <= 384) {
      const int wpb = kWavesPerBlock;
      COOP_LAUNCH(K_RW_WALK, k_rw_walk<8>, dim3(blocks_for(n_dst, wpb)), dim3(kBlock), (size_t)wpb * 2 * 512 * 4, s, cx.g->indptr,
                  cx.g->indices, cx.g->n_vertices, dst, n_dst, rp, wpb, rows, cnt, cx.d_ctl);
    } else {
      const int wpb = 2;
      COOP_LAUNCH(K_RW_WALK, k_rw_walk<32>, dim3(blocks_for(n_dst, wpb)), dim3(kBlock), (size_t)wpb * 2 * 2048 * 4, s, cx.g->indptr,
                  cx.g->indices, cx.g->n_vertices, dst, n_dst, rp, wpb, rows, cnt, cx.d_ctl);
    }
  }
  if (defer) {
    scan_i32_to_i64(cnt, n_dst, blk->indptr, &cx.d_ctl->total_edges, scan_tmp, s, nullptr);  // the count stays on the device
  } else {
    const Publish pub = begin_publish(cx.d_ctl, cx.h_ctl);  // the scan's last thread also sends the sizes to the host
    scan_i32_to_i64(cnt, n_dst, blk->indptr, &cx.d_ctl->total_edges, scan_tmp, s, &pub);  // m_l = indptr[n_dst]
    const int rc = wait_ctl(pub, cx.h_ctl, s);
    if (rc != COOP_OK) return rc;
  }
  const int64_t m = defer ? edge_cap : cx.h_ctl->total_edges;  // entries of the edge arrays
  blk->n_edges = defer ? -1 : m;
  blk->col_global = alloc.get<int32_t>(m, COOP_TAG_OUTPUT);
  blk->eid = alloc.get<int64_t>(m, COOP_TAG_OUTPUT);
  blk->col_local = alloc.get<int32_t>(m, COOP_TAG_OUTPUT);
  if (alloc.failed) return COOP_E_NOMEM;
  if (m > 0 && n_dst > 0)
    COOP_LAUNCH(K_RW_FILL, k_rw_fill, dim3(blocks_for(n_dst * (int64_t)rp.k_eff, kBlock)), dim3(kBlock), 0, s, rows, rp.k_eff, n_dst,
                blk->indptr, blk->col_global, blk->eid, m);
  return COOP_OK;
}

}  // namespace coop
