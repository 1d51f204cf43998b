// Sampling layers of Algorithm 1 on one GPU.  Per layer: a neighbour-scan pass (one wave64 per destination vertex,
// 16-byte coalesced reads of its neighbour list), a device-wide scan of the per-destination counts, a fill pass,
// then dedup + relabel (unique.hip).
//
//   LABOR-0 (App. A.1.2): edge (t -> s) is kept iff r_t <= k / d_s, i.e. R_t * d_s <= k * 2^32 in integers,
//                         which for d_s > k is R_t <= floor(k * 2^32 / d_s).
//   NS      (App. A.1.1): d_s <= k keeps N(s); otherwise the k neighbours with the smallest (R_ts, position).
// Kept edges leave in (destination order, adjacency order).
//
// LABOR-0 examines every neighbour once: the scan pass parks the kept (vertex, position) pairs of each destination
// in a small per-destination staging row, so the fill pass is a copy and the adjacency is not read again.  A row
// that overflows (more kept edges than the row holds) is rare and handled by a second scan of just those lists.
#include <math.h>

#include "coop_internal.h"
#include "device_utils.h"
#include "variates.h"

namespace coop {

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Visits the neighbour list [beg, beg + d) of one destination with the whole wave and calls emit(rank, t, j) for
// every kept neighbour t at list position j; rank counts kept neighbours in adjacency order.  `all` keeps
// everything (d <= k).  Returns the number kept (same value in every lane).
//
// VEC == 4: the list is read as 16-byte aligned groups of four entries, two groups per lane and step (2 KiB per
// wave and step), with the next step's groups requested before the current ones are hashed.  Positions are kept
// relative to the first aligned group, so one unsigned compare tells whether an entry belongs to the list.
template <bool BLEND, int VEC, typename Emit>
__device__ __forceinline__ uint32_t labor_scan_list(const int32_t* __restrict__ g_indices, int64_t n_edges_total, int64_t beg,
                                                    int64_t d64, bool all, uint32_t thr, const VariateParams& vp, Emit emit) {
  const int lane = lane_id();
  const uint32_t d = (uint32_t)d64;
  uint32_t count = 0;
  if (all || VEC == 1) {
    for (uint32_t base = 0; base < d; base += kWave) {
      const uint32_t j = base + lane;
      bool kp = j < d;
      int32_t t = 0;
      if (kp) {
        t = g_indices[beg + j];
        if (!all) kp = variate<false, BLEND>(vp, (uint32_t)t, 0u, 0u) <= thr;
      }
      const uint64_t m = ballot64(kp);
      if (kp) emit(count + lanes_below(m), t, j);
      count += (uint32_t)__popcll(m);
    }
    return count;
  }
  constexpr int kGroups = 2;                    // 16-byte groups per lane and step
  constexpr uint32_t kStep = kWave * 4 * kGroups;
  const int64_t abeg = beg & ~(int64_t)3;       // first aligned group
  const uint32_t head = (uint32_t)(beg - abeg); // entries of that group that precede the list
  const uint32_t total = head + d;              // list end, relative to abeg
  const int32_t* __restrict__ p = g_indices + abeg;
  // entries readable from p without leaving the array (the last group of the whole array may be partial)
  const int64_t avail = n_edges_total - abeg;

  auto load_group = [&](uint32_t r) -> i32x4 {  // r: relative index of the group's first entry, multiple of 4
    i32x4 v = {0, 0, 0, 0};
    if (r < total) {
      if ((int64_t)r + 3 < avail) {
        v = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(p + r));
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((int64_t)r + e < avail) v[e] = p[r + e];
      }
    }
    return v;
  };

  i32x4 nxt[kGroups];
#pragma unroll
  for (int gq = 0; gq < kGroups; ++gq) nxt[gq] = load_group((uint32_t)(gq * kWave * 4 + lane * 4));
  for (uint32_t base = 0; base < total; base += kStep) {
    i32x4 cur[kGroups];
#pragma unroll
    for (int gq = 0; gq < kGroups; ++gq) cur[gq] = nxt[gq];
    if (base + kStep < total) {
#pragma unroll
      for (int gq = 0; gq < kGroups; ++gq) nxt[gq] = load_group(base + kStep + (uint32_t)(gq * kWave * 4 + lane * 4));
    }
#pragma unroll
    for (int gq = 0; gq < kGroups; ++gq) {
      const uint32_t r = base + (uint32_t)(gq * kWave * 4 + lane * 4);
      bool keep[4];
      uint64_t m[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t j = r + e - head;  // position in the list; wraps to a huge value in front of the list
        const uint32_t R = variate<false, BLEND>(vp, (uint32_t)cur[gq][e], 0u, 0u);
        keep[e] = (j < d) & (R <= thr);
        m[e] = ballot64(keep[e]);
      }
      if ((m[0] | m[1] | m[2] | m[3]) != 0) {
        uint32_t rank = count + lanes_below(m[0]) + lanes_below(m[1]) + lanes_below(m[2]) + lanes_below(m[3]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (keep[e]) {
            emit(rank, cur[gq][e], r + e - head);
            ++rank;
          }
        }
        count += (uint32_t)(__popcll(m[0]) + __popcll(m[1]) + __popcll(m[2]) + __popcll(m[3]));
      }
    }
  }
  return count;
}

struct StageEntry { int32_t t; uint32_t j; };  // kept source vertex, its position in the destination's list

// ---- LABOR-0 --------------------------------------------------------------------------------------------------
template <bool BLEND, int VEC>
__global__ __launch_bounds__(kBlock) void k_labor_count(const int64_t* __restrict__ g_indptr,
                                                        const int32_t* __restrict__ g_indices, int64_t n_vertices,
                                                        int64_t n_edges_total, const int32_t* __restrict__ dst, int64_t n_dst,
                                                        uint32_t k, VariateParams vp, uint32_t stage_cap,
                                                        StageEntry* __restrict__ stage, int32_t* __restrict__ cnt, Ctl* ctl) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + wave_in_block();
  if (w >= n_dst) return;
  const int lane = lane_id();
  const int32_t s = dst[w];
  if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
    if (lane == 0) { atomicOr(&ctl->err_range, 1); cnt[w] = 0; }
    return;
  }
  const int64_t beg = g_indptr[s];
  const int64_t d = g_indptr[s + 1] - beg;
  const bool all = d <= (int64_t)k;
  const uint32_t thr = all ? 0xFFFFFFFFu : (uint32_t)(((uint64_t)k << 32) / (uint64_t)d);
  StageEntry* row = stage + (size_t)w * stage_cap;
  const uint32_t c = labor_scan_list<BLEND, VEC>(g_indices, n_edges_total, beg, d, all, thr, vp,
                                                 [&](uint32_t rank, int32_t t, uint32_t j) {
                                                   if (rank < stage_cap) row[rank] = StageEntry{t, j};
                                                 });
  if (lane == 0) {
    cnt[w] = (int32_t)c;
    if (c > stage_cap) atomicAdd(&ctl->n_overflow, 1);
  }
}

// copy of the staged rows into the block's edge arrays: one thread per (destination, row slot)
__global__ __launch_bounds__(kBlock) void k_labor_fill_staged(const int64_t* __restrict__ g_indptr,
                                                              const int32_t* __restrict__ dst, int64_t n_dst,
                                                              int stage_cap_log2, const StageEntry* __restrict__ stage,
                                                              const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                              int64_t* __restrict__ eid) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t w = idx >> stage_cap_log2;
  if (w >= n_dst) return;
  const int64_t slot = idx & (((int64_t)1 << stage_cap_log2) - 1);
  const int64_t o = eptr[w];
  const int64_t c = eptr[w + 1] - o;
  if (slot >= c || c > ((int64_t)1 << stage_cap_log2)) return;
  const StageEntry e = stage[idx];
  col_global[o + slot] = e.t;
  eid[o + slot] = g_indptr[dst[w]] + e.j;
}

// second scan of the (rare) destinations whose staging row overflowed, writing straight to the edge arrays
template <bool BLEND, int VEC>
__global__ __launch_bounds__(kBlock) void k_labor_fill_overflow(const int64_t* __restrict__ g_indptr,
                                                                const int32_t* __restrict__ g_indices, int64_t n_edges_total,
                                                                const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k,
                                                                VariateParams vp, uint32_t stage_cap,
                                                                const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                                int64_t* __restrict__ eid) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + wave_in_block();
  if (w >= n_dst) return;
  const int64_t o = eptr[w];
  if (eptr[w + 1] - o <= (int64_t)stage_cap) return;
  const int32_t s = dst[w];
  const int64_t beg = g_indptr[s];
  const int64_t d = g_indptr[s + 1] - beg;
  const bool all = d <= (int64_t)k;
  const uint32_t thr = all ? 0xFFFFFFFFu : (uint32_t)(((uint64_t)k << 32) / (uint64_t)d);
  labor_scan_list<BLEND, VEC>(g_indices, n_edges_total, beg, d, all, thr, vp, [&](uint32_t rank, int32_t t, uint32_t j) {
    col_global[o + rank] = t;
    eid[o + rank] = beg + j;
  });
}

// ---- NS -------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_ns_count(const int64_t* __restrict__ g_indptr, int64_t n_vertices,
                                                     const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k,
                                                     int32_t* __restrict__ cnt, Ctl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_dst) return;
  const int32_t s = dst[i];
  if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
    atomicOr(&ctl->err_range, 1);
    cnt[i] = 0;
    return;
  }
  const int64_t d = g_indptr[s + 1] - g_indptr[s];
  cnt[i] = (int32_t)(d < (int64_t)k ? d : (int64_t)k);
}

constexpr uint32_t kNsMaxSelect = 1024;  // largest fanout for which a longer list can be subsampled

// Selection of the k smallest (R, j) among d > k neighbours, one wave per destination:
//   1. one pass over the list keeps, in LDS and in adjacency order, the candidates with R <= bound, where bound is
//      chosen so that about `target` of them are expected (target > k, target < cap);
//   2. if fewer than k or more than cap candidates turn up, the bound is bisected and the pass repeated (rare);
//   3. each candidate's rank among the candidates is counted; ranks below k are emitted, still in adjacency order.
template <bool BLEND>
__global__ __launch_bounds__(kBlock) void k_ns_fill(const int64_t* __restrict__ g_indptr,
                                                    const int32_t* __restrict__ g_indices,
                                                    const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k,
                                                    uint32_t cap, uint32_t target, int waves_per_block, VariateParams vp,
                                                    const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                    int64_t* __restrict__ eid, Ctl* ctl) {
  extern __shared__ uint64_t lds_keys[];  // per wave: cap variates (u32) followed by cap list positions (u32)
  const int wib = wave_in_block();
  if (wib >= waves_per_block) return;
  const int64_t w = (int64_t)blockIdx.x * waves_per_block + wib;
  if (w >= n_dst) return;
  const int lane = lane_id();
  int64_t o = eptr[w];
  if (o == eptr[w + 1]) return;
  const int32_t s = dst[w];
  const int64_t beg = g_indptr[s];
  const int64_t d = g_indptr[s + 1] - beg;
  if (d <= (int64_t)k) {
    for (int64_t j = lane; j < d; j += kWave) {
      col_global[o + j] = g_indices[beg + j];
      eid[o + j] = beg + j;
    }
    return;
  }
  if (k > kNsMaxSelect) {  // a degree above a fanout that the candidate buffer cannot serve
    if (lane == 0) atomicOr(&ctl->err_capacity, 1);
    return;
  }
  uint32_t* cand_r = (uint32_t*)(lds_keys + (size_t)wib * cap);  // [cap] variates
  uint32_t* cand_j = cand_r + cap;                               // [cap] positions (d < 2^31)
  const uint32_t sigma_a = ns_sigma(vp.Ka, (uint32_t)s);
  const uint32_t sigma_b = BLEND ? ns_sigma(vp.Kb, (uint32_t)s) : 0u;

  // bound such that E[#candidates] = target: R <= bound with probability (bound + 1) / 2^32
  uint64_t lo = 0, hi = 0xFFFFFFFFull;  // bisection bracket on the bound, used only after a failed pass
  uint64_t bound = ((uint64_t)target << 32) / (uint64_t)d;
  if (bound > 0xFFFFFFFFull || (uint64_t)d <= cap) bound = 0xFFFFFFFFull;
  uint32_t n_c = 0;
  for (int attempt = 0; attempt < 40; ++attempt) {
    n_c = 0;
    for (int64_t base = 0; base < d; base += kWave) {
      const int64_t j = base + lane;
      bool in = false;
      uint32_t r = 0;
      if (j < d) {
        r = variate<true, BLEND>(vp, (uint32_t)g_indices[beg + j], sigma_a, sigma_b);
        in = r <= (uint32_t)bound;
      }
      const uint64_t mask = ballot64(in);
      const uint32_t p = n_c + lanes_below(mask);
      if (in && p < cap) { cand_r[p] = r; cand_j[p] = (uint32_t)j; }
      n_c += (uint32_t)__popcll(mask);
    }
    if (n_c >= k && n_c <= cap) break;
    // cannot be bracketed (more than cap - k equal variates): report instead of guessing
    if (n_c < k) {
      if (bound >= 0xFFFFFFFFull) { n_c = 0; break; }
      lo = bound + 1;
    } else {
      if (bound == 0) { n_c = 0; break; }
      hi = bound - 1;
    }
    if (lo > hi) { n_c = 0; break; }
    bound = lo + (hi - lo) / 2;
  }
  if (n_c < k || n_c > cap) {
    if (lane == 0) atomicOr(&ctl->err_capacity, 1);
    return;
  }
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  // rank counting; candidates are in adjacency order, so ties on R are broken by list position for free
  for (uint32_t base = 0; base < n_c; base += kWave) {
    const uint32_t i = base + lane;
    bool keep = false;
    uint32_t my_j = 0;
    if (i < n_c) {
      const uint32_t my_r = cand_r[i];
      my_j = cand_j[i];
      uint32_t rank = 0;
      for (uint32_t q = 0; q < n_c; ++q) {
        const uint32_t r = cand_r[q];
        rank += (r < my_r) || (r == my_r && q < i);
      }
      keep = rank < k;
    }
    const uint64_t mask = ballot64(keep);
    if (keep) {
      const int64_t p = o + lanes_below(mask);
      col_global[p] = g_indices[beg + my_j];
      eid[p] = beg + my_j;
    }
    o += __popcll(mask);
  }
}

// ---- small kernels --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_copy_i32(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = in[i];
}

__global__ void k_clear_ctl(Ctl* ctl) { *ctl = Ctl{}; }

__global__ void k_publish_edges(Ctl* ctl, const int64_t* __restrict__ total) { ctl->total_edges = *total; }

static inline unsigned blocks_for(int64_t n, int64_t per_block) { return (unsigned)((n + per_block - 1) / per_block); }

static int read_ctl(Ctl* d_ctl, Ctl* h_ctl, hipStream_t s) {
  COOP_HIP_TRY(hipMemcpyAsync(h_ctl, d_ctl, sizeof(Ctl), hipMemcpyDeviceToHost, s));
  COOP_HIP_TRY(hipStreamSynchronize(s));
  if (h_ctl->err_range) return COOP_E_RANGE;
  if (h_ctl->err_dup) return COOP_E_DUPSEED;
  if (h_ctl->err_capacity) return COOP_E_CAPACITY;
  return COOP_OK;
}

int g_stage_cap_override = 0;  // COOP_TUNE_STAGE_CAP

}  // namespace coop

using namespace coop;

extern "C" int coop_tune(int knob, int64_t value) {
  switch (knob) {
    case COOP_TUNE_STAGE_CAP:
      if (value != 0 && (value < 1 || value > 4096 || (value & (value - 1)))) return COOP_E_ARG;
      g_stage_cap_override = (int)value;
      return COOP_OK;
    default:
      return COOP_E_ARG;
  }
}

// dispatch on (BLEND, VEC)
#define COOP_LABOR_DISPATCH(id, name, grid, ...)                                                                    \
  do {                                                                                                              \
    if (blend) {                                                                                                    \
      if (vec4) COOP_LAUNCH(id, (name<true, 4>), grid, dim3(kBlock), 0, s, __VA_ARGS__);                            \
      else COOP_LAUNCH(id, (name<true, 1>), grid, dim3(kBlock), 0, s, __VA_ARGS__);                                 \
    } else {                                                                                                        \
      if (vec4) COOP_LAUNCH(id, (name<false, 4>), grid, dim3(kBlock), 0, s, __VA_ARGS__);                           \
      else COOP_LAUNCH(id, (name<false, 1>), grid, dim3(kBlock), 0, s, __VA_ARGS__);                                \
    }                                                                                                               \
  } while (0)

extern "C" int coop_sample(const coop_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int L,
                           int sampler, uint64_t iter, uint32_t kappa, uint64_t seed, coop_alloc_fn alloc_fn,
                           void* alloc_ctx, void* stream, coop_block* blocks_out) {
  if (!g || !fanouts || !blocks_out || !alloc_fn || (!seeds && n_seeds > 0)) return COOP_E_NULL;
  if (L < 1 || L > 255 || n_seeds < 0 || n_seeds >= ((int64_t)1 << 31)) return COOP_E_ARG;
  if (sampler != COOP_NS && sampler != COOP_LABOR0) return COOP_E_ARG;
  for (int l = 0; l < L; ++l)
    if (fanouts[l] < 1) return COOP_E_ARG;
  for (int l = 0; l < L; ++l) blocks_out[l] = coop_block{};

  hipStream_t s = (hipStream_t)stream;
  Alloc alloc{alloc_fn, alloc_ctx};
  const bool vec4 = ((uintptr_t)g->indices & 15) == 0;

  // group / interpolation state of App. A.7: g = floor(iter / kappa), c = (iter mod kappa) / kappa
  VariateParams vp{};
  uint64_t group = 0;
  bool blend = false;
  vp.cw = 1.0; vp.sw = 0.0;
  if (kappa != 0) {
    const uint64_t i = iter % kappa;
    group = iter / kappa;
    blend = i != 0;
    const double c = (double)i / (double)kappa;
    vp.cw = cos(c * 1.5707963267948966);
    vp.sw = sin(c * 1.5707963267948966);
  }

  // pinned landing pad for the size read-backs, one per calling thread, kept for the life of the process
  static thread_local Ctl* h_ctl = nullptr;
  if (!h_ctl) COOP_HIP_TRY(hipHostMalloc((void**)&h_ctl, sizeof(Ctl), hipHostMallocDefault));
  Ctl* d_ctl = alloc.get<Ctl>(1, COOP_TAG_SCRATCH);
  int32_t* seed_copy = alloc.get<int32_t>(n_seeds, COOP_TAG_OUTPUT);
  if (alloc.failed) return COOP_E_NOMEM;
  COOP_LAUNCH(K_FILL, k_clear_ctl, dim3(1), dim3(1), 0, s, d_ctl);
  if (n_seeds > 0)
    COOP_LAUNCH(K_COPY_IDS, k_copy_i32, dim3(blocks_for(n_seeds, kBlock)), dim3(kBlock), 0, s, seeds, seed_copy, n_seeds);

  const int32_t* dst = seed_copy;
  int64_t n_dst = n_seeds;
  int rc = COOP_OK;
  for (int l = 0; l < L && rc == COOP_OK; ++l) {
    const uint32_t k = (uint32_t)fanouts[l];
    layer_keys(seed, sampler, l, group, vp.Ka);
    layer_keys(seed, sampler, l, group + 1, vp.Kb);
    coop_block blk{};
    blk.n_dst = n_dst;
    blk.dst_ids = const_cast<int32_t*>(dst);
    blk.indptr = alloc.get<int64_t>(n_dst + 1, COOP_TAG_OUTPUT);
    int32_t* cnt = alloc.get<int32_t>(n_dst, COOP_TAG_SCRATCH);
    void* scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_dst), COOP_TAG_SCRATCH);

    // LABOR-0 staging rows: room for 2k + 16 kept edges (a row overflows with probability < 1e-8 at k = 10),
    // between 32 and 256 entries, shrunk while the whole staging area would exceed 1 GiB
    uint32_t stage_cap = 32;
    int stage_cap_log2 = 5;
    StageEntry* stage = nullptr;
    if (sampler == COOP_LABOR0) {
      while (stage_cap < 2 * (uint64_t)k + 16 && stage_cap < 256) { stage_cap <<= 1; ++stage_cap_log2; }
      while (stage_cap > 32 && (uint64_t)n_dst * stage_cap * sizeof(StageEntry) > ((uint64_t)1 << 30)) { stage_cap >>= 1; --stage_cap_log2; }
      if (g_stage_cap_override) {
        stage_cap = (uint32_t)g_stage_cap_override;
        stage_cap_log2 = 0;
        while ((1u << stage_cap_log2) < stage_cap) ++stage_cap_log2;
      }
      stage = alloc.get<StageEntry>(n_dst * (int64_t)stage_cap, COOP_TAG_SCRATCH);
    }
    if (alloc.failed) { rc = COOP_E_NOMEM; break; }

    // neighbour scan / count pass
    if (n_dst > 0) {
      if (sampler == COOP_LABOR0) {
        const dim3 grid(blocks_for(n_dst, kWavesPerBlock));
        COOP_LABOR_DISPATCH(K_LABOR_COUNT, k_labor_count, grid, g->indptr, g->indices, g->n_vertices, g->n_edges, dst, n_dst, k,
                            vp, stage_cap, stage, cnt, d_ctl);
      } else {
        COOP_LAUNCH(K_NS_COUNT, k_ns_count, dim3(blocks_for(n_dst, kBlock)), dim3(kBlock), 0, s, g->indptr, g->n_vertices, dst,
                    n_dst, k, cnt, d_ctl);
      }
    }
    scan_i32_to_i64(cnt, n_dst, blk.indptr, scan_tmp, s);
    COOP_LAUNCH(K_FILL, k_publish_edges, dim3(1), dim3(1), 0, s, d_ctl, blk.indptr + n_dst);  // m_l = indptr[n_dst]
    rc = read_ctl(d_ctl, h_ctl, s);
    if (rc != COOP_OK) break;
    const int64_t m = h_ctl->total_edges;
    if (n_dst + m >= ((int64_t)1 << 32) - 1) { rc = COOP_E_CAPACITY; break; }
    blk.n_edges = m;
    blk.col_global = alloc.get<int32_t>(m, COOP_TAG_OUTPUT);
    blk.eid = alloc.get<int64_t>(m, COOP_TAG_OUTPUT);
    blk.col_local = alloc.get<int32_t>(m, COOP_TAG_OUTPUT);
    if (alloc.failed) { rc = COOP_E_NOMEM; break; }

    // fill pass
    if (m > 0) {
      if (sampler == COOP_LABOR0) {
        COOP_LAUNCH(K_LABOR_FILL, k_labor_fill_staged, dim3(blocks_for(n_dst * (int64_t)stage_cap, kBlock)), dim3(kBlock), 0, s,
                    g->indptr, dst, n_dst, stage_cap_log2, stage, blk.indptr, blk.col_global, blk.eid);
        if (h_ctl->n_overflow > 0) {
          const dim3 grid(blocks_for(n_dst, kWavesPerBlock));
          COOP_LABOR_DISPATCH(K_LABOR_OVERFLOW, k_labor_fill_overflow, grid, g->indptr, g->indices, g->n_edges, dst, n_dst, k, vp,
                              stage_cap, blk.indptr, blk.col_global, blk.eid);
        }
      } else {
        // candidate buffer: cap >= 4k (power of two, at least 256); expected candidates: 3k + 24.  A fanout above
        // kNsMaxSelect is served only while no degree exceeds it (the kernel reports the first that does).
        const uint32_t k_sel = k < kNsMaxSelect ? k : kNsMaxSelect;
        uint32_t cap = 256;
        while (cap < 4 * k_sel) cap <<= 1;
        const uint32_t target = 3 * k_sel + 24;
        int wpb = kWavesPerBlock;
        while (wpb > 1 && (size_t)wpb * cap * 8 > 32768) wpb >>= 1;
        const size_t shmem = (size_t)wpb * cap * 8;
        const dim3 grid(blocks_for(n_dst, wpb));
        if (blend)
          COOP_LAUNCH(K_NS_FILL, k_ns_fill<true>, grid, dim3(kBlock), shmem, s, g->indptr, g->indices, dst, n_dst, k, cap, target,
                      wpb, vp, blk.indptr, blk.col_global, blk.eid, d_ctl);
        else
          COOP_LAUNCH(K_NS_FILL, k_ns_fill<false>, grid, dim3(kBlock), shmem, s, g->indptr, g->indices, dst, n_dst, k, cap, target,
                      wpb, vp, blk.indptr, blk.col_global, blk.eid, d_ctl);
      }
    }

    // S^{l+1} and local ids (Eq. 2)
    int32_t* src = nullptr;
    int64_t n_src = 0;
    rc = unique_relabel(dst, n_dst, blk.col_global, m, blk.col_local, &src, &n_src, alloc, d_ctl, h_ctl, s);
    if (rc != COOP_OK) break;
    blk.src_ids = src;
    blk.n_src = n_src;
    blocks_out[l] = blk;
    dst = src;
    n_dst = n_src;
  }
  if (rc != COOP_OK) {
    (void)hipStreamSynchronize(s);
    for (int l = 0; l < L; ++l) blocks_out[l] = coop_block{};
  }
  return rc;
}
