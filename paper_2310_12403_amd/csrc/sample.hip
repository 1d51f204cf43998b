// Sampling layers of Algorithm 1 on one GPU: per layer a count pass, a device-wide scan and a fill pass
// (one wave64 per destination vertex, coalesced reads of its neighbour list), then dedup + relabel.
//
//   LABOR-0 (App. A.1.2): edge (t -> s) is kept iff r_t <= k / d_s, i.e. R_t * d_s <= k * 2^32 in integers,
//                         which for d_s > k is R_t <= floor(k * 2^32 / d_s).
//   NS      (App. A.1.1): d_s <= k keeps N(s); otherwise the k neighbours with the smallest (R_ts, position).
// Kept edges leave in (destination order, adjacency order).
#include <math.h>

#include "coop_internal.h"
#include "device_utils.h"
#include "variates.h"

namespace coop {

// ---- LABOR-0 --------------------------------------------------------------------------------------------------
template <bool BLEND>
__global__ __launch_bounds__(kBlock) void k_labor_count(const int64_t* __restrict__ g_indptr,
                                                        const int32_t* __restrict__ g_indices, int64_t n_vertices,
                                                        const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k,
                                                        VariateParams vp, int32_t* __restrict__ cnt, Ctl* ctl) {
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
  uint32_t c;
  if (d <= (int64_t)k) {
    c = (uint32_t)d;
  } else {
    const uint32_t thr = (uint32_t)(((uint64_t)k << 32) / (uint64_t)d);
    c = 0;
    for (int64_t base = 0; base < d; base += kWave) {
      const int64_t j = base + lane;
      bool keep = false;
      if (j < d) {
        const uint32_t t = (uint32_t)g_indices[beg + j];
        keep = variate<BLEND>(vp, t, 0xFFFFFFFFu) <= thr;
      }
      c += (uint32_t)__popcll(ballot64(keep));
    }
  }
  if (lane == 0) cnt[w] = (int32_t)c;
}

template <bool BLEND>
__global__ __launch_bounds__(kBlock) void k_labor_fill(const int64_t* __restrict__ g_indptr,
                                                       const int32_t* __restrict__ g_indices,
                                                       const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k,
                                                       VariateParams vp, const int64_t* __restrict__ eptr,
                                                       int32_t* __restrict__ col_global, int64_t* __restrict__ eid) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + wave_in_block();
  if (w >= n_dst) return;
  const int lane = lane_id();
  int64_t o = eptr[w];
  const int64_t o_end = eptr[w + 1];
  if (o == o_end) return;  // nothing kept (also covers out-of-range seeds, whose count is 0)
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
  const uint32_t thr = (uint32_t)(((uint64_t)k << 32) / (uint64_t)d);
  for (int64_t base = 0; base < d; base += kWave) {
    const int64_t j = base + lane;
    bool keep = false;
    uint32_t t = 0;
    if (j < d) {
      t = (uint32_t)g_indices[beg + j];
      keep = variate<BLEND>(vp, t, 0xFFFFFFFFu) <= thr;
    }
    const uint64_t mask = ballot64(keep);
    if (keep) {
      const int64_t p = o + lanes_below(mask);
      col_global[p] = (int32_t)t;
      eid[p] = beg + j;
    }
    o += __popcll(mask);
  }
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
        r = variate<BLEND>(vp, (uint32_t)g_indices[beg + j], (uint32_t)s);
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

// ---- small copies ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_copy_i32(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = in[i];
}

__global__ void k_clear_ctl(Ctl* ctl) {
  ctl->total_edges = 0; ctl->total_new = 0; ctl->err_range = 0; ctl->err_dup = 0; ctl->err_capacity = 0; ctl->pad = 0;
}

static inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

static int read_ctl(Ctl* d_ctl, Ctl* h_ctl, hipStream_t s) {
  COOP_HIP_TRY(hipMemcpyAsync(h_ctl, d_ctl, sizeof(Ctl), hipMemcpyDeviceToHost, s));
  COOP_HIP_TRY(hipStreamSynchronize(s));
  if (h_ctl->err_range) return COOP_E_RANGE;
  if (h_ctl->err_dup) return COOP_E_DUPSEED;
  if (h_ctl->err_capacity) return COOP_E_CAPACITY;
  return COOP_OK;
}

}  // namespace coop

using namespace coop;

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

  // group / interpolation state of App. A.7
  VariateParams vp{};
  vp.key0 = (uint32_t)seed;
  vp.key1 = (uint32_t)(seed >> 32);
  bool blend = false;
  vp.g = 0; vp.cw = 1.0; vp.sw = 0.0;
  if (kappa != 0) {
    const uint64_t i = iter % kappa;
    vp.g = (uint32_t)(iter / kappa);
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
    vp.c2 = (uint32_t)l | ((uint32_t)sampler << 8);
    coop_block blk{};
    blk.n_dst = n_dst;
    blk.dst_ids = const_cast<int32_t*>(dst);
    blk.indptr = alloc.get<int64_t>(n_dst + 1, COOP_TAG_OUTPUT);
    int32_t* cnt = alloc.get<int32_t>(n_dst, COOP_TAG_SCRATCH);
    void* scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_dst), COOP_TAG_SCRATCH);
    if (alloc.failed) { rc = COOP_E_NOMEM; break; }

    // count pass
    if (n_dst > 0) {
      if (sampler == COOP_LABOR0) {
        const dim3 grid(blocks_for(n_dst, kWavesPerBlock));
        if (blend)
          COOP_LAUNCH(K_LABOR_COUNT, k_labor_count<true>, grid, dim3(kBlock), 0, s, g->indptr, g->indices, g->n_vertices, dst,
                      n_dst, k, vp, cnt, d_ctl);
        else
          COOP_LAUNCH(K_LABOR_COUNT, k_labor_count<false>, grid, dim3(kBlock), 0, s, g->indptr, g->indices, g->n_vertices, dst,
                      n_dst, k, vp, cnt, d_ctl);
      } else {
        COOP_LAUNCH(K_NS_COUNT, k_ns_count, dim3(blocks_for(n_dst, kBlock)), dim3(kBlock), 0, s, g->indptr, g->n_vertices, dst,
                    n_dst, k, cnt, d_ctl);
      }
    }
    scan_i32_to_i64(cnt, n_dst, blk.indptr, scan_tmp, s);
    // m_l = indptr[n_dst]
    COOP_HIP_TRY(hipMemcpyAsync(&d_ctl->total_edges, blk.indptr + n_dst, sizeof(int64_t), hipMemcpyDeviceToDevice, s));
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
        const dim3 grid(blocks_for(n_dst, kWavesPerBlock));
        if (blend)
          COOP_LAUNCH(K_LABOR_FILL, k_labor_fill<true>, grid, dim3(kBlock), 0, s, g->indptr, g->indices, dst, n_dst, k, vp,
                      blk.indptr, blk.col_global, blk.eid);
        else
          COOP_LAUNCH(K_LABOR_FILL, k_labor_fill<false>, grid, dim3(kBlock), 0, s, g->indptr, g->indices, dst, n_dst, k, vp,
                      blk.indptr, blk.col_global, blk.eid);
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
