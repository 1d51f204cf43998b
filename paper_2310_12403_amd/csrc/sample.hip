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

// One destination's neighbour list as the scan kernels see it: where it starts, how long it is, and the LABOR-0
// keep threshold floor(k 2^32 / d) (all ones when d <= k: everything is kept).  Built by k_segments, one coalesced
// 16-byte record per destination, so that a wave can fetch the records of all its lists with one load.
struct Segment { int64_t beg; uint32_t d; uint32_t thr; };

struct StageEntry { int32_t t; uint32_t j; };  // kept source vertex, its position in the destination's list

constexpr uint32_t kAllThr = 0xFFFFFFFFu;
constexpr int kScanGroups = 4;  // 16-byte groups per lane and step of the fast scan (4 KiB per wave and step)

__global__ __launch_bounds__(kBlock) void k_segments(const int64_t* __restrict__ g_indptr, int64_t n_vertices,
                                                     const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k,
                                                     Segment* __restrict__ seg, int32_t* __restrict__ ns_cnt, Ctl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_dst) return;
  const int32_t s = dst[i];
  Segment g{0, 0, kAllThr};
  if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
    atomicOr(&ctl->err_range, 1);
  } else {
    g.beg = g_indptr[s];
    g.d = (uint32_t)(g_indptr[s + 1] - g.beg);
    if (g.d > k) g.thr = (uint32_t)(((uint64_t)k << 32) / (uint64_t)g.d);
  }
  seg[i] = g;
  if (ns_cnt) ns_cnt[i] = (int32_t)(g.d < k ? g.d : k);  // NS: min(k, d) edges
}

// Ordered visit of the neighbour list [beg, beg + d) of one destination by the whole wave, one entry per lane and
// step: calls emit(rank, t, j) for every kept neighbour t at list position j, rank counting kept neighbours in
// adjacency order.  `all` keeps everything (d <= k).  Returns the number kept (same value in every lane).
// Used for short lists, for an indices array that is not 16-byte aligned, and for the overflow pass.
template <bool BLEND, typename Emit>
__device__ __forceinline__ uint32_t labor_scan_ordered(const int32_t* __restrict__ g_indices, int64_t beg, uint32_t d, bool all,
                                                       uint32_t thr, const VariateParams& vp, Emit emit) {
  const int lane = lane_id();
  uint32_t count = 0;
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

// Fast scan of a long list.  The list is read as 16-byte aligned groups of four entries, kScanGroups groups per lane
// and step (4 KiB per wave and step), all requested before the first is hashed.  Positions are relative to the first
// aligned group; steps that lie wholly inside the list (all but the first and the last) need no bounds test.  Per
// entry the hot loop is the mixer and one compare; one ballot per group tells whether any lane kept anything.  Only
// then are the (few) kept entries picked off per-entry ballot masks by a wave-uniform loop and parked in lane
// `count` of a register pair (ent_t, ent_j): up to 64 kept entries per list, in no particular order.
template <bool CHECK, bool BLEND>
__device__ __forceinline__ void labor_stage_step(const i32x4 (&cur)[kScanGroups], uint32_t base, uint32_t head, uint32_t d,
                                                 uint32_t thr, const VariateParams& vp, int32_t& ent_t, int32_t& ent_j,
                                                 uint32_t& count) {
  const uint32_t lane = (uint32_t)lane_id();
#pragma unroll
  for (int gq = 0; gq < kScanGroups; ++gq) {
    const uint32_t r0 = base + (uint32_t)(gq * kWave * 4);  // wave-uniform
    bool f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t R = variate<false, BLEND>(vp, (uint32_t)cur[gq][e], 0u, 0u);
      f[e] = R <= thr;
      if (CHECK) f[e] &= (r0 + lane * 4 + e - head) < d;  // position in the list; wraps to a huge value in front of it
    }
    if (ballot64(f[0] | f[1] | f[2] | f[3]) != 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        uint64_t mm = ballot64(f[e]);
        while (mm != 0) {
          const int src_lane = __builtin_ctzll(mm);
          mm &= mm - 1;
          const int32_t t = __builtin_amdgcn_readlane(cur[gq][e], src_lane);
          const int32_t j = (int32_t)(r0 + (uint32_t)src_lane * 4 + e - head);
          if (lane == (count & 63u)) { ent_t = t; ent_j = j; }
          ++count;
        }
      }
    }
  }
}

// returns the number kept; if it is at most min(stage_cap, 64) the kept entries are written to `row` in adjacency order
template <bool BLEND>
__device__ __forceinline__ uint32_t labor_scan_staged(const int32_t* __restrict__ g_indices, int64_t beg, uint32_t d, uint32_t thr,
                                                      const VariateParams& vp, StageEntry* __restrict__ row, uint32_t stage_cap) {
  constexpr uint32_t kStep = kWave * 4 * kScanGroups;
  const int64_t abeg = beg & ~(int64_t)3;         // first aligned group
  const uint32_t head = (uint32_t)(beg - abeg);   // entries of that group that precede the list
  const uint32_t total = head + d;                // list end, relative to abeg
  const uint32_t vec_end = total & ~3u;           // groups that start below this end inside the list
  const int32_t* __restrict__ p = g_indices + abeg;
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t lane4 = lane * 4;
  uint32_t count = 0;
  int32_t ent_t = 0, ent_j = 0;

  for (uint32_t base = 0; base < total; base += kStep) {
    i32x4 buf[kScanGroups];
#pragma unroll
    for (int gq = 0; gq < kScanGroups; ++gq) {
      const uint32_t r = base + (uint32_t)(gq * kWave * 4) + lane4;
      i32x4 v = {0, 0, 0, 0};
      if (r < vec_end) {
        v = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(p + r));
      } else if (r < total) {  // the list's last, partial group: entry by entry, never past the list
#pragma unroll
        for (int e = 0; e < 3; ++e)
          if (r + e < total) v[e] = p[r + e];
      }
      buf[gq] = v;
    }
    if (base >= head && base + kStep <= total) labor_stage_step<false, BLEND>(buf, base, head, d, thr, vp, ent_t, ent_j, count);
    else labor_stage_step<true, BLEND>(buf, base, head, d, thr, vp, ent_t, ent_j, count);
  }
  // adjacency order: an entry's place is the number of kept entries in front of it in the list
  if (count <= stage_cap && count <= (uint32_t)kWave) {
    uint32_t rank = 0;
    for (uint32_t q = 0; q < count; ++q) rank += (uint32_t)(__builtin_amdgcn_readlane(ent_j, (int)q) < ent_j);
    if (lane < count) row[rank] = StageEntry{ent_t, (uint32_t)ent_j};
  }
  return count;
}

// ---- LABOR-0 --------------------------------------------------------------------------------------------------
// Each wave takes `lists_per_wave` consecutive destinations: their segment records are fetched by one coalesced load
// (lane i holds record i), so the pointer chase destination -> list start is paid once per wave, not once per list.
template <bool BLEND, int VEC>
__global__ __launch_bounds__(kBlock) void k_labor_count(const int32_t* __restrict__ g_indices, const Segment* __restrict__ seg,
                                                        int64_t n_dst, int lists_per_wave, VariateParams vp, uint32_t stage_cap,
                                                        StageEntry* __restrict__ stage, int32_t* __restrict__ cnt, Ctl* ctl) {
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + uniform_wave_in_block();
  const int64_t first = wave * lists_per_wave;
  if (first >= n_dst) return;
  const int lane = lane_id();
  const int64_t mine = first + lane;
  const bool has = lane < lists_per_wave && mine < n_dst;
  Segment g{0, 0, kAllThr};
  if (has) g = seg[mine];
  const uint32_t beg_lo = (uint32_t)g.beg, beg_hi = (uint32_t)((uint64_t)g.beg >> 32);
  uint32_t my_count = 0;
  const int n_lists = (int)(n_dst - first < lists_per_wave ? n_dst - first : lists_per_wave);
  for (int i = 0; i < n_lists; ++i) {
    const int64_t beg = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)beg_hi, i) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane((int)beg_lo, i));
    const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)g.d, i);
    const uint32_t thr = (uint32_t)__builtin_amdgcn_readlane((int)g.thr, i);
    StageEntry* row = stage + (size_t)(first + i) * stage_cap;
    uint32_t c;
    if (VEC == 4 && thr != kAllThr && d > (uint32_t)kWave) {
      c = labor_scan_staged<BLEND>(g_indices, beg, d, thr, vp, row, stage_cap);
    } else {
      c = labor_scan_ordered<BLEND>(g_indices, beg, d, thr == kAllThr, thr, vp, [&](uint32_t rank, int32_t t, uint32_t j) {
        if (rank < stage_cap) row[rank] = StageEntry{t, j};
      });
    }
    if (lane == i) my_count = c;
  }
  if (has) {
    cnt[mine] = (int32_t)my_count;
    if (my_count > stage_cap) atomicAdd(&ctl->n_overflow, 1);
  }
}

// staged rows -> the block's edge arrays: kFillLanes threads per destination, each taking every kFillLanes-th slot
constexpr int kFillLanesLog2 = 3;
__global__ __launch_bounds__(kBlock) void k_labor_fill_staged(const Segment* __restrict__ seg, int64_t n_dst, uint32_t stage_cap,
                                                              const StageEntry* __restrict__ stage, const int64_t* __restrict__ eptr,
                                                              int32_t* __restrict__ col_global, int64_t* __restrict__ eid) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t w = idx >> kFillLanesLog2;
  if (w >= n_dst) return;
  const int64_t o = eptr[w];
  const int64_t c = eptr[w + 1] - o;
  if (c > (int64_t)stage_cap) return;  // overflowed row: the overflow pass writes these edges
  const StageEntry* __restrict__ row = stage + (size_t)w * stage_cap;
  const int64_t beg = seg[w].beg;
  for (int64_t slot = idx & ((1 << kFillLanesLog2) - 1); slot < c; slot += 1 << kFillLanesLog2) {
    const StageEntry e = row[slot];
    col_global[o + slot] = e.t;
    eid[o + slot] = beg + e.j;
  }
}

// second, ordered scan of the (rare) destinations whose staging row overflowed, writing straight to the edge arrays
template <bool BLEND>
__global__ __launch_bounds__(kBlock) void k_labor_fill_overflow(const int32_t* __restrict__ g_indices, const Segment* __restrict__ seg,
                                                                int64_t n_dst, VariateParams vp, uint32_t stage_cap,
                                                                const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                                int64_t* __restrict__ eid) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + uniform_wave_in_block();
  if (w >= n_dst) return;
  const int64_t o = eptr[w];
  if (eptr[w + 1] - o <= (int64_t)stage_cap) return;
  const Segment g = seg[w];
  labor_scan_ordered<BLEND>(g_indices, g.beg, g.d, g.thr == kAllThr, g.thr, vp, [&](uint32_t rank, int32_t t, uint32_t j) {
    col_global[o + rank] = t;
    eid[o + rank] = g.beg + j;
  });
}

// ---- NS -------------------------------------------------------------------------------------------------------
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
int g_lists_per_wave = 0;      // COOP_TUNE_LISTS_PER_WAVE (0 = automatic)

}  // namespace coop

using namespace coop;

extern "C" int coop_tune(int knob, int64_t value) {
  switch (knob) {
    case COOP_TUNE_STAGE_CAP:
      if (value != 0 && (value < 1 || value > kWave || (value & (value - 1)))) return COOP_E_ARG;
      g_stage_cap_override = (int)value;
      return COOP_OK;
    case COOP_TUNE_LISTS_PER_WAVE:
      if (value < 0 || value > kWave) return COOP_E_ARG;
      g_lists_per_wave = (int)value;
      return COOP_OK;
    default:
      return COOP_E_ARG;
  }
}

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

    // LABOR-0 staging rows: room for 2k + 16 kept edges (a row overflows with probability < 1e-8 at k = 10), 32 or
    // 64 entries (what one wave can hold in a register pair); a row that overflows is redone by the overflow pass
    uint32_t stage_cap = 32;
    StageEntry* stage = nullptr;
    Segment* seg = alloc.get<Segment>(n_dst, COOP_TAG_SCRATCH);
    if (sampler == COOP_LABOR0) {
      if (2 * (uint64_t)k + 16 > 32) stage_cap = 64;
      if (g_stage_cap_override) stage_cap = (uint32_t)g_stage_cap_override;
      stage = alloc.get<StageEntry>(n_dst * (int64_t)stage_cap, COOP_TAG_SCRATCH);
    }
    if (alloc.failed) { rc = COOP_E_NOMEM; break; }

    // list records (and, for NS, the counts min(k, d)); then the LABOR-0 neighbour scan
    if (n_dst > 0) {
      COOP_LAUNCH(K_SEGMENTS, k_segments, dim3(blocks_for(n_dst, kBlock)), dim3(kBlock), 0, s, g->indptr, g->n_vertices, dst, n_dst, k,
                  seg, sampler == COOP_NS ? cnt : nullptr, d_ctl);
      if (sampler == COOP_LABOR0) {
        // lists per wave: one measured as good as several on the papers100M-shaped graph (the knob stays for tuning)
        int lpw = g_lists_per_wave;
        if (lpw == 0) {
          lpw = 1;
        }
        const int64_t n_waves = (n_dst + lpw - 1) / lpw;
        const dim3 grid(blocks_for(n_waves, kWavesPerBlock));
#define COOP_COUNT_ARGS g->indices, seg, n_dst, lpw, vp, stage_cap, stage, cnt, d_ctl
        if (blend) {
          if (vec4) COOP_LAUNCH(K_LABOR_COUNT, (k_labor_count<true, 4>), grid, dim3(kBlock), 0, s, COOP_COUNT_ARGS);
          else COOP_LAUNCH(K_LABOR_COUNT, (k_labor_count<true, 1>), grid, dim3(kBlock), 0, s, COOP_COUNT_ARGS);
        } else {
          if (vec4) COOP_LAUNCH(K_LABOR_COUNT, (k_labor_count<false, 4>), grid, dim3(kBlock), 0, s, COOP_COUNT_ARGS);
          else COOP_LAUNCH(K_LABOR_COUNT, (k_labor_count<false, 1>), grid, dim3(kBlock), 0, s, COOP_COUNT_ARGS);
        }
#undef COOP_COUNT_ARGS
      }
    }
    scan_i32_to_i64(cnt, n_dst, blk.indptr, &d_ctl->total_edges, scan_tmp, s);  // m_l = indptr[n_dst]
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
        COOP_LAUNCH(K_LABOR_FILL, k_labor_fill_staged, dim3(blocks_for(n_dst << kFillLanesLog2, kBlock)), dim3(kBlock), 0, s, seg, n_dst,
                    stage_cap, stage, blk.indptr, blk.col_global, blk.eid);
        if (h_ctl->n_overflow > 0) {
          const dim3 grid(blocks_for(n_dst, kWavesPerBlock));
          if (blend)
            COOP_LAUNCH(K_LABOR_OVERFLOW, k_labor_fill_overflow<true>, grid, dim3(kBlock), 0, s, g->indices, seg, n_dst, vp, stage_cap,
                        blk.indptr, blk.col_global, blk.eid);
          else
            COOP_LAUNCH(K_LABOR_OVERFLOW, k_labor_fill_overflow<false>, grid, dim3(kBlock), 0, s, g->indices, seg, n_dst, vp, stage_cap,
                        blk.indptr, blk.col_global, blk.eid);
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
