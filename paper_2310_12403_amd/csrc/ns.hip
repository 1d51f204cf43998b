// NS layers (App. A.1.1): a destination of degree d <= k keeps all of N(s); otherwise it keeps the k neighbours with
// the smallest (R_ts, list position), a uniform k-subset.  Kept edges leave in (destination order, adjacency order).
// The count is known without looking at the list (min(k, d)), so every list is read once, by the fill pass.
#include "blend_filters.h"
#include "device_utils.h"
#include "sample_internal.h"

namespace coop {

// Filters between a blended NS variate and its exact evaluation, for the candidate test R <= bound (c > 0 only).
struct NsBlendThr {
  uint32_t a2, a1, b2;  // integer bounds on min(U1, U2) and max(U1, U2), as for LABOR-0
  float lim2;           // the blend in fp32 above this cannot be a candidate
};
__device__ __forceinline__ NsBlendThr ns_blend_thresholds(uint32_t bound, double cw, double sw) {
  const PreThr p = blend_first_thresholds(bound, cw, sw);
  return NsBlendThr{p.a2, p.a1, p.b2, blend_second_threshold(bound, cw + sw)};
}

// One destination's neighbour list as the fill pass sees it (written by the count pass, so that the fill pass
// reaches the list with one dependent load instead of three).
struct NsRecord {
  int64_t beg;
  uint32_t d;
  int32_t s;
  uint32_t bound;  // first candidate bound: about `target` of the d variates are expected below it
  uint32_t pad;
};

// (long_min > 0: the destinations whose list is longer than long_min entries, and than k, are also queued in long_list,
// in no particular order, *n_long counting them: the traversal kernels give those to their first waves, see there)
__global__ __launch_bounds__(kBlock) void k_ns_count(const int64_t* __restrict__ g_indptr, int64_t n_vertices,
                                                     const int32_t* __restrict__ dst, int64_t n_dst, uint32_t k, uint32_t target,
                                                     int32_t* __restrict__ cnt, NsRecord* __restrict__ rec,
                                                     NsBlendThr* __restrict__ bthr /* null when c = 0 */, double cw, double sw, Ctl* ctl,
                                                     uint32_t long_min, uint32_t* __restrict__ long_list, uint32_t* __restrict__ n_long) {
  __shared__ uint32_t wave_long[kWavesPerBlock];
  __shared__ uint32_t block_base;
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  bool is_long = false;
  if (i < n_dst) {
    const int32_t s = dst[i];
    if ((uint64_t)(uint32_t)s >= (uint64_t)n_vertices) {
      atomicOr(&ctl->err_range, 1);
      cnt[i] = 0;
      rec[i] = NsRecord{0, 0u, 0, 0u, 0u};
      if (bthr) bthr[i] = NsBlendThr{0u, 0u, 0u, 0.0f};
    } else {
      const int64_t beg = g_indptr[s];
      const int64_t d = g_indptr[s + 1] - beg;
      cnt[i] = (int32_t)(d < (int64_t)k ? d : (int64_t)k);
      // bound such that E[#candidates] = target: R <= bound with probability (bound + 1) / 2^32 (one 64-bit division per
      // list, here where every lane has a list of its own)
      uint64_t bound = d > 0 ? ((uint64_t)target << 32) / (uint64_t)d : 0xFFFFFFFFull;
      if (bound > 0xFFFFFFFFull) bound = 0xFFFFFFFFull;  // d <= target: every neighbour is a candidate
      rec[i] = NsRecord{beg, (uint32_t)d, s, (uint32_t)bound, 0u};
      if (bthr) bthr[i] = d > (int64_t)k ? ns_blend_thresholds((uint32_t)bound, cw, sw) : NsBlendThr{0u, 0u, 0u, 0.0f};
      is_long = long_min != 0 && d > (int64_t)long_min && d > (int64_t)k;
    }
  }
  if (long_min == 0) return;  // (the same for every thread)
  const uint64_t m = ballot64(is_long);
  const int wib = wave_in_block();
  if (lane_id() == 0) wave_long[wib] = (uint32_t)__popcll(m);
  __syncthreads();
  if (threadIdx.x == 0) {  // one reservation per block
    uint32_t total = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) total += wave_long[w];
    block_base = total ? atomicAdd(n_long, total) : 0u;
  }
  __syncthreads();
  if (is_long) {
    uint32_t at = block_base + lanes_below(m);
    for (int w = 0; w < wib; ++w) at += wave_long[w];
    if ((int64_t)at < n_dst) long_list[at] = (uint32_t)i;  // (always: every destination is queued at most once; the queue has n_dst places)
  }
}

constexpr uint32_t kNsMaxSelect = 1024;  // largest fanout for which a longer list is subsampled through the candidate arrays
constexpr int64_t kNsQueueFrom = 32768;  // destinations from which the long lists are queued for the first waves
constexpr int kNsLongDefault = 2048;
int g_ns_long_min = kNsLongDefault;      // COOP_TUNE_NS_LONG_LIST: lists longer than this are queued (0 = none)
constexpr uint32_t kNsRedo = 0xFFFFFFFFu;  // candidate count of a destination that the two-kernel path leaves to k_ns_fill

typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr int kNsGroups = 4;  // 16-byte groups per lane and step of the fast traversal

// Stage-1 passers of the blended path wait here (per wave, in LDS) until 64 of them can be evaluated together.
constexpr int kNsQueueCap = 2 * kWave;
struct NsQueue {
  int32_t t[kNsQueueCap];
  uint32_t j[kNsQueueCap];
  uint32_t u1[kNsQueueCap];
  uint32_t u2[kNsQueueCap];
};

// One pass over the list [beg, beg + d): every neighbour whose variate is <= bound is appended to the candidate
// arrays in LDS (key = variate in the upper, list position in the lower half of 64 bits: the order of the selection;
// vertex), in no particular order; returns how many qualified (entries beyond
// `cap` are counted but not stored).  Long lists in a 16-byte aligned array are read as aligned groups of four
// entries, kNsGroups groups per lane and step, whole groups in the main loop and the ragged ends in one extra step.
// With c > 0 the variate of an entry is evaluated exactly only if the integer bounds and then the fp32 blend cannot
// rule it out; the survivors of the integer bounds are evaluated 64 at a time.
// STAGED (with c > 0): the exact evaluation is left to a later kernel; everything that the fp32 blend cannot rule out
// is stored as a candidate (variate 0).
template <bool BLEND, bool VEC4, bool STAGED = false>
__device__ __forceinline__ uint32_t ns_collect(const int32_t* __restrict__ g_indices, int64_t beg, uint32_t d, uint32_t bound,
                                               const NsBlendThr& bt, const VariateParams& vp, uint32_t sigma_a, uint32_t sigma_b,
                                               uint64_t* __restrict__ cand_key, int32_t* __restrict__ cand_t, uint32_t cap,
                                               NsQueue* __restrict__ q) {
  const uint32_t lane = (uint32_t)lane_id();
  uint32_t n_c = 0;
  auto append = [&](bool in, uint32_t r, uint32_t j, int32_t t) {
    const uint64_t mask = ballot64(in);
    if (mask == 0) return;
    const uint32_t p = n_c + lanes_below(mask);
    if (in && p < cap) {
      uint32_t* half = reinterpret_cast<uint32_t*>(cand_key + p);  // two 32-bit stores: no register pair needed in the hot loop
      half[0] = j;
      half[1] = r;
      cand_t[p] = t;
    }
    n_c += (uint32_t)__popcll(mask);
  };
  // ---- blended path: queue, and evaluation of its first n entries --------------------------------------------------
  uint32_t qn = 0;
  const float cwf = (float)vp.cw, swf = (float)vp.sw;
  auto evaluate = [&](uint32_t n) {
    int32_t t = 0;
    uint32_t j = 0, R = 0;
    bool in = false;
    if (lane < n) {
      t = q->t[lane];
      j = q->j[lane];
      const uint32_t u1 = q->u1[lane], u2 = q->u2[lane];
      if (__builtin_fmaf(cwf, approx_phi_inv_f32(u1), swf * approx_phi_inv_f32(u2)) <= bt.lim2) {
        if constexpr (STAGED) {
          in = true;
        } else {
          R = kit_phi_to_u32(__builtin_fma(vp.cw, kit_phi_inv_u32(u1), vp.sw * kit_phi_inv_u32(u2)));
          in = R <= bound;
        }
      }
    }
    append(in, R, j, t);
  };
  auto enqueue = [&](bool pre, int32_t t, uint32_t j, uint32_t u1, uint32_t u2) {
    const uint64_t mask = ballot64(pre);
    if (mask == 0) return;
    if (pre) {
      const uint32_t at = qn + lanes_below(mask);  // below 128
      q->t[at] = t; q->j[at] = j; q->u1[at] = u1; q->u2[at] = u2;
    }
    qn += (uint32_t)__popcll(mask);
    __builtin_amdgcn_wave_barrier();
    if (qn >= (uint32_t)kWave) {
      evaluate(kWave);
      const uint32_t rest = qn - kWave;  // fewer than 64: to the front
      int32_t mt = 0;
      uint32_t mj = 0, m1 = 0, m2 = 0;
      if (lane < rest) { mt = q->t[kWave + lane]; mj = q->j[kWave + lane]; m1 = q->u1[kWave + lane]; m2 = q->u2[kWave + lane]; }
      __builtin_amdgcn_wave_barrier();
      if (lane < rest) { q->t[lane] = mt; q->j[lane] = mj; q->u1[lane] = m1; q->u2[lane] = m2; }
      qn = rest;
      __builtin_amdgcn_wave_barrier();
    }
  };
  // first look at one entry: its variate (c = 0) or the integer bounds on its two uniforms (c > 0)
  auto first_look = [&](bool valid, int32_t t, uint32_t& r, uint32_t& u2) -> bool {
    r = keyed_uniform<true>(vp.K.Ka, (uint32_t)t, sigma_a);
    if constexpr (!BLEND) {
      return valid & (r <= bound);
    } else {
      u2 = keyed_uniform<true>(vp.K.Kb, (uint32_t)t, sigma_b);
      const uint32_t lo = r < u2 ? r : u2, hi = r < u2 ? u2 : r;
      return valid & ((lo <= bt.a1) | ((lo <= bt.a2) & (hi <= bt.b2)));
    }
  };
  auto take = [&](bool flag, int32_t t, uint32_t j, uint32_t r, uint32_t u2) {
    if constexpr (!BLEND) append(flag, r, j, t);
    else enqueue(flag, t, j, r, u2);
  };

  if (!VEC4 || d <= (uint32_t)kWave) {
    for (uint32_t base = 0; base < d; base += kWave) {
      const uint32_t j = base + lane;
      int32_t t = 0;
      if (j < d) t = g_indices[beg + j];
      uint32_t r = 0, u2 = 0;
      const bool flag = first_look(j < d, t, r, u2);
      take(flag, t, j, r, u2);
    }
  } else {
    constexpr uint32_t kStep = kWave * 4 * kNsGroups;
    const int64_t abeg = beg & ~(int64_t)3;        // first aligned group
    const uint32_t head = (uint32_t)(beg - abeg);  // entries of that group that precede the list
    const uint32_t total = head + d;               // list end, relative to abeg
    const uint32_t vec_end = total & ~3u;          // whole groups end here
    const uint32_t vec_beg = head ? 4u : 0u;       // whole groups start here
    const int32_t* __restrict__ p = g_indices + abeg;
    // the loads of the next step are issued before this step's entries are hashed
    i32x4 nbuf[kNsGroups];
    auto fetch = [&](uint32_t at) {
#pragma unroll
      for (int gq = 0; gq < kNsGroups; ++gq) {
        const uint32_t r = at + (uint32_t)(gq * kWave * 4) + lane * 4;
        nbuf[gq] = i32x4{0, 0, 0, 0};
        if (r < vec_end) nbuf[gq] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(p + r));
      }
    };
    // (not with c > 0: the blended path needs the registers more than the overlap)
    if (!BLEND && vec_beg < vec_end) fetch(vec_beg);
    // the ragged ends (lanes 0..2: the entries in front of the first whole group; lanes 3..5: those behind the last one) are
    // requested now, not when the whole groups are done, so that a short list waits for memory once
    const uint32_t end_pos = lane < 3 ? head + lane : vec_end + (lane - 3);
    const bool end_valid = lane < 3 ? (head != 0 && end_pos < 4) : (lane < 6 && end_pos < total);
    int32_t end_t = 0;
    if (end_valid) end_t = p[end_pos];
    for (uint32_t base = vec_beg; base < vec_end; base += kStep) {
      if (BLEND) fetch(base);
      i32x4 buf[kNsGroups];
      bool ok[kNsGroups];
#pragma unroll
      for (int gq = 0; gq < kNsGroups; ++gq) {
        buf[gq] = nbuf[gq];
        ok[gq] = base + (uint32_t)(gq * kWave * 4) + lane * 4 < vec_end;
      }
      if (!BLEND && base + kStep < vec_end) fetch(base + kStep);
      auto group = [&](int gq, bool valid) {
        const uint32_t r = base + (uint32_t)(gq * kWave * 4) + lane * 4;
        uint32_t R[4], U2[4];
        bool flag[4];
        bool any = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          flag[e] = first_look(valid, buf[gq][e], R[e], U2[e]);
          any |= flag[e];
        }
        if (ballot64(any) != 0) {
#pragma unroll
          for (int e = 0; e < 4; ++e) take(flag[e], buf[gq][e], r + e - head, R[e], U2[e]);
        }
      };
#pragma unroll
      for (int gq = 0; gq < kNsGroups; ++gq) {
        if (base + (uint32_t)(gq * kWave * 4) >= vec_end) break;  // wave-uniform: the rest of this step lies behind the list
        group(gq, ok[gq]);
      }
    }
    {  // the ragged ends
      uint32_t r = 0, u2 = 0;
      const bool flag = first_look(end_valid, end_t, r, u2);
      take(flag, end_t, end_pos - head, r, u2);
    }
  }
  if constexpr (BLEND) {
    if (qn != 0) evaluate(qn);
    __builtin_amdgcn_wave_barrier();
  }
  return n_c;
}

// The k smallest by (variate, list position) among the n_c candidates in LDS (k <= n_c <= cap), written to the edge arrays
// from o on in adjacency order: every candidate's rank among the candidates is counted, ranks below k are kept, and a
// kept candidate's place is the number of kept candidates in front of it in the list.
__device__ __forceinline__ void ns_rank_write(uint32_t n_c, uint32_t k, const uint64_t* cand_key, uint32_t* cand_k, const int32_t* cand_t,
                                              int64_t o, int64_t beg, int32_t* __restrict__ col_global, int64_t* __restrict__ eid) {
  const uint32_t lane = (uint32_t)lane_id();
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  if (n_c <= (uint32_t)kWave) {
    // the usual case: one candidate per lane; every lane reads the keys one after the other from LDS (the same address
    // for all lanes: a broadcast), two vector instructions per candidate where reading variate and position out of the
    // other lanes' registers cost seven
    const bool has = lane < n_c;
    const uint64_t my_key = has ? cand_key[lane] : ~0ull;
    const uint32_t my_j = (uint32_t)my_key;
    const int32_t my_t = has ? cand_t[lane] : 0;
    uint32_t rank = 0;
    const uint32_t n_u = (uint32_t)__builtin_amdgcn_readfirstlane((int)n_c);
    for (uint32_t q = 0; q < n_u; ++q) rank += cand_key[q] < my_key;
    const bool keep = has && rank < k;
    const uint64_t kept = ballot64(keep);
    uint32_t place = 0;  // kept candidates in front of this one in the list
    uint64_t rest = kept;
    while (rest != 0) {
      const int q = __builtin_ctzll(rest);
      rest &= rest - 1;
      place += (uint32_t)__builtin_amdgcn_readlane((int)my_j, q) < my_j;
    }
    if (keep) {
      col_global[o + place] = my_t;
      eid[o + place] = beg + my_j;
    }
    return;
  }
  for (uint32_t i = lane; i < n_c; i += kWave) {
    const uint64_t my_key = cand_key[i];
    uint32_t rank = 0;
    for (uint32_t q = 0; q < n_c; ++q) rank += cand_key[q] < my_key;
    cand_k[i] = rank < k;
  }
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  for (uint32_t i = lane; i < n_c; i += kWave) {
    if (!cand_k[i]) continue;
    const uint32_t my_j = (uint32_t)cand_key[i];
    uint32_t place = 0;
    for (uint32_t q = 0; q < n_c; ++q) place += cand_k[q] && (uint32_t)cand_key[q] < my_j;
    col_global[o + place] = cand_t[i];
    eid[o + place] = beg + my_j;
  }
}

// Selection of the k smallest (R, j) among d > k neighbours, one wave per destination:
//   1. one pass over the list collects, in LDS, the candidates with R <= bound, where bound is chosen so that about
//      `target` of them are expected (target > k, target < cap);
//   2. if fewer than k or more than cap candidates turn up, the bound is bisected and the pass repeated (rare);
//   3. every candidate's rank by (R, j) among the candidates is counted: ranks below k are kept;
//   4. every kept candidate's place is the number of kept candidates in front of it in the list.
//
// The degree distribution is heavy-tailed and a wave takes a whole list, so the lists longer than long_min entries
// are not left where the destination order puts them (a hub that starts late would keep the kernel waiting for one
// wave): k_ns_count queues them, the first long_blocks blocks of the grid stride over the queue (its length is read from
// device memory; every wave ends after a bounded number of steps), and the other blocks take the destinations in order
// and skip the queued ones.
template <bool BLEND, bool VEC4>
__device__ __forceinline__ void ns_fill_one(int64_t w, int wib, uint32_t* lds_words, NsQueue* queue, const int32_t* __restrict__ g_indices,
                                            const NsRecord* __restrict__ rec, const NsBlendThr* __restrict__ bthr, uint32_t k, uint32_t cap,
                                            const VariateParams& vp, const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                            int64_t* __restrict__ eid, int64_t edge_limit, Ctl* ctl, uint32_t skip_above) {
  const uint32_t lane = (uint32_t)lane_id();
  const int64_t o = eptr[w];
  if (eptr[w + 1] > edge_limit) return;  // the wave writes [o, eptr[w + 1]) only; no room: the caller redoes the layer
  const NsRecord g = rec[w];
  const int32_t s = g.s;
  const int64_t beg = g.beg;
  const uint32_t d = g.d;
  if (d == 0) return;
  if (d <= k) {
    for (uint32_t j = lane; j < d; j += kWave) {
      col_global[o + j] = g_indices[beg + j];
      eid[o + j] = beg + j;
    }
    return;
  }
  if (d > skip_above) return;    // queued: one of the first waves takes it
  if (k > kNsMaxSelect) return;  // a degree above a fanout that the candidate buffer cannot serve: left to k_ns_fill_wide
  uint64_t* cand_key = reinterpret_cast<uint64_t*>(lds_words + (size_t)wib * cap * 4);  // [cap] (variate, position), d < 2^31
  uint32_t* cand_k = lds_words + (size_t)wib * cap * 4 + 2 * cap;                       // [cap] 1 = among the k smallest
  int32_t* cand_t = reinterpret_cast<int32_t*>(cand_k + cap);                           // [cap] the neighbours themselves
  const uint32_t sigma_a = ns_sigma(vp.K.Ka, (uint32_t)s);
  const uint32_t sigma_b = BLEND ? ns_sigma(vp.K.Kb, (uint32_t)s) : 0u;

  uint64_t lo = 0, hi = 0xFFFFFFFFull;  // bisection bracket on the bound, used only after a failed pass
  uint64_t bound = g.bound;
  NsBlendThr bt{0u, 0u, 0u, 0.0f};
  if constexpr (BLEND) bt = bthr[w];
  uint32_t n_c = 0;
  for (int attempt = 0; attempt < 40; ++attempt) {
    n_c = ns_collect<BLEND, VEC4>(g_indices, beg, d, (uint32_t)bound, bt, vp, sigma_a, sigma_b, cand_key, cand_t, cap, queue);
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
    // too few and no upper failure yet: double the bound (a midpoint of the whole range would flood the buffer)
    bound = (hi == 0xFFFFFFFFull && n_c < k) ? (2 * bound + 1 < hi ? 2 * bound + 1 : hi) : lo + (hi - lo) / 2;
    if constexpr (BLEND) bt = ns_blend_thresholds((uint32_t)bound, vp.cw, vp.sw);  // (every lane computes the same)
    __builtin_amdgcn_wave_barrier();
  }
  if (n_c < k || n_c > cap) {
    if (lane == 0) atomicOr(&ctl->err_capacity, 1);
    return;
  }
  ns_rank_write(n_c, k, cand_key, cand_k, cand_t, o, beg, col_global, eid);
}

template <bool BLEND, bool VEC4>
__global__ __launch_bounds__(kBlock) void k_ns_fill(const int32_t* __restrict__ g_indices,
                                                    const NsRecord* __restrict__ rec, const NsBlendThr* __restrict__ bthr,
                                                    int64_t n_dst, uint32_t k,
                                                    uint32_t cap, int waves_per_block, VariateParams vp,
                                                    const int64_t* __restrict__ eptr, int32_t* __restrict__ col_global,
                                                    int64_t* __restrict__ eid, int64_t edge_limit, Ctl* ctl,
                                                    const uint32_t* __restrict__ only /* when not null: only lists marked kNsRedo */,
                                                    uint32_t long_min, const uint32_t* __restrict__ long_list,
                                                    const uint32_t* __restrict__ n_long, int long_blocks) {
  extern __shared__ __align__(16) uint32_t lds_words[];  // per wave: cap 64-bit keys, cap keep flags, cap vertex ids
  NsQueue* queues = reinterpret_cast<NsQueue*>(lds_words + (size_t)waves_per_block * cap * 4);  // (with c > 0; behind the candidates)
  const int wib = uniform_wave_in_block();
  if (wib >= waves_per_block) return;
  NsQueue* queue = &queues[BLEND ? wib : 0];
  const bool queue_wave = (int)blockIdx.x < long_blocks;
  int64_t w;
  if (queue_wave) {  // the q-th queued long list
    const int64_t q = (int64_t)blockIdx.x * waves_per_block + wib;
    int64_t n_queued = (int64_t)*n_long;
    if (n_queued > n_dst) n_queued = n_dst;  // (holds by construction; keeps every access inside the queue regardless)
    if (q >= n_queued) return;
    // (the same in every lane; said so, or everything derived from it would be kept per lane)
    w = (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)long_list[q]);
  } else {
    w = (int64_t)((int)blockIdx.x - long_blocks) * waves_per_block + wib;
    if (only != nullptr && w < n_dst && only[w] != kNsRedo) return;
  }
  if (w >= n_dst) return;
  ns_fill_one<BLEND, VEC4>(w, wib, lds_words, queue, g_indices, rec, bthr, k, cap, vp, eptr, col_global, eid, edge_limit, ctl,
                           !queue_wave && long_min != 0 ? long_min : 0xFFFFFFFFu);
}

// ---- c > 0 in two kernels ----------------------------------------------------------------------------------------
// The exact blend (two inverse normal distribution functions and one forward, in fp64) needs four times the registers of
// the traversal and is wanted for a few dozen candidates per list only.  So the traversal kernel stops at the fp32
// filter and leaves what passes, (list position, vertex) pairs, in a row of row_cap entries per destination; a second
// kernel evaluates those exactly, drops the ones above the bound and selects.  A destination whose row overflows, or
// that ends up with fewer than k candidates (about one in 10^4), is marked and done again by k_ns_fill, which adjusts
// the bound.
struct NsCand { uint32_t j; int32_t t; };

template <bool VEC4>
__global__ __launch_bounds__(kBlock) void k_ns_collect(const int32_t* __restrict__ g_indices, const NsRecord* __restrict__ rec,
                                                       const NsBlendThr* __restrict__ bthr, int64_t n_dst, uint32_t k, uint32_t cap,
                                                       int waves_per_block, VariateParams vp, const int64_t* __restrict__ eptr,
                                                       int32_t* __restrict__ col_global, int64_t* __restrict__ eid, int64_t edge_limit,
                                                       Ctl* ctl, NsCand* __restrict__ rows, uint32_t row_cap, uint32_t* __restrict__ n_cand,
                                                       uint32_t long_min, const uint32_t* __restrict__ long_list,
                                                       const uint32_t* __restrict__ n_long, int long_blocks) {
  extern __shared__ __align__(16) uint32_t lds_words[];
  NsQueue* queues = reinterpret_cast<NsQueue*>(lds_words + (size_t)waves_per_block * cap * 4);  // (behind the candidates)
  const int wib = uniform_wave_in_block();
  if (wib >= waves_per_block) return;
  const bool queue_wave = (int)blockIdx.x < long_blocks;  // the queued long lists first, as in k_ns_fill
  int64_t w;
  if (queue_wave) {
    const int64_t q = (int64_t)blockIdx.x * waves_per_block + wib;
    int64_t n_queued = (int64_t)*n_long;
    if (n_queued > n_dst) n_queued = n_dst;
    if (q >= n_queued) return;
    w = (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)long_list[q]);
  } else {
    w = (int64_t)((int)blockIdx.x - long_blocks) * waves_per_block + wib;
  }
  if (w >= n_dst) return;
  const uint32_t lane = (uint32_t)lane_id();
  const NsRecord g = rec[w];
  if (!queue_wave && long_min != 0 && g.d > long_min && g.d > k) return;  // queued: one of the first waves takes it
  if (lane == 0) n_cand[w] = 0;  // nothing left to do for this destination, unless said otherwise below
  const int64_t o = eptr[w];
  if (eptr[w + 1] > edge_limit) return;
  if (g.d == 0) return;
  if (g.d <= k) {
    for (uint32_t j = lane; j < g.d; j += kWave) {
      col_global[o + j] = g_indices[g.beg + j];
      eid[o + j] = g.beg + j;
    }
    return;
  }
  if (k > kNsMaxSelect) return;  // (k_ns_fill_wide)
  uint64_t* cand_key = reinterpret_cast<uint64_t*>(lds_words + (size_t)wib * cap * 4);
  int32_t* cand_t = reinterpret_cast<int32_t*>(lds_words + (size_t)wib * cap * 4 + 3 * cap);
  const uint32_t sigma_a = ns_sigma(vp.K.Ka, (uint32_t)g.s), sigma_b = ns_sigma(vp.K.Kb, (uint32_t)g.s);
  const uint32_t n_c = ns_collect<true, VEC4, true>(g_indices, g.beg, g.d, g.bound, bthr[w], vp, sigma_a, sigma_b, cand_key, cand_t, cap,
                                                    &queues[wib]);
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  if (n_c < k || n_c > row_cap || n_c > cap) {  // (too few even before the exact test, or no room)
    if (lane == 0) n_cand[w] = kNsRedo;
    return;
  }
  NsCand* row = rows + (size_t)w * row_cap;
  for (uint32_t i = lane; i < n_c; i += kWave) row[i] = NsCand{(uint32_t)cand_key[i], cand_t[i]};
  if (lane == 0) n_cand[w] = n_c;
}

__global__ __launch_bounds__(kBlock) void k_ns_select(const NsRecord* __restrict__ rec, int64_t n_dst, uint32_t k, uint32_t cap,
                                                      int waves_per_block, VariateParams vp, const int64_t* __restrict__ eptr,
                                                      int32_t* __restrict__ col_global, int64_t* __restrict__ eid,
                                                      const NsCand* __restrict__ rows, uint32_t row_cap, uint32_t* __restrict__ n_cand,
                                                      const NsBlendThr* __restrict__ bthr) {
  extern __shared__ __align__(16) uint32_t lds_words[];
  const int wib = uniform_wave_in_block();
  if (wib >= waves_per_block) return;
  const int64_t w = (int64_t)blockIdx.x * waves_per_block + wib;
  if (w >= n_dst) return;
  const uint32_t n = n_cand[w];
  if (n == 0 || n == kNsRedo) return;  // done by the collecting kernel, or left to k_ns_fill
  const uint32_t lane = (uint32_t)lane_id();
  const NsRecord g = rec[w];
  uint64_t* cand_key = reinterpret_cast<uint64_t*>(lds_words + (size_t)wib * cap * 4);
  uint32_t* cand_k = lds_words + (size_t)wib * cap * 4 + 2 * cap;
  int32_t* cand_t = reinterpret_cast<int32_t*>(cand_k + cap);
  const uint32_t sigma_a = ns_sigma(vp.K.Ka, (uint32_t)g.s), sigma_b = ns_sigma(vp.K.Kb, (uint32_t)g.s);
  const NsCand* row = rows + (size_t)w * row_cap;
  if (n <= (uint32_t)kWave) {
    // The usual case, one candidate per lane.  Only the set of the k smallest matters, so the fp32 blend (within
    // `allow` / 10 of the exact one in normal space) decides wherever it can: with e_k the k-th smallest estimate and
    // m = 2 allow, a candidate below e_k - m is among the k smallest, one above e_k + m is not, and the exact variates
    // are needed only to choose among those in between, and only if there are more of them than places left.
    const bool has = lane < n;
    NsCand c{0xFFFFFFFFu, 0};
    if (has) c = row[lane];
    const uint32_t u1 = keyed_uniform<true>(vp.K.Ka, (uint32_t)c.t, sigma_a), u2 = keyed_uniform<true>(vp.K.Kb, (uint32_t)c.t, sigma_b);
    const float est = has ? __builtin_fmaf((float)vp.cw, approx_phi_inv_f32(u1), (float)vp.sw * approx_phi_inv_f32(u2)) : __builtin_inff();
    // rank by (estimate, lane): the estimates (finite for every candidate) go to LDS as 64-bit keys, their bits mapped so
    // that unsigned order is numeric order, and every lane reads them back as broadcasts (as in ns_rank_write)
    const uint32_t eb = __float_as_uint(est);
    const uint64_t est_key = ((uint64_t)(eb ^ ((uint32_t)((int32_t)eb >> 31) | 0x80000000u)) << 32) | lane;
    if (has) cand_key[lane] = est_key;
    __builtin_amdgcn_wave_barrier();
    __threadfence_block();
    uint32_t rank_est = 0;
    const uint32_t n_u = (uint32_t)__builtin_amdgcn_readfirstlane((int)n);
    for (uint32_t q = 0; q < n_u; ++q) rank_est += cand_key[q] < est_key;
    const uint64_t kth = ballot64(has && rank_est == k - 1);  // exactly one lane (n >= k)
    const float e_k = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(est), __builtin_ctzll(kth)));
    const float allow = (float)((vp.cw + vp.sw) * kPhiInvF32Allow + 2.0 * kBlendAbsWiden);
    const float m = 2.0f * allow;
    // outside |e_k| <= 5 two different blends can share a 32-bit variate, and the estimate says nothing about ties; and
    // e_k must lie safely below what the traversal's filter let through, or a neighbour that it dropped could belong
    // to the k smallest
    if (!(e_k >= -5.0f && e_k <= 5.0f) || !(e_k + m <= bthr[w].lim2 - m)) {
      if (lane == 0) n_cand[w] = kNsRedo;
      return;
    }
    const bool in = has && est < e_k - m;
    const bool und = has && !in && est <= e_k + m;
    const uint64_t und_mask = ballot64(und);
    const uint32_t need = k - (uint32_t)__popcll(ballot64(in));  // >= 1: the k-th itself is undecided
    bool keep = in || und;
    if ((uint32_t)__popcll(und_mask) > need) {  // wave-uniform
      uint32_t R = 0;
      if (und) R = kit_phi_to_u32(__builtin_fma(vp.cw, kit_phi_inv_u32(u1), vp.sw * kit_phi_inv_u32(u2)));
      const uint64_t my_key = ((uint64_t)R << 32) | c.j;
      uint32_t rank_u = 0;
      uint64_t rest = und_mask;
      while (rest != 0) {
        const int q = __builtin_ctzll(rest);
        rest &= rest - 1;
        const uint64_t key = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)R, q) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)c.j, q);
        rank_u += key < my_key;
      }
      keep = in || (und && rank_u < need);
    }
    const uint64_t kept = ballot64(keep);
    uint32_t place = 0;  // kept candidates in front of this one in the list
    uint64_t rest = kept;
    while (rest != 0) {
      const int q = __builtin_ctzll(rest);
      rest &= rest - 1;
      place += (uint32_t)__builtin_amdgcn_readlane((int)c.j, q) < c.j;
    }
    if (keep) {
      const int64_t o = eptr[w];
      col_global[o + place] = c.t;
      eid[o + place] = g.beg + c.j;
    }
    return;
  }
  uint32_t n_c = 0;  // candidates with R <= bound, compacted into LDS
  for (uint32_t base = 0; base < n; base += kWave) {
    const uint32_t i = base + lane;
    NsCand c{0u, 0};
    uint32_t R = 0;
    bool in = false;
    if (i < n) {
      c = row[i];
      const uint32_t u1 = keyed_uniform<true>(vp.K.Ka, (uint32_t)c.t, sigma_a), u2 = keyed_uniform<true>(vp.K.Kb, (uint32_t)c.t, sigma_b);
      R = kit_phi_to_u32(__builtin_fma(vp.cw, kit_phi_inv_u32(u1), vp.sw * kit_phi_inv_u32(u2)));
      in = R <= g.bound;
    }
    const uint64_t mask = ballot64(in);
    const uint32_t at = n_c + lanes_below(mask);
    if (in) { cand_key[at] = ((uint64_t)R << 32) | c.j; cand_t[at] = c.t; }  // (n <= cap)
    n_c += (uint32_t)__popcll(mask);
  }
  if (n_c < k) {
    if (lane == 0) n_cand[w] = kNsRedo;
    return;
  }
  ns_rank_write(n_c, k, cand_key, cand_k, cand_t, eptr[w], g.beg, col_global, eid);
}

// ---- fanouts above kNsMaxSelect ----------------------------------------------------------------------------------
// The k smallest (R, j) of a list longer than k, for a k that the candidate arrays in LDS cannot hold: no candidates are
// stored at all.  A bisection over the 32-bit variates finds the smallest B with #{R <= B} >= k (one pass over the list
// per step, 32 steps); everything below B is kept, and of the entries with R = B (normally one) the first
// k - #{R < B} in list order.  The last pass writes the kept entries in adjacency order, 64 at a time, each at the
// running count plus its rank in the ballot.  One wave per destination; 34 passes over a list, variates recomputed in
// each: a path for the rare call with a fanout in the thousands, not for speed.
template <bool BLEND>
__global__ __launch_bounds__(kBlock) void k_ns_fill_wide(const int32_t* __restrict__ g_indices, const NsRecord* __restrict__ rec,
                                                         int64_t n_dst, uint32_t k, VariateParams vp, const int64_t* __restrict__ eptr,
                                                         int32_t* __restrict__ col_global, int64_t* __restrict__ eid, int64_t edge_limit) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + uniform_wave_in_block();
  if (w >= n_dst) return;
  const NsRecord g = rec[w];
  if (g.d <= k) return;  // (copied whole by the fill kernel)
  if (eptr[w + 1] > edge_limit) return;
  const uint32_t lane = (uint32_t)lane_id();
  const int32_t* __restrict__ list = g_indices + g.beg;
  const uint32_t d = g.d;
  const uint32_t sigma_a = ns_sigma(vp.K.Ka, (uint32_t)g.s);
  const uint32_t sigma_b = BLEND ? ns_sigma(vp.K.Kb, (uint32_t)g.s) : 0u;
  auto count_le = [&](uint32_t B) -> uint32_t {
    uint32_t n = 0;
    for (uint32_t base = 0; base < d; base += kWave) {
      const uint32_t j = base + lane;
      bool in = false;
      if (j < d) in = variate<true, BLEND>(vp, (uint32_t)list[j], sigma_a, sigma_b) <= B;
      n += (uint32_t)__popcll(ballot64(in));
    }
    return n;
  };
  uint64_t lo = 0, hi = 0xFFFFFFFFull;  // #{R <= hi} >= k throughout (d > k)
  while (lo < hi) {
    const uint64_t mid = lo + (hi - lo) / 2;
    if (count_le((uint32_t)mid) >= k) hi = mid;
    else lo = mid + 1;
  }
  const uint32_t B = (uint32_t)lo;
  const uint32_t below = B == 0 ? 0u : count_le(B - 1);
  const uint32_t need = k - below;  // of the entries with R = B, the first `need` in list order (>= 1)
  const int64_t o = eptr[w];
  uint32_t placed = 0, ties = 0;
  for (uint32_t base = 0; base < d; base += kWave) {
    const uint32_t j = base + lane;
    int32_t t = 0;
    uint32_t R = 0xFFFFFFFFu;
    if (j < d) {
      t = list[j];
      R = variate<true, BLEND>(vp, (uint32_t)t, sigma_a, sigma_b);
    }
    const bool eq = j < d && R == B;
    const uint64_t eq_mask = ballot64(eq);
    const bool keep = j < d && (R < B || (eq && ties + lanes_below(eq_mask) < need));
    const uint64_t keep_mask = ballot64(keep);
    if (keep) {
      const uint32_t at = placed + lanes_below(keep_mask);  // below k: exactly k entries are kept
      col_global[o + at] = t;
      eid[o + at] = g.beg + j;
    }
    placed += (uint32_t)__popcll(keep_mask);
    ties += (uint32_t)__popcll(eq_mask);
  }
}

int ns_layer(const SampleCtx& cx, int l, const int32_t* dst, int64_t n_dst, coop_block* blk, int64_t edge_cap) {
  const bool defer = edge_cap > 0;
  hipStream_t s = cx.s;
  Alloc& alloc = *cx.alloc;
  const uint32_t k = (uint32_t)cx.fanouts[l];
  VariateParams vp{};
  layer_keys(cx.seed, COOP_NS, l, cx.group, vp.K.Ka);
  layer_keys(cx.seed, COOP_NS, l, cx.group + 1, vp.K.Kb);
  vp.cw = cx.cw;
  vp.sw = cx.sw;
  blk->indptr = alloc.get<int64_t>(n_dst + 1, COOP_TAG_OUTPUT);
  int32_t* cnt = alloc.get<int32_t>(n_dst, COOP_TAG_SCRATCH);
  NsRecord* rec = alloc.get<NsRecord>(n_dst, COOP_TAG_SCRATCH);
  NsBlendThr* bthr = cx.blend ? alloc.get<NsBlendThr>(n_dst, COOP_TAG_SCRATCH) : nullptr;
  void* scan_tmp = alloc.get<char>((int64_t)scan_tmp_bytes(n_dst), COOP_TAG_SCRATCH);
  if (alloc.failed) return COOP_E_NOMEM;
  // candidate buffer: cap >= 4k (power of two, at least 256).  With a fanout above kNsMaxSelect the lists longer than
  // the fanout are left to k_ns_fill_wide, which keeps no candidates.
  const uint32_t k_sel = k < kNsMaxSelect ? k : kNsMaxSelect;
  uint32_t cap = 256;
  while (cap < 4 * k_sel) cap <<= 1;
  // expected candidates (at most 2k + 16): k + 2 sqrt(k) + 2 with independent variates, where a list that turns up fewer
  // than k candidates (two in a hundred at k = 10) is simply collected again with twice the bound, and every candidate
  // costs an append and ranking work (measured: 5 % off the fill pass against k + 4 sqrt(k) + 4); k + 4 sqrt(k) + 4 with
  // dependent variates, where a list that falls short (one in 10^4) goes through the one-kernel path again.
  uint32_t root = 1;
  while (root * root < k_sel) ++root;
  uint32_t target = cx.blend ? k_sel + 4 * root + 4 : k_sel + 2 * root + 2;
  if (target > 2 * k_sel + 16) target = 2 * k_sel + 16;
  // long lists first (see k_ns_fill): worth its queue from a few tens of thousands of destinations on
  // (default: passes over many destinations of a graph with hubs; where the registration has added the entries of the
  // lists above kLongListDegree up, a graph on which they hold less than an eighth of the edges is left alone: the queue
  // costs the count pass a reservation per block and buys nothing there)
  const bool hubs = !cx.g->symmetric || cx.g->long_mass >= cx.g->n_edges / 8;
  const bool queue_long = g_ns_long_min != 0 && (g_ns_long_min != kNsLongDefault || (n_dst >= kNsQueueFrom && hubs));
  const uint32_t long_min = queue_long ? (uint32_t)g_ns_long_min : 0u;
  uint32_t* long_list = queue_long ? alloc.get<uint32_t>(n_dst, COOP_TAG_SCRATCH) : nullptr;
  uint32_t* n_long = cx.d_piece_count + l;  // (zero at the start of the call and whenever the layer is redone)
  if (alloc.failed) return COOP_E_NOMEM;
  if (n_dst > 0)
    COOP_LAUNCH(K_NS_COUNT, k_ns_count, dim3(blocks_for(n_dst, kBlock)), dim3(kBlock), 0, s, cx.g->indptr, cx.g->n_vertices, dst, n_dst,
                k, target, cnt, rec, bthr, cx.cw, cx.sw, cx.d_ctl, long_min, long_list, n_long);
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
  if (m > 0 && n_dst > 0) {
    // one wave per block: a block leaves the CU when its slowest wave is done, and a wave takes one list, short or long;
    // with four waves a block's slots stood empty for much of its life (fill 1.61 -> 1.52 ms on the papers100M-shaped
    // layer; with dependent variates the traversal 3.0 -> 2.57 ms and the selection 0.99 -> 0.91)
    const int wpb = 1;
    const size_t shmem = (size_t)wpb * cap * 16 + (cx.blend ? (size_t)wpb * sizeof(NsQueue) : 0);
    const dim3 grid(blocks_for(n_dst, wpb));
#define COOP_NS_ARGS cx.g->indices, rec, bthr, n_dst, k, cap, wpb, vp, blk->indptr, blk->col_global, blk->eid, m, cx.d_ctl
    // the queue's waves, one per queued list: as many as there can be lists that long, by the degree census of the
    // registration and by the number of edges (the unused ones end at once)
    int64_t most_long = cx.g->n_edges / (int64_t)(long_min ? long_min : 1) + 1;
    if (most_long > n_dst) most_long = n_dst;
    if (long_min != 0 && most_long > cx.g->lists_longer_than(long_min)) most_long = cx.g->lists_longer_than(long_min);
    const int long_blocks = queue_long ? (int)blocks_for(most_long, wpb) : 0;
    const dim3 grid_q(grid.x + (unsigned)long_blocks);
    if (cx.blend) {
      // rows of the two-kernel path: room for twice the expected candidates (at least 64, at most the LDS capacity)
      uint32_t row_cap = 64;
      while (row_cap < 2 * target && row_cap < cap) row_cap <<= 1;
      NsCand* rows = alloc.get<NsCand>(n_dst * (int64_t)row_cap, COOP_TAG_SCRATCH);
      uint32_t* n_cand = alloc.get<uint32_t>(n_dst, COOP_TAG_SCRATCH);
      if (alloc.failed) return COOP_E_NOMEM;
      if (cx.vec4) COOP_LAUNCH(K_NS_FILL, k_ns_collect<true>, grid_q, dim3(wpb * kWave), shmem, s, COOP_NS_ARGS, rows, row_cap, n_cand, long_min,
                               (const uint32_t*)long_list, (const uint32_t*)n_long, long_blocks);
      else COOP_LAUNCH(K_NS_FILL, k_ns_collect<false>, grid_q, dim3(wpb * kWave), shmem, s, COOP_NS_ARGS, rows, row_cap, n_cand, long_min,
                       (const uint32_t*)long_list, (const uint32_t*)n_long, long_blocks);
      COOP_LAUNCH(K_NS_SELECT, k_ns_select, grid, dim3(wpb * kWave), shmem, s, rec, n_dst, k, cap, wpb, vp, blk->indptr, blk->col_global, blk->eid,
                  (const NsCand*)rows, row_cap, n_cand, (const NsBlendThr*)bthr);
      if (cx.vec4) COOP_LAUNCH(K_NS_FILL, (k_ns_fill<true, true>), grid, dim3(wpb * kWave), shmem, s, COOP_NS_ARGS, (const uint32_t*)n_cand, 0u,
                               (const uint32_t*)nullptr, (const uint32_t*)nullptr, 0);
      else COOP_LAUNCH(K_NS_FILL, (k_ns_fill<true, false>), grid, dim3(wpb * kWave), shmem, s, COOP_NS_ARGS, (const uint32_t*)n_cand, 0u,
                       (const uint32_t*)nullptr, (const uint32_t*)nullptr, 0);
    } else {
      if (cx.vec4) COOP_LAUNCH(K_NS_FILL, (k_ns_fill<false, true>), grid_q, dim3(wpb * kWave), shmem, s, COOP_NS_ARGS, (const uint32_t*)nullptr, long_min,
                               (const uint32_t*)long_list, (const uint32_t*)n_long, long_blocks);
      else COOP_LAUNCH(K_NS_FILL, (k_ns_fill<false, false>), grid_q, dim3(wpb * kWave), shmem, s, COOP_NS_ARGS, (const uint32_t*)nullptr, long_min,
                       (const uint32_t*)long_list, (const uint32_t*)n_long, long_blocks);
    }
#undef COOP_NS_ARGS
    if (k > kNsMaxSelect) {  // the lists longer than such a fanout (the kernels above skip them)
      const dim3 grid_w(blocks_for(n_dst, kWavesPerBlock));
      if (cx.blend) COOP_LAUNCH(K_NS_FILL, k_ns_fill_wide<true>, grid_w, dim3(kBlock), 0, s, cx.g->indices, rec, n_dst, k, vp, blk->indptr,
                                blk->col_global, blk->eid, m);
      else COOP_LAUNCH(K_NS_FILL, k_ns_fill_wide<false>, grid_w, dim3(kBlock), 0, s, cx.g->indices, rec, n_dst, k, vp, blk->indptr,
                       blk->col_global, blk->eid, m);
    }
  }
  return COOP_OK;
}

}  // namespace coop
