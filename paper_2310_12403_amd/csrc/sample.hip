// coop_sample: the sampling loop of Algorithm 1 on one GPU.  Per layer: the sampler (labor.hip / ns.hip) produces the
// kept edges of S^l in (destination order, adjacency order); unique.hip forms S^{l+1} (Eq. 2) and the local ids.
#include <math.h>

#include "device_utils.h"
#include "sample_internal.h"

namespace coop {

__global__ __launch_bounds__(kBlock) void k_copy_i32(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = in[i];
}

// start of a sampling call: the seed list is copied to the first block's dst_ids and the control data cleared
__global__ __launch_bounds__(kBlock) void k_begin_call(const int32_t* __restrict__ seeds, int32_t* __restrict__ seed_copy, int64_t n_seeds,
                                                       Ctl* ctl, uint32_t* piece_count, int L) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n_seeds) seed_copy[i] = seeds[i];
  if (i == 0) {
    *ctl = Ctl{};
    for (int l = 0; l < L; ++l) piece_count[l] = 0;
  }
}

// The control block travels to the host by a one-thread kernel that stores it into mapped pinned memory and then a
// ticket; the host polls the ticket.  That is a few microseconds quicker per read-back than an asynchronous copy
// followed by a stream synchronisation, and a sampling call has one read-back per layer (two for a layer that is redone or has a large fanout).  The wait is bounded: after
// a while the host falls back to synchronising the stream.
__global__ void k_publish_ctl(const Ctl* __restrict__ d_ctl, HostCtl* h, uint64_t ticket) {
  h->ctl = *d_ctl;
  __threadfence_system();
  __hip_atomic_store(&h->ticket, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

Publish begin_publish(Ctl* d_ctl, Ctl* h_ctl) {
  HostCtl* h = reinterpret_cast<HostCtl*>(h_ctl);  // h_ctl is the first member of a HostCtl in mapped pinned memory
  return Publish{d_ctl, h, ++h->next_ticket};
}

int launch_publish(const Publish& pub, hipStream_t s) {
  hipLaunchKernelGGL(k_publish_ctl, dim3(1), dim3(1), 0, s, pub.d_ctl, pub.h, pub.ticket);
  return hipGetLastError() == hipSuccess ? COOP_OK : COOP_E_HIP;
}

int wait_ctl(const Publish& pub, Ctl* h_ctl, hipStream_t s) {
  HostCtl* h = pub.h;
  const uint64_t ticket = pub.ticket;
  bool seen = false;
  for (int64_t spin = 0; spin < ((int64_t)1 << 26); ++spin) {
    if (__atomic_load_n(&h->ticket, __ATOMIC_ACQUIRE) == ticket) { seen = true; break; }
    if ((spin & 0xFFFF) == 0xFFFF && hipStreamQuery(s) == hipSuccess) break;  // the stream ran dry: look once more below
    __builtin_ia32_pause();
  }
  if (!seen) {
    if (hipStreamSynchronize(s) != hipSuccess) return COOP_E_HIP;
    if (__atomic_load_n(&h->ticket, __ATOMIC_ACQUIRE) != ticket) return COOP_E_HIP;
  }
  if (h_ctl->err_range) return COOP_E_RANGE;
  if (h_ctl->err_dup) return COOP_E_DUPSEED;
  if (h_ctl->err_capacity) return COOP_E_CAPACITY;
  return COOP_OK;
}

int read_ctl(Ctl* d_ctl, Ctl* h_ctl, hipStream_t s) {
  const Publish pub = begin_publish(d_ctl, h_ctl);
  if (launch_publish(pub, s) != COOP_OK) return COOP_E_HIP;
  return wait_ctl(pub, h_ctl, s);
}

int g_stage_cap_override = 0;  // COOP_TUNE_STAGE_CAP
int g_lists_per_wave = 0;      // COOP_TUNE_LISTS_PER_WAVE (0 = automatic)
int g_fuse_layers = 1;         // COOP_TUNE_FUSE_LAYERS
int g_piece_len = 4096;        // COOP_TUNE_PIECE_LEN
int g_split_min = 0;           // COOP_TUNE_SPLIT_MIN (0 = twice the piece length)
int64_t g_blend_candidates = 0;  // COOP_TUNE_BLEND_CANDIDATES (0 = automatic)
int g_defer_sizes = 1;         // COOP_TUNE_DEFER_SIZES
int g_enum_degree = 8192;      // COOP_TUNE_ENUM_DEGREE

// puts back what a LABOR-0 pass at layer l changed in the control data, before the pass is run again
__global__ void k_reset_layer(Ctl* ctl, uint32_t* piece_count) {
  ctl->cand_overflow = 0;
  *piece_count = 0;
}

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
    case COOP_TUNE_FUSE_LAYERS:
      if (value < 0 || value > 2) return COOP_E_ARG;
      g_fuse_layers = (int)value;
      return COOP_OK;
    case COOP_TUNE_PIECE_LEN:
      if (value != 0 && (value < 256 || value > ((int64_t)1 << 24) || (value & 3))) return COOP_E_ARG;
      g_piece_len = (int)value;
      return COOP_OK;
    case COOP_TUNE_BLEND_CANDIDATES:
      if (value < 0 || value > ((int64_t)1 << 30)) return COOP_E_ARG;
      g_blend_candidates = value;
      return COOP_OK;
    case COOP_TUNE_UNIQUE:
      if (value < 0 || value > 3) return COOP_E_ARG;
      g_unique_mode = (int)value;
      return COOP_OK;
    case COOP_TUNE_ENUM_DEGREE:
      if (value != 0 && (value < 64 || value > ((int64_t)1 << 30))) return COOP_E_ARG;
      g_enum_degree = (int)value;
      return COOP_OK;
    case COOP_TUNE_DEFER_SIZES:
      if (value < 0 || value > 2) return COOP_E_ARG;
      g_defer_sizes = (int)value;
      return COOP_OK;
    case COOP_TUNE_SPLIT_MIN:
      if (value != 0 && (value < 64 || value > ((int64_t)1 << 30))) return COOP_E_ARG;
      g_split_min = (int)value;
      return COOP_OK;
    case COOP_TUNE_NS_LONG_LIST:
      if (value != 0 && (value < 64 || value > ((int64_t)1 << 30))) return COOP_E_ARG;
      g_ns_long_min = (int)value;
      return COOP_OK;
    default:
      return COOP_E_ARG;
  }
}

static int sample_layers(const coop_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int L,
                         int sampler, const RwConfig* rw, uint64_t iter, uint32_t kappa, uint64_t seed, coop_alloc_fn alloc_fn,
                         void* alloc_ctx, void* stream, coop_block* blocks_out) {
  if (!g || !fanouts || !blocks_out || !alloc_fn || (!seeds && n_seeds > 0)) return COOP_E_NULL;
  if (L < 1 || L > 255 || n_seeds < 0 || n_seeds >= ((int64_t)1 << 31)) return COOP_E_ARG;
  if (sampler != COOP_NS && sampler != COOP_LABOR0 && !(sampler == COOP_RW && rw)) return COOP_E_ARG;
  for (int l = 0; l < L; ++l)
    if (fanouts[l] < 1) return COOP_E_ARG;
  for (int l = 0; l < L; ++l) blocks_out[l] = coop_block{};

  hipStream_t s = (hipStream_t)stream;
  Alloc alloc{alloc_fn, alloc_ctx};

  SampleCtx cx{};
  cx.g = g; cx.s = s; cx.alloc = &alloc; cx.fanouts = fanouts; cx.L = L; cx.sampler = sampler; cx.seed = seed;
  cx.vec4 = ((uintptr_t)g->indices & 15) == 0;
  // group / interpolation state of App. A.7: g = floor(iter / kappa), c = (iter mod kappa) / kappa
  cx.group = 0; cx.blend = false; cx.cw = 1.0; cx.sw = 0.0;
  if (kappa != 0) {
    const uint64_t i = iter % kappa;
    cx.group = iter / kappa;
    cx.blend = i != 0;
    const double c = (double)i / (double)kappa;
    cx.cw = cos(c * 1.5707963267948966);
    cx.sw = sin(c * 1.5707963267948966);
  }

  // pinned landing pad for the size read-backs, one per calling thread, kept for the life of the process
  static thread_local HostCtl* h_pad = nullptr;
  if (!h_pad) {
    COOP_HIP_TRY(hipHostMalloc((void**)&h_pad, sizeof(HostCtl), hipHostMallocMapped | hipHostMallocCoherent));
    *h_pad = HostCtl{};
  }
  Ctl* h_ctl = &h_pad->ctl;
  cx.h_ctl = h_ctl;
  cx.d_ctl = alloc.get<Ctl>(1, COOP_TAG_SCRATCH);
  cx.d_piece_count = alloc.get<uint32_t>(L, COOP_TAG_SCRATCH);
  int32_t* seed_copy = alloc.get<int32_t>(n_seeds, COOP_TAG_OUTPUT);
  if (alloc.failed) return COOP_E_NOMEM;
  COOP_LAUNCH(K_COPY_IDS, k_begin_call, dim3(n_seeds > 0 ? blocks_for(n_seeds, kBlock) : 1u), dim3(kBlock), 0, s, seeds, seed_copy, n_seeds,
              cx.d_ctl, cx.d_piece_count, L);

  LaborState labor;
  bool defer_ok = true;
  const int32_t* dst = seed_copy;
  int64_t n_dst = n_seeds;
  int rc = COOP_OK;
  for (int l = 0; l < L && rc == COOP_OK; ++l) {
    coop_block blk{};
    blk.n_dst = n_dst;
    blk.dst_ids = const_cast<int32_t*>(dst);
    // Edge arrays sized from a bound on m_l instead of m_l itself: the layer then needs one read-back (after the
    // dedup's scan, which brings m_l along) instead of two.  NS and random walks keep at most k per destination; LABOR-0
    // keeps sum min(d, k) in expectation with a variance below k per destination, so 8 standard deviations of room
    // all but never fall short, and when they do (or a staging row or the candidate buffer overflows) the layer is
    // redone the slow way.
    const int64_t k_l = sampler == COOP_RW ? (fanouts[l] < rw->walk_length * rw->n_walks ? fanouts[l] : rw->walk_length * rw->n_walks)
                                           : fanouts[l];
    int64_t edge_cap = 0;
    // (only for the small fanouts of GNN training: with a large one the bound can exceed the count many times over)
    if (g_defer_sizes != 0 && defer_ok && n_dst > 0 && k_l <= 64 && k_l * n_dst <= ((int64_t)1 << 28)) {
      edge_cap = k_l * n_dst;
      if (sampler == COOP_LABOR0) edge_cap += 8 * (int64_t)sqrt((double)edge_cap) + 4096;
      if (g_defer_sizes == 2) edge_cap = edge_cap / 2 + 1;  // (test knob) a bound that falls short
      if (n_dst + edge_cap >= ((int64_t)1 << 32) - 1) edge_cap = 0;
    }
    const LaborState labor_before = labor;
    auto sample_layer = [&](int64_t cap) {
      return sampler == COOP_LABOR0 ? labor_layer(labor, cx, l, dst, n_dst, &blk, cap)
             : sampler == COOP_NS   ? ns_layer(cx, l, dst, n_dst, &blk, cap)
                                    : rw_layer(cx, *rw, l, dst, n_dst, &blk, cap);
    };
    UniqueWork uw{};
    int32_t* src = nullptr;
    int64_t n_src = 0;
    bool done = false, redone = false;
    if (edge_cap > 0) {
      rc = sample_layer(edge_cap);
      if (rc != COOP_OK) break;
      const int64_t* m_dev = &cx.d_ctl->total_edges;
      rc = unique_front_launch(dst, n_dst, blk.col_global, edge_cap, m_dev, &uw, alloc, cx.d_ctl, h_ctl, s);
      if (rc != COOP_OK) break;
      // S^{l+1} and local ids (Eq. 2) are queued before the sizes are back, with room for the bound, so that the device
      // is at work while the host waits for the sizes and sets up the next layer
      src = alloc.get<int32_t>(n_dst + edge_cap, COOP_TAG_OUTPUT);
      if (alloc.failed) { rc = COOP_E_NOMEM; break; }
      rc = unique_back(dst, n_dst, blk.col_global, edge_cap, m_dev, uw, blk.col_local, src, s);
      if (rc != COOP_OK) break;
      rc = unique_front_finish(dst, n_dst, blk.col_global, edge_cap, m_dev, &uw, alloc, cx.d_ctl, h_ctl, s, &redone);
      if (rc != COOP_OK) break;
      if (h_ctl->n_overflow > 0) defer_ok = false;  // the counter is never reset: the overflow pass runs from here on
      if (h_ctl->total_edges <= edge_cap && h_ctl->n_overflow == 0 && h_ctl->cand_overflow == 0) {
        blk.n_edges = h_ctl->total_edges;
        if (redone) rc = unique_back(dst, n_dst, blk.col_global, edge_cap, m_dev, uw, blk.col_local, src, s);
        if (rc != COOP_OK) break;
        done = true;
      } else {
        labor = labor_before;
        hipLaunchKernelGGL(k_reset_layer, dim3(1), dim3(1), 0, s, cx.d_ctl, cx.d_piece_count + l);
        blk = coop_block{};
        blk.n_dst = n_dst;
        blk.dst_ids = const_cast<int32_t*>(dst);
      }
    }
    if (!done) {
      rc = sample_layer(0);
      if (rc != COOP_OK) break;
      if (n_dst + blk.n_edges >= ((int64_t)1 << 32) - 1) { rc = COOP_E_CAPACITY; break; }
      rc = unique_front_launch(dst, n_dst, blk.col_global, blk.n_edges, nullptr, &uw, alloc, cx.d_ctl, h_ctl, s);
      if (rc != COOP_OK) break;
      rc = unique_front_finish(dst, n_dst, blk.col_global, blk.n_edges, nullptr, &uw, alloc, cx.d_ctl, h_ctl, s, &redone);
      if (rc != COOP_OK) break;
      src = alloc.get<int32_t>(n_dst + uw.n_new, COOP_TAG_OUTPUT);
      if (alloc.failed) { rc = COOP_E_NOMEM; break; }
      rc = unique_back(dst, n_dst, blk.col_global, blk.n_edges, nullptr, uw, blk.col_local, src, s);
      if (rc != COOP_OK) break;
    }
    n_src = n_dst + uw.n_new;
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

extern "C" int coop_sample(const coop_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int L,
                           int sampler, uint64_t iter, uint32_t kappa, uint64_t seed, coop_alloc_fn alloc_fn,
                           void* alloc_ctx, void* stream, coop_block* blocks_out) {
  if (sampler == COOP_RW) return COOP_E_ARG;  // the random-walk sampler has parameters of its own: coop_sample_rw
  return sample_layers(g, seeds, n_seeds, fanouts, L, sampler, nullptr, iter, kappa, seed, alloc_fn, alloc_ctx, stream, blocks_out);
}

extern "C" int coop_sample_rw(const coop_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int L,
                              int32_t walk_length, int32_t n_walks, double restart_p, uint64_t iter, uint64_t seed,
                              coop_alloc_fn alloc_fn, void* alloc_ctx, void* stream, coop_block* blocks_out) {
  if (walk_length < 1 || n_walks < 1 || (int64_t)walk_length * n_walks > ((int64_t)1 << 20)) return COOP_E_ARG;
  if (!(restart_p >= 0.0 && restart_p <= 1.0)) return COOP_E_ARG;
  RwConfig rw{};
  rw.walk_length = walk_length;
  rw.n_walks = n_walks;
  rw.restart_thr = restart_p >= 1.0 ? (uint64_t)1 << 32 : (uint64_t)(restart_p * 4294967296.0);
  // the paper defines no dependent variates for random walks: every iteration draws afresh (group = iteration)
  return sample_layers(g, seeds, n_seeds, fanouts, L, COOP_RW, &rw, iter, 1u, seed, alloc_fn, alloc_ctx, stream, blocks_out);
}

extern "C" int coop_copy_ids(const int32_t* in, int32_t* out, int64_t n, void* stream) {
  if ((!in || !out) && n > 0) return COOP_E_NULL;
  if (n < 0 || n >= ((int64_t)1 << 39)) return COOP_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (n > 0) COOP_LAUNCH(K_COPY_IDS, k_copy_i32, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, s, in, out, n);
  return COOP_OK;
}
