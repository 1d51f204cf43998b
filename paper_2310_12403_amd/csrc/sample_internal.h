// Pieces shared by the sampling driver (sample.hip) and the two samplers (labor.hip, ns.hip).
#pragma once
#include "coop_internal.h"
#include "variates.h"

namespace coop {

constexpr int kMaxFuse = 4;  // LABOR-0: most layers whose keep tests are evaluated in one scan of a list

// Everything a sampler needs to know about the call.
struct SampleCtx {
  const coop_graph* g;
  hipStream_t s;
  Alloc* alloc;
  Ctl* d_ctl;
  Ctl* h_ctl;
  uint32_t* d_piece_count;  // [L] zeroed at the start of the call: pieces queued by the LABOR-0 pass that ran at layer l
  const int32_t* fanouts;
  int L;
  int sampler;
  uint64_t seed;   // user seed
  uint64_t group;  // g = floor(iter / kappa)
  bool blend;      // c > 0
  double cw, sw;   // cos(c pi/2), sin(c pi/2)
  bool vec4;       // the graph's indices array is 16-byte aligned
};

// One destination's neighbour list as the scan kernels see it.
struct Segment { int64_t beg; uint32_t d; uint32_t split; };  // split != 0: scanned piecewise by several waves

// The q-th stretch of a long list, scanned by one wave (LABOR-0).  list == kNoPiece: an empty queue slot.
struct Piece { uint32_t list, q; };
constexpr uint32_t kNoPiece = 0xFFFFFFFFu;

struct StageEntry { int32_t t; uint32_t j; };  // kept source vertex, its position in the destination's list

// What one LABOR-0 scan pass leaves behind for the layers it covered (f = 0 is the pass's own layer).
struct LaborPass {
  int first_layer = 0;               // the layer at which the pass ran
  int64_t start = 0, n_new = 0;      // destinations [start, start + n_new) of the layer were scanned in this pass
  Segment* seg = nullptr;            // [n_new]
  uint32_t* thr = nullptr;           // [nf][n_new] keep thresholds, layer-major
  int nf = 0;                        // layers covered: l .. l + nf - 1
  StageEntry* stage[kMaxFuse] = {};  // [n_new][stage_cap] kept edges per covered layer
  int32_t* cnt[kMaxFuse] = {};       // [n_new] kept-edge counts per covered layer
};

struct LaborState {
  LaborPass pass[kMaxFuse];  // the passes that covered all remaining layers of their destinations
  int n_pass = 0;
  int64_t covered = 0;       // destinations [0, covered) have every remaining layer staged by those passes
  bool fuse = false;
  uint32_t stage_cap = 32;
  // LABOR-0 from the neighbours' side: the item list of the vertices with a small variate, per layer, for passes that
  // come later and cover the same layer (device memory of this call's scratch)
  struct Listed { struct EnumItem* item = nullptr; uint32_t* n = nullptr; uint32_t cap = 0, u_max = 0; };
  static constexpr int kMaxListed = 8;
  Listed listed[kMaxListed];
};

// Parameters of the random-walk sampler (App. A.1.3).
struct RwConfig {
  int32_t walk_length;   // o
  int32_t n_walks;       // a
  uint64_t restart_thr;  // floor(p 2^32); a step restarts iff its draw is below
};

// Each fills blk->indptr, n_edges, col_global, eid and allocates col_local for layer l over dst[0..n_dst).
// With edge_cap == 0 the edge count is read back (the stream is synchronised once) and the arrays have its size.
// With edge_cap > 0 nothing is read back: the arrays get edge_cap entries, the fill writes no edge beyond them, the
// exact count stays on the device (control block, total_edges) and blk->n_edges is left at -1; the caller learns the
// count with its next read-back and must redo the layer with edge_cap == 0 if the count exceeds edge_cap, if LABOR-0
// reports a staging-row or candidate-buffer overflow, or whenever it prefers to.
int labor_layer(LaborState& st, const SampleCtx& cx, int l, const int32_t* dst, int64_t n_dst, coop_block* blk, int64_t edge_cap);
int ns_layer(const SampleCtx& cx, int l, const int32_t* dst, int64_t n_dst, coop_block* blk, int64_t edge_cap);
int rw_layer(const SampleCtx& cx, const RwConfig& rw, int l, const int32_t* dst, int64_t n_dst, coop_block* blk, int64_t edge_cap);

// tuning knobs (coop_tune)
extern int g_stage_cap_override;
extern int g_lists_per_wave;
extern int g_fuse_layers;
extern int g_piece_len;
extern int g_split_min;
extern int64_t g_blend_candidates;
extern int g_defer_sizes;
extern int g_enum_degree;
extern int g_ns_long_min;   // COOP_TUNE_NS_LONG_LIST (defined in ns.hip)

static inline unsigned blocks_for(int64_t n, int64_t per_block) { return (unsigned)((n + per_block - 1) / per_block); }

}  // namespace coop
