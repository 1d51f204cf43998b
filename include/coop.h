/*
 * coop.h — C ABI of libcoop: minibatch subgraph sampling and feature loading for GNN
 * training on one AMD MI355X (gfx950), after "Cooperative Minibatching in Graph Neural
 * Networks".  One GPU plays the single large processor that owns the whole cooperative
 * batch (Sec. 3.1): Algorithm 1's sampling loop without the all-to-all, then its feature
 * loading step.
 *
 * Conventions
 *   - Every function returns COOP_OK (0) or a negative COOP_E_* code; nothing throws or
 *     aborts across this boundary.  coop_strerror() names a code.
 *   - "device" pointers are HIP device addresses valid on the current device; "host"
 *     pointers are ordinary host memory.  All device arrays passed IN are borrowed: the
 *     caller keeps them alive and unchanged until the call's work on `stream` is done.
 *   - Device memory handed OUT comes from the caller's allocator callback, so the caller
 *     (e.g. a PyTorch caching allocator) owns all of it.  The library frees none of it.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All kernels
 *     of a call run on it.  Calls that return sizes to the host synchronise that stream.
 *   - Vertex ids are int32 (0 <= id < n_vertices < 2^31); edge positions are int64.
 */
#ifndef COOP_H_
#define COOP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* error codes */
#define COOP_OK 0
#define COOP_E_NULL (-1)      /* a required pointer is NULL */
#define COOP_E_RANGE (-2)     /* a vertex id / seed is outside [0, n_vertices) */
#define COOP_E_DUPSEED (-3)   /* the seed list holds a vertex twice */
#define COOP_E_ARG (-4)       /* bad scalar argument (L < 1, fanout < 1, unknown sampler/dtype, ...) */
#define COOP_E_NOMEM (-5)     /* the allocator callback returned NULL */
#define COOP_E_CAPACITY (-6)  /* a fixed-size workspace would overflow */
#define COOP_E_HIP (-7)       /* a HIP runtime call failed */
#define COOP_E_GRAPH (-8)     /* malformed CSR (COOP_VALIDATE), or a graph registered with COOP_SYMMETRIC is not symmetric */

/* samplers (App. A.1) */
#define COOP_NS 0       /* neighbour sampling: d_s <= k -> all neighbours, else k uniform without replacement */
#define COOP_LABOR0 1   /* LABOR-0: edge (t->s) kept iff r_t <= k/d_s, one r_t per source vertex and layer */
#define COOP_RW 2       /* random walks (coop_sample_rw only) */

/* feature element types */
#define COOP_F32 0
#define COOP_F16 1

/* coop_graph_load flags */
#define COOP_VALIDATE 1
#define COOP_SYMMETRIC 2 /* the caller states that every list is strictly ascending and that t is in N(s) exactly when s is
                            in N(t) (an undirected graph stored both ways); lets LABOR-0 serve its longest lists from the
                            other side */

/* allocator tags: what the requested buffer is for */
#define COOP_TAG_OUTPUT 0   /* referenced by a coop_block; lives as long as the caller wants */
#define COOP_TAG_SCRATCH 1  /* dead once the call that asked for it has returned */
#define COOP_TAG_GRAPH 2    /* belongs to a graph handle (coop_graph_load_with): must stay valid until coop_graph_free */

/* Returns a device pointer to at least `bytes` bytes, 256-byte aligned, or NULL. */
typedef void* (*coop_alloc_fn)(void* ctx, size_t bytes, int tag);

/* A bump allocator over one caller-provided device buffer, usable as (coop_arena_alloc, &arena)
 * wherever a coop_alloc_fn is asked for: no allocation happens inside the sampling call.
 * Set used = 0 to recycle the buffer once the previous call's blocks are no longer needed. */
typedef struct {
  void* base;    /* device, 256-byte aligned */
  size_t bytes;  /* size of the buffer */
  size_t used;   /* bump offset, advanced by coop_arena_alloc */
} coop_arena;
void* coop_arena_alloc(void* arena /* coop_arena* */, size_t bytes, int tag);

typedef struct coop_graph coop_graph; /* opaque */
typedef struct coop_cache coop_cache; /* opaque */

/*
 * Registers a graph (Sec. 2: N(s) = { t | (t -> s) in E }) given as CSR over destinations:
 * the in-neighbours of s are indices[indptr[s] .. indptr[s+1]).
 *   indptr  device int64 [n_vertices + 1], indptr[0] = 0, nondecreasing, indptr[n_vertices] = n_edges
 *   indices device int32 [n_edges], each in [0, n_vertices)
 * Both arrays are borrowed for the lifetime of the handle.  With COOP_VALIDATE the arrays are
 * checked on the GPU (on `stream`, synchronously) and COOP_E_GRAPH is returned if malformed.  With COOP_SYMMETRIC the
 * arrays are checked as well, together with the caller's statement (COOP_E_GRAPH if it does not hold), and the library
 * builds an index of reverse-edge positions on the device: 4 bytes per edge, allocated with hipMalloc, one bisection per
 * edge (about a second per billion edges), released by coop_graph_free.
 */
int coop_graph_load(const int64_t* indptr, const int32_t* indices, int64_t n_vertices, int64_t n_edges,
                    int flags, void* stream, coop_graph** out);
/* The same, with every byte of device memory from the caller's allocator (Sec. 2's graph is the caller's; so is what is built
 * on it): the index of reverse positions of a COOP_SYMMETRIC graph (4 * n_edges bytes, tag COOP_TAG_GRAPH, the caller keeps
 * it alive until coop_graph_free and frees it afterwards) and a few bytes for the checks (tag COOP_TAG_SCRATCH).  With a
 * NULL allocator it is coop_graph_load.  COOP_E_NOMEM if the allocator returns NULL. */
int coop_graph_load_with(const int64_t* indptr, const int32_t* indices, int64_t n_vertices, int64_t n_edges, int flags,
                         coop_alloc_fn alloc, void* alloc_ctx, void* stream, coop_graph** out);
int coop_graph_free(coop_graph* g);

/*
 * One sampling layer l of Algorithm 1 as a bipartite block S^{l+1} -> S^l with edges E^l.
 * All pointers are device memory from the allocator (tag COOP_TAG_OUTPUT).
 */
typedef struct {
  int64_t n_dst;       /* |S^l|      */
  int64_t n_src;       /* |S^{l+1}|  */
  int64_t n_edges;     /* |E^l|      */
  int32_t* dst_ids;    /* [n_dst]    S^l, global ids; layer 0: a copy of the seeds; layer l > 0: the previous src_ids */
  int64_t* indptr;     /* [n_dst+1]  edges sampled for dst i are [indptr[i], indptr[i+1]), in adjacency order */
  int32_t* col_local;  /* [n_edges]  position of the edge's source vertex in src_ids */
  int32_t* col_global; /* [n_edges]  global id of the edge's source vertex */
  int64_t* eid;        /* [n_edges]  position of the edge in the graph's `indices` array (NS, LABOR-0); for random
                                     walks, whose sampled edges are edges of A + A^2 + .. + A^o, the visit count */
  int32_t* src_ids;    /* [n_src]    S^{l+1} = S^l ∪ sampled sources (Eq. 2): S^l first, in order, then every new
                                     vertex in order of first appearance in col_global */
} coop_block;

/*
 * Multi-layer minibatch sampling: the sampling loop of Algorithm 1 on one processor.
 * For l = 0 .. L-1, with S^0 = seeds: samples the in-neighbourhood of every s in S^l with fanout
 * fanouts[l] (fanouts[0] is the seeds' hop) by NS (App. A.1.1) or LABOR-0 (App. A.1.2), then forms
 * S^{l+1} (Eq. 2) and relabels the edges.
 *
 * Random variates (App. A.7): r = R / 2^32 where, for group g = floor(iter / kappa) and c = (iter mod kappa) / kappa,
 *   (K0..K3)(g) = Philox4x32-10 with key (seed low, seed high) and counter (g low, g high, l | sampler << 8, 0x434F4F50);
 *   U(g) = mix(t ^ K0) ^ K1 for LABOR-0 (one number per source vertex t and layer),
 *          mix(mix(t ^ K0) ^ K1 ^ mix(s ^ K2)) ^ K3 for NS (one number per edge t -> s),
 *          mix(x): x ^= x >> 16; x *= 0x7FEB352D; x ^= x >> 15; x *= 0x846CA68B; x ^= x >> 16  (32-bit);
 *   c = 0:  R = U(g);
 *   c > 0:  R = floor(2^32 Phi(cos(c pi/2) Phi^-1(u1) + sin(c pi/2) Phi^-1(u2))), u_i = (U(g+i-1) + 1/2) / 2^32.
 * kappa = 0 stands for kappa = infinity (g = 0, c = 0).  The result is a pure function of the arguments:
 * the same (seeds, fanouts, sampler, iter, kappa, seed) give the same bytes on every call.
 *
 *   g          graph handle
 *   seeds      device int32 [n_seeds], distinct, in range (else COOP_E_DUPSEED / COOP_E_RANGE)
 *   fanouts    host int32 [L], each >= 1, no upper limit (NS with a fanout above 1024: the lists longer than the fanout
 *              go through a slower selection that bisects on the variate instead of collecting candidates)
 *   blocks_out host coop_block [L], filled on success
 * Waits on `stream` once per layer, for |E^l| and |S^{l+1}| together: with a fanout of at most 64 the edge arrays are
 * obtained from the allocator with room for a bound on |E^l| (fanout x |S^l|, plus a little for LABOR-0) and src_ids
 * with room for |S^l| plus that bound, so they may be longer than n_edges / n_src entries; a layer whose bound falls
 * short is redone.  With a larger fanout |E^l| is read back
 * first (a second wait) and the arrays have exactly n_edges entries.  When it returns all
 * sizes in blocks_out are final, while the kernels that fill the last layer's col_local / src_ids may still be running
 * on `stream`: work queued on the same stream sees complete blocks, anything else must synchronise the stream first.
 * On error blocks_out is zeroed; buffers already obtained from the allocator stay with the caller.
 */
int coop_sample(const coop_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int L,
                int sampler, uint64_t iter, uint32_t kappa, uint64_t seed, coop_alloc_fn alloc, void* alloc_ctx,
                void* stream, coop_block* blocks_out);

/*
 * Multi-layer minibatch sampling with the random-walk sampler (App. A.1.3): as coop_sample, but the neighbourhood of
 * every s in S^l is formed by n_walks random walks of walk_length steps from s.  The first step of a walk goes to a
 * uniformly drawn in-neighbour of s; each later step goes to a uniformly drawn in-neighbour of the current vertex or,
 * with probability restart_p, of s; a walk that reaches a vertex without in-neighbours ends.  The fanouts[l] most
 * visited vertices (ties: smaller id first; s itself counts only when a step lands on it) become the sources of s,
 * emitted in that order; eid holds their visit counts.
 *
 * Draws: the paper defines no dependent variates for random walks, so every iteration draws afresh.  With
 * (K0..K3) = the key words above for sampler COOP_RW, layer l and g = iter, draw number c of destination s is
 * U_c = mix(mix(c ^ K0) ^ K1 ^ mix(s ^ K2)) ^ K3; step i of walk w picks neighbour floor(U_{2(w o + i)} d / 2^32) of
 * its base vertex (d = that vertex's degree) and, for i >= 1, restarts iff U_{2(w o + i) + 1} < floor(restart_p 2^32).
 *
 *   walk_length >= 1, n_walks >= 1, walk_length * n_walks <= 2^20, 0 <= restart_p <= 1 (else COOP_E_ARG); with more than
 *   1024 steps per destination the visit tallies live in device memory (a slower kernel)
 * Everything else (arguments, ownership, synchronisation, errors) is as for coop_sample.
 */
int coop_sample_rw(const coop_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int L,
                   int32_t walk_length, int32_t n_walks, double restart_p, uint64_t iter, uint64_t seed,
                   coop_alloc_fn alloc, void* alloc_ctx, void* stream, coop_block* blocks_out);

/*
 * Feature-loading step of Algorithm 1 (the input-layer rows of the vertices in S^L): out[i, :] = feat[ids[i], :],
 * an exact copy of bits.
 *   feat   device (or host memory mapped into the device address space) [n_rows, dim] row-major, dtype elements
 *   ids    device int32 [n_ids], each in [0, n_rows) (else COOP_E_RANGE, reported by coop_gather_status)
 *   out    device [n_ids, dim]
 * Asynchronous on `stream`: returns after the launch.  Host-checkable errors are returned at once.
 */
int coop_gather(const void* feat, int64_t n_rows, int32_t dim, int dtype, const int32_t* ids, int64_t n_ids,
                void* out, void* stream);

/*
 * Neighbour mean fused with the feature load: the aggregation of Eq. (1) with a mean aggregator over one sampled
 * block (normally the last one, whose sources are S^L), without materialising the gathered rows:
 *   out[i, :] = (1 / deg_i) * sum over e in [indptr[i], indptr[i+1]) of feat[col_global[e], :],   0 if deg_i = 0.
 * Sums are accumulated in fp32 in edge order; `out` has the dtype of `feat`.
 *   feat        device (or mapped pinned host) [n_rows, dim]
 *   indptr      device int64 [n_dst + 1] (a coop_block's indptr), col_global device int32 [indptr[n_dst]], global ids
 *   out         device [n_dst, dim]
 * Asynchronous on `stream`; ids out of range are skipped and reported by coop_gather_status.
 */
int coop_gather_mean(const void* feat, int64_t n_rows, int32_t dim, int dtype, const int64_t* indptr,
                     const int32_t* col_global, int64_t n_dst, void* out, void* stream);

/* Synchronises `stream` and returns COOP_E_RANGE if any coop_gather / coop_gather_mean / coop_bucket_by_owner since the
 * last call of this function met an id outside its range (such rows of `out` are left zero-filled; such ids are left
 * out of every group), else COOP_OK.  Clears the condition. */
int coop_gather_status(void* stream);

/* vertex partitions of Sec. 3.1 (1-D: every vertex, with its in-edges, belongs to one PE) */
#define COOP_OWNER_RANGE 0  /* contiguous ranges: owner(v) = floor(v * n_parts / n_vertices) */
#define COOP_OWNER_HASH 1   /* random partition: owner(v) = floor(mix(v ^ key) * n_parts / 2^32), mix = the 32-bit mixer of
                               the variates, key = low word of seed xor high word */

/*
 * The local half of the id redistribution of Algorithm 1 (every PE sends the vertices of its frontier to the PEs that
 * own them; Sec. 3.1): the ids grouped by owner, in their original order within each group.  What one GPU does before
 * the all-to-all; the exchange itself is not part of this library.
 *   ids          device int32 [n], each in [0, n_vertices) (others: left out, reported by coop_gather_status)
 *   n_parts      1 .. 64
 *   ids_out      device int32 [n]: group p is [offsets_out[p], offsets_out[p + 1])
 *   origin_out   device int32 [n] or NULL: the position that each entry of ids_out had in ids (the way back for what the
 *                owner returns)
 *   offsets_out  device int64 [n_parts + 1]
 *   workspace    device, 8-byte aligned, at least coop_bucket_workspace_bytes(n, n_parts) bytes; contents undefined after
 * Asynchronous on `stream`; allocates nothing.
 */
size_t coop_bucket_workspace_bytes(int64_t n, int n_parts);
int coop_bucket_by_owner(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, uint64_t seed,
                         int32_t* ids_out, int32_t* origin_out, int64_t* offsets_out, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * coop_bucket_by_owner for callers that cannot allocate and have no workspace to pass: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as coop_bucket_by_owner,
 * without `workspace`: the counter matrix, its scan and the scan's tile sums live in a device array that is part of the
 * library's code object (4 MiB + 64 KiB; every GPU that the library runs on holds its copy until the process ends).
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library routine), launches the same kernels on
 * `stream` and returns after the launches.
 * Limits: n < 2^31 ids, n_parts <= 64, as for coop_bucket_by_owner (COOP_E_ARG beyond them); a call whose workspace
 * would not fit the array gets COOP_E_CAPACITY (none does within those limits).
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams, different threads) race
 * and give wrong groups; calls queued on one stream, or ordered by events, are fine.  Nothing in the array has to
 * survive from call to call or start at zero.
 */
int coop_bucket_by_owner_static(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, uint64_t seed,
                                int32_t* ids_out, int32_t* origin_out, int64_t* offsets_out, void* stream);

/*
 * LRU vertex cache on the GPU in front of a feature table that the device can read but that is slow to read
 * (pinned host memory over the host link; Sec. 4.2 measures this cache's miss rate as kappa grows).
 *
 * Semantics: a textbook LRU fed, per call, first the ids that are cached when the call starts, then the ids
 * that are not, each in list order.  Hits are served from the cache and become most recent; misses are read
 * from `table`; after the call the cache holds the `capacity_rows` most recently touched vertices.
 *
 * coop_cache_create: all device memory (slot map int32[n_vertices], capacity_rows rows, stamps, and scratch for
 * up to max_ids ids per call) comes from the allocator once; later calls allocate nothing.
 * Synchronises `stream`.
 */
int coop_cache_create(int64_t capacity_rows, int64_t n_vertices, int32_t dim, int dtype, int64_t max_ids,
                      coop_alloc_fn alloc, void* alloc_ctx, void* stream, coop_cache** out);
int coop_cache_free(coop_cache* c);

/*
 * out[i, :] = table[ids[i], :] through the cache.
 *   table      [table_rows, dim] rows of the dtype given at creation: device memory, or pinned host memory
 *              mapped into the device address space (read by the kernels directly, no staging copy)
 *   table_rows rows in `table` (>= 1).  Vertex v reads row v mod table_rows: pass n_vertices for a full table; a
 *              shorter table aliases rows (for benchmarks whose full table would not fit in host memory: miss
 *              counts and bytes per miss are those of the full table)
 *   ids        device int32 [n_ids], DISTINCT, each in [0, n_vertices) (else COOP_E_RANGE); n_ids <= max_ids
 *              (else COOP_E_CAPACITY)
 *   out        device [n_ids, dim]
 *   n_miss_out host, number of ids that were not cached when the call started (may be NULL)
 * Returns once the hit / miss counts are known (the host waits for that much of `stream`, no more); the eviction and
 * the copies of the miss rows are queued on `stream` and may still be running when it returns: a host that wants `out`
 * synchronises `stream`.  Calls on one cache must not overlap, and follow one another on one stream or are ordered by
 * the caller.  After COOP_E_RANGE the in-range cached ids of the
 * call count as touched and nothing was inserted; `out` is then unspecified.
 */
int coop_cache_gather(coop_cache* c, const void* table, int64_t table_rows, const int32_t* ids, int64_t n_ids, void* out,
                      int64_t* n_miss_out, void* stream);

/*
 * Checkpoint / resume of a cache.  coop_cache_export writes the cached vertices and their recency stamps (in no
 * particular order; state_out->size of them) to two caller-owned device arrays of `capacity_rows` entries each and
 * the scalar state to state_out; it synchronises `stream`.  coop_cache_import puts a cache created with the same
 * capacity (or a larger one) into exactly that state, reading the rows again from `table`; duplicate vertices or
 * vertices out of range in the list give COOP_E_RANGE (the cache is then empty).  After an import the cache answers
 * every later coop_cache_gather as the exported one would have.
 */
typedef struct {
  int64_t size;    /* cached vertices */
  uint64_t clock;  /* next recency stamp */
  uint64_t base;   /* lower bound of the live stamps */
} coop_cache_state;
int coop_cache_export(coop_cache* c, int32_t* vertices_out, uint64_t* stamps_out, coop_cache_state* state_out, void* stream);
int coop_cache_import(coop_cache* c, const void* table, int64_t table_rows, const int32_t* vertices, const uint64_t* stamps,
                      const coop_cache_state* state, void* stream);

/* Device-side address of pinned (page-locked, mapped) host memory, for use as `table` / `feat` above.
 * COOP_E_ARG if `host` is not such memory: nothing is ever dereferenced that the device cannot read. */
int coop_map_host_pointer(const void* host, void** device_out);

/* Device pointer to the cache's slot table (vertex id per slot, -1 = empty, int32 [capacity_rows]) and the
 * number of cached vertices; valid until coop_cache_free.  For inspection and tests. */
int coop_cache_vertices(const coop_cache* c, const int32_t** vertex_of_out, int64_t* size_out);

/* Name of an error code (static string). */
const char* coop_strerror(int code);

/*
 * Tuning knobs (process-wide; for experiments and tests, results never depend on them).
 *   COOP_TUNE_STAGE_CAP    entries per LABOR-0 staging row (power of two, 1..64; 0 = automatic)
 *   COOP_TUNE_LISTS_PER_WAVE  see below
 */
#define COOP_TUNE_STAGE_CAP 1
#define COOP_TUNE_LISTS_PER_WAVE 2 /* neighbour lists handled by one wave of the LABOR-0 scan: 1..64, 0 = automatic */
#define COOP_TUNE_FUSE_LAYERS 3    /* 1 (default): a LABOR-0 list is scanned once for all remaining layers, except that a
                                      pass over fewer than 32768 lists covers its own layer only; 2: always fused; 0: never */
#define COOP_TUNE_PIECE_LEN 4      /* a LABOR-0 list longer than twice this many entries is cut into pieces of about this
                                      many entries, each scanned by a wave of its own: multiple of 4 in 256..2^24
                                      (default 4096); 0: lists are never cut */
#define COOP_TUNE_BLEND_CANDIDATES 5 /* first size (entries) of the buffer that holds the candidates of the exact blend of a
                                      LABOR-0 pass with c > 0; a pass that overflows it is redone with 8 times the size;
                                      0 (default): k / 2 entries per destination and layer plus 65536 */
#define COOP_TUNE_DEFER_SIZES 6    /* 1 (default): a layer's edge arrays are sized from a bound on |E^l| and the exact size
                                      is read back together with |S^{l+1}|; 0: |E^l| is read back first and the arrays have
                                      exactly that size; 2: as 1 with a bound that falls short, so that every layer is redone
                                      (exercises the fallback) */
#define COOP_TUNE_UNIQUE 7         /* how the frontier is deduplicated.  0 (default): lists of 262,144 entries or more (S^l and
                                      the sampled edges together) by partition into buckets that are deduplicated in LDS,
                                      shorter ones through a hash table in HBM; 1: always the table in HBM; 2: by partition
                                      whatever the length; 3: as 2 with buckets 16 times too large, so that buckets overflow
                                      and the call falls back to the table (exercises the fallback) */
#define COOP_TUNE_ENUM_DEGREE 8    /* LABOR-0 with independent variates on a graph registered with COOP_SYMMETRIC: lists
                                      longer than this many entries are not read; their kept neighbours are found from the
                                      neighbours' side (default 8192; 0: never; otherwise at least 64).  Applies while no
                                      fanout exceeds 64; at 8192 and above only to passes over 65536 lists or more of a
                                      graph whose lists above 8192 entries hold an eighth of its edges (below that the
                                      listing costs more than it saves); smaller values, meant for tests, apply always */
#define COOP_TUNE_NS_LONG_LIST 9   /* NS with independent variates: destinations whose list is longer than this many entries
                                      are queued and taken by the first waves of the traversal, so that no hub starts late
                                      (default 2048, for passes over 32768 destinations or more; 0: never; other values,
                                      64..2^30, meant for tests, apply to every pass) */
#define COOP_TUNE_SPLIT_MIN 10     /* LABOR-0: lists longer than this many entries are handed to the piece waves (in pieces of
                                      about COOP_TUNE_PIECE_LEN entries, a single piece if they are shorter than that);
                                      0 (default): twice the piece length with independent variates, 2048 with dependent
                                      ones; otherwise 64..2^30 */
int coop_tune(int knob, int64_t value);

/* out[i] = in[i] for a device id list (a plain streaming copy on `stream`: 4n bytes read, 4n written).  Besides its
 * use for snapshotting seed lists it is the known-size reference that the byte counters of a profiler are scaled by. */
int coop_copy_ids(const int32_t* in, int32_t* out, int64_t n, void* stream);

/*
 * Self-check of the arithmetic behind the dependent variates of App. A.7 (c > 0): the kernels settle most neighbours
 * with Phi^-1 evaluated in fp32 by this GPU's own logarithm, square root and reciprocal instructions, and take the exact
 * binary64 evaluation only where the fp32 value lies within a margin of the decision.  That margin presumes a bound on
 * the distance between the two evaluations; this call measures the distance for the 32-bit uniforms
 * U = first .. first + count - 1 (first + count <= 2^32; the whole range takes a fraction of a second).
 *   max_gap_out host: max |fp32 Phi^-1((U + 1/2) / 2^32) - binary64 Phi^-1((U + 1/2) / 2^32)|
 *   arg_out     host, may be NULL: the smallest U at which the maximum is reached (0xFFFFFFFF for an empty range)
 *   workspace   device, 8-byte aligned, 16 bytes, contents undefined after
 * Synchronises `stream`.
 */
int coop_selftest_phi_inv_gap(uint64_t first, uint64_t count, double* max_gap_out, uint32_t* arg_out, void* workspace,
                              void* stream);

/* Library ABI version (bumped when a signature in this file changes). */
int coop_version(void);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of the library is bracketed
 * by HIP events on its stream; coop_profile_read synchronises outstanding events and returns the
 * accumulated duration and launch count of kernel `id` (0 <= id < coop_profile_kernels()).
 */
int coop_profile_enable(int on);
int coop_profile_filter(int id); /* time only kernel `id` while enabled; id < 0: every kernel (default) */
int coop_profile_reset(void);
int coop_profile_kernels(void);
const char* coop_profile_name(int id);
int coop_profile_read(int id, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* COOP_H_ */
