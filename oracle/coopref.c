/*
 * coopref — plain, slow CPU oracle for minibatch subgraph sampling.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or
 * call this file; it exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have an independent definition to compare the GPU library
 * against.  It shares no source with the GPU library.
 *
 * What it computes (paper: "Cooperative Minibatching in Graph Neural Networks"):
 *   - the recursive layer expansion S^{l+1} = S^l ∪ N~(S^l) of Eq. (2), with the
 *     neighbourhood of every s in S^l sampled by
 *       NS       (App. A.1.1): d_s <= k -> all of N(s), else k random neighbours,
 *       LABOR-0  (App. A.1.2): edge (t->s) kept iff r_t <= k / d_s, r_t shared by
 *                              every seed of the layer;
 *       RW       (App. A.1.3): a random walks of length o from s with restart
 *                              probability p, the k most visited vertices;
 *   - the random variates r_t / r_ts of App. A.7 (smoothed dependent
 *     minibatching): a PRNG keyed by (z, t, s) whose first output is the
 *     variate, two seeds z1, z2 per group of kappa iterations blended in normal
 *     space, n(c) = cos(c pi/2) n1 + sin(c pi/2) n2, r = Phi(n(c)), c = i/kappa;
 *   - the feature loading of Algorithm 1: out[i,:] = feat[S^L[i],:], and the neighbour mean of
 *     Eq. (1) over a sampled block (what a mean-aggregating first layer does with those rows);
 *   - an LRU vertex cache (Sec. 4.2 names "an LRU cache" only).
 *
 * Readings where the paper is silent (each is listed in the design notes):
 *   - the "PRNG initialised with z, t and s" is a keyed hash in two stages:
 *       (K0,K1,K2,K3) = Philox4x32-10 (Salmon et al., SC'11) with key (seed lo, seed hi)
 *                       and counter (g lo, g hi, layer | sampler<<8, 0x434F4F50);
 *       LABOR:  U = mix(t ^ K0) ^ K1                      (one number per source vertex)
 *       NS:     U = mix(mix(t ^ K0) ^ K1 ^ mix(s ^ K2)) ^ K3    (one number per edge)
 *     where mix is a 32-bit mixing permutation (xorshift-multiply, two multiplies).
 *     The variate is U read as the fixed-point number R / 2^32.  One Philox call per
 *     (seed, group, layer, sampler) keeps the group seeds z_g independent; the
 *     per-vertex part is an Even-Mansour keyed permutation and costs a few integer
 *     instructions per examined neighbour, which is what lets the GPU count pass run
 *     at memory speed rather than at the speed of ten Philox rounds.
 *   - g = floor(iter/kappa) names the seed z_g; z1 = z_g, z2 = z_{g+1}.
 *     kappa == 0 means kappa = infinity (g = 0, c = 0 for ever).
 *   - n1, n2 are Phi^-1 of the two uniforms ((U + 1/2) / 2^32), so that c = 0
 *     gives back U exactly; that case is taken in integers.
 *   - LABOR-0 compares exactly: R * d_s <= k * 2^32 in 64-bit unsigned integers.
 *   - NS keeps the k smallest (R_ts, position) pairs.
 *   - edges are emitted in (seed order, adjacency order); S^{l+1} lists S^l
 *     first (same order) and then every new vertex in order of first appearance.
 *   - RW (the paper gives it no dependent variates): draw number c of destination s at
 *     layer l of iteration iter is U = mix(mix(c ^ K0) ^ K1 ^ mix(s ^ K2)) ^ K3 with the keys
 *     of (seed, sampler 2, layer, g = iter); step i of walk w picks neighbour
 *     floor(U_{2(w o + i)} d / 2^32) of its base vertex and, for i >= 1, restarts (base = s
 *     instead of the current vertex) iff U_{2(w o + i) + 1} < floor(p 2^32); a walk that
 *     reaches a vertex without neighbours ends; the walk's start s counts as visited only
 *     when a step lands on it; ties in the visit counts go to the smaller vertex id; the
 *     kept sources leave in that order (count descending, id ascending) and a block's eid
 *     holds the visit count (these edges are edges of sum_i A^i, not of the graph).
 *   - Phi and Phi^-1 are *defined* as fixed sequences of IEEE binary64
 *     add / mul / fma and bit operations (no libm, no division, no sqrt), so
 *     that any IEEE machine reproduces them bit for bit.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (published Philox known-answer vectors, brute force in pure Python on tiny
 * graphs, closed-form expectations, BFS balls, scipy ndtr/ndtri, textbook LRU).
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared coopref.c -o libcoopref.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define COOPREF_NS 0
#define COOPREF_LABOR0 1
#define COOPREF_RW 2

#define COOPREF_OK 0
#define COOPREF_E_NULL (-1)
#define COOPREF_E_RANGE (-2)
#define COOPREF_E_DUPSEED (-3)
#define COOPREF_E_ARG (-4)
#define COOPREF_E_NOMEM (-5)

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as    */
/* easy as 1, 2, 3", SC'11, Sec. 3.3 / Table 2 constants).                     */
/* ------------------------------------------------------------------------- */
void coopref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; /* golden-ratio Weyl step */
    k1 += 0xBB67AE85u; /* sqrt(3)-1 Weyl step */
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------- */
/* Reproducible binary64 kit: only +, *, fma and bit moves.                    */
/* ------------------------------------------------------------------------- */
static inline uint64_t d2u(double x) { uint64_t u; memcpy(&u, &x, 8); return u; }
static inline double u2d(uint64_t u) { double x; memcpy(&x, &u, 8); return x; }

/* 1/x for positive normal x: bit-trick first guess (relative error < 0.13),
 * then six Newton steps y <- y + y(1 - xy); each squares the error. */
double coopref_rcp(double x) {
  double y = u2d(0x7FDE623822FC16E6ull - d2u(x));
  for (int i = 0; i < 6; ++i) {
    double e = fma(-x, y, 1.0);
    y = fma(y, e, y);
  }
  return y;
}

/* 1/sqrt(x) for positive normal x: bit-trick first guess (relative error
 * < 0.035), then five Newton steps y <- y (3/2 - x y^2 / 2). */
double coopref_rsqrt(double x) {
  double y = u2d(0x5FE6EB50C7B537A9ull - (d2u(x) >> 1));
  for (int i = 0; i < 5; ++i) {
    double t = x * y;
    t = t * y;
    y = y * fma(-0.5, t, 1.5);
  }
  return y;
}

/* natural log of a positive normal x: x = m 2^e with m in [1/sqrt2, sqrt2),
 * log m = 2 atanh(z), z = (m-1)/(m+1), odd series to z^17. */
double coopref_log(double x) {
  uint64_t b = d2u(x);
  int64_t e = (int64_t)(b >> 52) - 1023;
  double m = u2d((b & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull);
  if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
  double z = (m - 1.0) * coopref_rcp(m + 1.0);
  double z2 = z * z;
  double p = 1.0 / 17.0;
  p = fma(p, z2, 1.0 / 15.0);
  p = fma(p, z2, 1.0 / 13.0);
  p = fma(p, z2, 1.0 / 11.0);
  p = fma(p, z2, 1.0 / 9.0);
  p = fma(p, z2, 1.0 / 7.0);
  p = fma(p, z2, 1.0 / 5.0);
  p = fma(p, z2, 1.0 / 3.0);
  p = fma(p, z2, 1.0);
  double lm = (2.0 * z) * p;
  return fma((double)e, 0.6931471805599453, lm);
}

/* exp(y) for y in [-700, 0]: y = k ln2 + r, |r| <= ln2/2, Taylor to r^13. */
double coopref_exp(double y) {
  const double magic = 6755399441055744.0; /* 1.5 * 2^52: add/subtract rounds to an integer */
  double kf = fma(y, 1.4426950408889634, magic) - magic;
  double r = fma(-kf, 0.6931471803691238, y);      /* ln2 high part (low 21 bits zero) */
  r = fma(-kf, 1.9082149292705877e-10, r);         /* ln2 low part */
  double p = 1.0 / 6227020800.0;                   /* 1/13! */
  p = fma(p, r, 1.0 / 479001600.0);
  p = fma(p, r, 1.0 / 39916800.0);
  p = fma(p, r, 1.0 / 3628800.0);
  p = fma(p, r, 1.0 / 362880.0);
  p = fma(p, r, 1.0 / 40320.0);
  p = fma(p, r, 1.0 / 5040.0);
  p = fma(p, r, 1.0 / 720.0);
  p = fma(p, r, 1.0 / 120.0);
  p = fma(p, r, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  int64_t k = (int64_t)kf;
  return p * u2d((uint64_t)(k + 1023) << 52);
}

/* Phi^-1 of u = (U + 1/2) / 2^32 (App. A.7 needs n ~ N(0,1) from a uniform).
 * P. J. Acklam's rational approximation (relative error 1.15e-9): a central
 * branch in q = p - 1/2 and a tail branch in sqrt(-2 log p); the upper half
 * is the mirror image of the lower half, taken on the integer U. */
double coopref_phi_inv_u32(uint32_t U) {
  int upper = U >= 0x80000000u;
  uint32_t Ul = upper ? (0xFFFFFFFFu - U) : U;
  double p = ((double)Ul + 0.5) * (1.0 / 4294967296.0); /* exact, in (0, 1/2) */
  double x;
  if (p < 0.02425) {
    double w = -2.0 * coopref_log(p);
    double q = w * coopref_rsqrt(w);
    double num = -7.784894002430293e-03;
    num = fma(num, q, -3.223964580411365e-01);
    num = fma(num, q, -2.400758277161838e+00);
    num = fma(num, q, -2.549732539343734e+00);
    num = fma(num, q, 4.374664141464968e+00);
    num = fma(num, q, 2.938163982698783e+00);
    double den = 7.784695709041462e-03;
    den = fma(den, q, 3.224671290700398e-01);
    den = fma(den, q, 2.445134137142996e+00);
    den = fma(den, q, 3.754408661907416e+00);
    den = fma(den, q, 1.0);
    x = num * coopref_rcp(den);
  } else {
    double q = p - 0.5;
    double r = q * q;
    double num = -3.969683028665376e+01;
    num = fma(num, r, 2.209460984245205e+02);
    num = fma(num, r, -2.759285104469687e+02);
    num = fma(num, r, 1.383577518672690e+02);
    num = fma(num, r, -3.066479806614716e+01);
    num = fma(num, r, 2.506628277459239e+00);
    double den = -5.447609879822406e+01;
    den = fma(den, r, 1.615858368580409e+02);
    den = fma(den, r, -1.556989798598866e+02);
    den = fma(den, r, 6.680131188771972e+01);
    den = fma(den, r, -1.328068155288572e+01);
    den = fma(den, r, 1.0);
    x = (q * num) * coopref_rcp(den);
  }
  return upper ? -x : x;
}

/* Upper tail Q(a) = 1 - Phi(a), a >= 0.
 *   a < 3 : Phi(a) = 1/2 + phi(a) (a + a^3/3 + a^5/(3*5) + ...), 28 terms;
 *   else  : Laplace continued fraction Q = phi(a) / (a + 1/(a + 2/(a + ...)))
 *           cut at depth 24 and evaluated bottom-up as a ratio p/q.
 * Both are within 1e-10 (relative) of the true tail on their range. */
static const double inv_odd[29] = {
  1.0,        1.0 / 3.0,  1.0 / 5.0,  1.0 / 7.0,  1.0 / 9.0,  1.0 / 11.0, 1.0 / 13.0, 1.0 / 15.0,
  1.0 / 17.0, 1.0 / 19.0, 1.0 / 21.0, 1.0 / 23.0, 1.0 / 25.0, 1.0 / 27.0, 1.0 / 29.0, 1.0 / 31.0,
  1.0 / 33.0, 1.0 / 35.0, 1.0 / 37.0, 1.0 / 39.0, 1.0 / 41.0, 1.0 / 43.0, 1.0 / 45.0, 1.0 / 47.0,
  1.0 / 49.0, 1.0 / 51.0, 1.0 / 53.0, 1.0 / 55.0, 1.0 / 57.0};

double coopref_qtail(double a) {
  double a2 = a * a;
  double pdf = coopref_exp(-0.5 * a2) * 0.3989422804014327; /* 1/sqrt(2 pi) */
  if (a < 3.0) {
    double s = 1.0;
    for (int n = 28; n >= 1; --n) {
      /* s <- 1 + a^2/(2n+1) * s */
      s = fma(a2 * inv_odd[n], s, 1.0);
    }
    return fma(-(pdf * a), s, 0.5);
  } else {
    double p = 0.0, q = 1.0;
    for (int n = 24; n >= 1; --n) {
      double pn = (double)n * q;
      q = fma(a, q, p);
      p = pn;
    }
    double den = fma(a, q, p);
    return (pdf * q) * coopref_rcp(den);
  }
}

/* R = floor(Phi(x) * 2^32) clamped to [0, 2^32-1]; the upper half mirrors the
 * lower half in integers so that Phi(x) + Phi(-x) = 1 holds on the grid. */
uint32_t coopref_phi_to_u32(double x) {
  int neg = x < 0.0;
  double a = neg ? -x : x;
  double Q = coopref_qtail(a);
  double s = Q * 4294967296.0;
  uint64_t f = (uint64_t)s; /* s in [0, 2^31]: truncation == floor */
  if (f > 0xFFFFFFFFull) f = 0xFFFFFFFFull;
  uint32_t lo = (uint32_t)f;
  return neg ? lo : (0xFFFFFFFFu - lo);
}

/* ------------------------------------------------------------------------- */
/* Variates of App. A.7.                                                       */
/* ------------------------------------------------------------------------- */
/* 32-bit mixing permutation: xor-shift / odd-multiply rounds (each invertible). */
uint32_t coopref_mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

/* The four key words of (seed, sampler, layer, group g). */
void coopref_layer_keys(uint64_t seed, int sampler, int layer, uint64_t g, uint32_t K[4]) {
  uint32_t ctr[4] = {(uint32_t)g, (uint32_t)(g >> 32), (uint32_t)layer | ((uint32_t)sampler << 8), 0x434F4F50u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  coopref_philox4x32_10(ctr, key, K);
}

static uint32_t keyed_uniform(const uint32_t K[4], int sampler, uint32_t t, uint32_t s) {
  uint32_t a = coopref_mix32(t ^ K[0]) ^ K[1];
  if (sampler == COOPREF_LABOR0) return a;
  return coopref_mix32(a ^ coopref_mix32(s ^ K[2])) ^ K[3];
}

typedef struct {
  uint64_t seed;
  uint64_t g;      /* group index floor(iter/kappa) */
  int blend;       /* 0: c == 0, integer path */
  double cw, sw;   /* cos(c pi/2), sin(c pi/2) */
  /* per (sampler, layer), filled by variate_layer(): keys of group g and of group g+1 */
  int sampler;
  uint32_t K1[4], K2[4];
} variate_state;

static void variate_setup(variate_state* st, uint64_t seed, uint64_t iter, uint32_t kappa) {
  st->seed = seed;
  if (kappa == 0) { st->g = 0; st->blend = 0; st->cw = 1.0; st->sw = 0.0; return; }
  uint64_t i = iter % kappa;
  st->g = iter / kappa;
  st->blend = i != 0;
  double c = (double)i / (double)kappa;
  st->cw = cos(c * 1.5707963267948966);
  st->sw = sin(c * 1.5707963267948966);
}

static void variate_layer(variate_state* st, int sampler, int layer) {
  st->sampler = sampler;
  coopref_layer_keys(st->seed, sampler, layer, st->g, st->K1);
  coopref_layer_keys(st->seed, sampler, layer, st->g + 1, st->K2);
}

static uint32_t variate_draw(const variate_state* st, uint32_t t, uint32_t s) {
  uint32_t U1 = keyed_uniform(st->K1, st->sampler, t, s);
  if (!st->blend) return U1;
  uint32_t U2 = keyed_uniform(st->K2, st->sampler, t, s);
  double n1 = coopref_phi_inv_u32(U1);
  double n2 = coopref_phi_inv_u32(U2);
  double n = fma(st->cw, n1, st->sw * n2);
  return coopref_phi_to_u32(n);
}

/* R for one (t, s): what the samplers below call, exported for the tests. */
uint32_t coopref_variate(uint64_t seed, int sampler, int layer, uint64_t iter, uint32_t kappa,
                         uint32_t t, uint32_t s) {
  variate_state st;
  variate_setup(&st, seed, iter, kappa);
  variate_layer(&st, sampler, layer);
  return variate_draw(&st, t, s);
}

/* ------------------------------------------------------------------------- */
/* One sampling layer + dedup/relabel; L layers; gather.                       */
/* ------------------------------------------------------------------------- */
typedef struct {
  int64_t n_dst, n_src, n_edges;
  int32_t* dst_ids;    /* [n_dst]    S^l                                        */
  int64_t* indptr;     /* [n_dst+1]  edges of dst i are [indptr[i], indptr[i+1]) */
  int32_t* col_local;  /* [n_edges]  index of the source vertex in src_ids      */
  int32_t* col_global; /* [n_edges]  global id of the source vertex             */
  int64_t* eid;        /* [n_edges]  position of the edge in the graph's indices */
  int32_t* src_ids;    /* [n_src]    S^{l+1}; src_ids[0:n_dst] == dst_ids       */
} coopref_block;

typedef struct { uint32_t r; int64_t j; } ns_pair;

static int ns_pair_cmp(const void* a, const void* b) {
  const ns_pair* x = (const ns_pair*)a; const ns_pair* y = (const ns_pair*)b;
  if (x->r != y->r) return x->r < y->r ? -1 : 1;
  if (x->j != y->j) return x->j < y->j ? -1 : 1;
  return 0;
}
static int i64_cmp(const void* a, const void* b) {
  int64_t x = *(const int64_t*)a, y = *(const int64_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

void coopref_free_blocks(coopref_block* blocks, int L) {
  if (!blocks) return;
  for (int l = 0; l < L; ++l) {
    free(blocks[l].dst_ids); free(blocks[l].indptr); free(blocks[l].col_local);
    free(blocks[l].col_global); free(blocks[l].eid); free(blocks[l].src_ids);
    memset(&blocks[l], 0, sizeof(coopref_block));
  }
}

/* S^{l+1}: S^l in order, then new sources by first appearance (Eq. 2); col_local. */
static int finish_block(const int32_t* dst, int64_t n_dst, coopref_block* blk, int32_t* pos_of /* all -1 */) {
  const int64_t m = blk->n_edges;
  blk->src_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_dst + m > 0 ? n_dst + m : 1));
  blk->col_local = (int32_t*)malloc(sizeof(int32_t) * (size_t)(m > 0 ? m : 1));
  if (!blk->src_ids || !blk->col_local) return COOPREF_E_NOMEM;
  int64_t n_src = 0;
  for (int64_t i = 0; i < n_dst; ++i) { pos_of[dst[i]] = (int32_t)n_src; blk->src_ids[n_src++] = dst[i]; }
  for (int64_t e = 0; e < m; ++e) {
    int32_t t = blk->col_global[e];
    if (pos_of[t] < 0) { pos_of[t] = (int32_t)n_src; blk->src_ids[n_src++] = t; }
    blk->col_local[e] = pos_of[t];
  }
  blk->n_src = n_src;
  for (int64_t i = 0; i < n_src; ++i) pos_of[blk->src_ids[i]] = -1; /* leave pos_of all -1 */
  return COOPREF_OK;
}

/* Samples the neighbourhoods of dst[0..n_dst) with fanout k and fills one block. */
static int sample_layer(const int64_t* g_indptr, const int32_t* g_indices, int64_t n_vertices,
                        const int32_t* dst, int64_t n_dst, int32_t k, int sampler, int layer,
                        variate_state* st, int32_t* pos_of /* [n_vertices], all -1 */,
                        coopref_block* blk) {
  /* upper bound on kept edges: every neighbour examined */
  int64_t D = 0, dmax = 0;
  for (int64_t i = 0; i < n_dst; ++i) {
    int64_t d = g_indptr[dst[i] + 1] - g_indptr[dst[i]];
    D += d; if (d > dmax) dmax = d;
  }
  int64_t cap = D > 0 ? D : 1;
  blk->n_dst = n_dst;
  blk->dst_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_dst > 0 ? n_dst : 1));
  blk->indptr = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_dst + 1));
  blk->col_global = (int32_t*)malloc(sizeof(int32_t) * (size_t)cap);
  blk->eid = (int64_t*)malloc(sizeof(int64_t) * (size_t)cap);
  ns_pair* pairs = (ns_pair*)malloc(sizeof(ns_pair) * (size_t)(dmax > 0 ? dmax : 1));
  int64_t* chosen = (int64_t*)malloc(sizeof(int64_t) * (size_t)(k > 0 ? k : 1));
  if (!blk->dst_ids || !blk->indptr || !blk->col_global || !blk->eid || !pairs || !chosen) {
    free(pairs); free(chosen); return COOPREF_E_NOMEM;
  }
  memcpy(blk->dst_ids, dst, sizeof(int32_t) * (size_t)n_dst);
  variate_layer(st, sampler, layer);

  int64_t m = 0;
  for (int64_t i = 0; i < n_dst; ++i) {
    uint32_t s = (uint32_t)dst[i];
    int64_t beg = g_indptr[s], d = g_indptr[s + 1] - beg;
    blk->indptr[i] = m;
    if (sampler == COOPREF_LABOR0) {
      /* r_t <= k/d_s  <=>  R d_s <= k 2^32 (exact in uint64) */
      for (int64_t j = 0; j < d; ++j) {
        uint32_t t = (uint32_t)g_indices[beg + j];
        uint64_t R = variate_draw(st, t, s);
        if (R * (uint64_t)d <= ((uint64_t)k << 32)) {
          blk->col_global[m] = (int32_t)t; blk->eid[m] = beg + j; ++m;
        }
      }
    } else { /* NS */
      if (d <= k) {
        for (int64_t j = 0; j < d; ++j) {
          blk->col_global[m] = g_indices[beg + j]; blk->eid[m] = beg + j; ++m;
        }
      } else {
        for (int64_t j = 0; j < d; ++j) {
          pairs[j].r = variate_draw(st, (uint32_t)g_indices[beg + j], s);
          pairs[j].j = j;
        }
        qsort(pairs, (size_t)d, sizeof(ns_pair), ns_pair_cmp);
        for (int32_t q = 0; q < k; ++q) chosen[q] = pairs[q].j;
        qsort(chosen, (size_t)k, sizeof(int64_t), i64_cmp);
        for (int32_t q = 0; q < k; ++q) {
          blk->col_global[m] = g_indices[beg + chosen[q]]; blk->eid[m] = beg + chosen[q]; ++m;
        }
      }
    }
  }
  blk->indptr[n_dst] = m;
  blk->n_edges = m;
  free(pairs); free(chosen);
  (void)n_vertices;
  return finish_block(dst, n_dst, blk, pos_of);
}

int coopref_sample(const int64_t* g_indptr, const int32_t* g_indices, int64_t n_vertices,
                   int64_t n_edges, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts,
                   int L, int sampler, uint64_t iter, uint32_t kappa, uint64_t seed,
                   coopref_block* blocks_out) {
  if (!g_indptr || (!g_indices && n_edges > 0) || (!seeds && n_seeds > 0) || !fanouts || !blocks_out)
    return COOPREF_E_NULL;
  if (L < 1 || L > 255 || n_seeds < 0 || n_vertices < 0) return COOPREF_E_ARG;
  if (sampler != COOPREF_NS && sampler != COOPREF_LABOR0) return COOPREF_E_ARG;
  for (int l = 0; l < L; ++l) if (fanouts[l] < 1) return COOPREF_E_ARG;
  memset(blocks_out, 0, sizeof(coopref_block) * (size_t)L);

  int32_t* pos_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_vertices > 0 ? n_vertices : 1));
  if (!pos_of) return COOPREF_E_NOMEM;
  for (int64_t v = 0; v < n_vertices; ++v) pos_of[v] = -1;
  /* seeds: in range and pairwise distinct (the paper draws them without replacement) */
  for (int64_t i = 0; i < n_seeds; ++i) {
    if (seeds[i] < 0 || seeds[i] >= n_vertices) { free(pos_of); return COOPREF_E_RANGE; }
    if (pos_of[seeds[i]] >= 0) { free(pos_of); return COOPREF_E_DUPSEED; }
    pos_of[seeds[i]] = 1;
  }
  for (int64_t i = 0; i < n_seeds; ++i) pos_of[seeds[i]] = -1;

  variate_state st;
  variate_setup(&st, seed, iter, kappa);
  const int32_t* dst = seeds; int64_t n_dst = n_seeds;
  for (int l = 0; l < L; ++l) {
    int rc = sample_layer(g_indptr, g_indices, n_vertices, dst, n_dst, fanouts[l], sampler, l, &st,
                          pos_of, &blocks_out[l]);
    if (rc != COOPREF_OK) { coopref_free_blocks(blocks_out, L); free(pos_of); return rc; }
    dst = blocks_out[l].src_ids; n_dst = blocks_out[l].n_src;
  }
  free(pos_of);
  return COOPREF_OK;
}

/* ------------------------------------------------------------------------- */
/* Random-walk sampling (App. A.1.3).                                          */
/* ------------------------------------------------------------------------- */
typedef struct { int32_t v; int64_t count; } rw_visit;

static int i32_cmp(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}
static int rw_visit_cmp(const void* a, const void* b) { /* count descending, then id ascending */
  const rw_visit* x = (const rw_visit*)a; const rw_visit* y = (const rw_visit*)b;
  if (x->count != y->count) return x->count > y->count ? -1 : 1;
  return x->v < y->v ? -1 : (x->v > y->v ? 1 : 0);
}

/* draw number c of destination s */
static uint32_t rw_draw(const uint32_t K[4], uint32_t c, uint32_t s) {
  return coopref_mix32(coopref_mix32(c ^ K[0]) ^ K[1] ^ coopref_mix32(s ^ K[2])) ^ K[3];
}
uint32_t coopref_rw_draw(uint64_t seed, int layer, uint64_t iter, uint32_t s, uint32_t c) {
  uint32_t K[4];
  coopref_layer_keys(seed, COOPREF_RW, layer, iter, K);
  return rw_draw(K, c, s);
}
static uint64_t rw_restart_threshold(double p) { /* restart iff U < floor(p 2^32) */
  if (p >= 1.0) return (uint64_t)1 << 32;
  if (!(p > 0.0)) return 0;
  return (uint64_t)(p * 4294967296.0);
}

int coopref_sample_rw(const int64_t* g_indptr, const int32_t* g_indices, int64_t n_vertices,
                      int64_t n_edges, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts,
                      int L, int32_t walk_length, int32_t n_walks, double restart_p, uint64_t iter,
                      uint64_t seed, coopref_block* blocks_out) {
  if (!g_indptr || (!g_indices && n_edges > 0) || (!seeds && n_seeds > 0) || !fanouts || !blocks_out)
    return COOPREF_E_NULL;
  if (L < 1 || L > 255 || n_seeds < 0 || n_vertices < 0) return COOPREF_E_ARG;
  if (walk_length < 1 || n_walks < 1 || (int64_t)walk_length * n_walks > ((int64_t)1 << 20)) return COOPREF_E_ARG;
  if (!(restart_p >= 0.0 && restart_p <= 1.0)) return COOPREF_E_ARG;
  for (int l = 0; l < L; ++l) if (fanouts[l] < 1) return COOPREF_E_ARG;
  memset(blocks_out, 0, sizeof(coopref_block) * (size_t)L);

  int32_t* pos_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_vertices > 0 ? n_vertices : 1));
  const int64_t n_steps = (int64_t)walk_length * n_walks;
  int32_t* visited = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_steps);
  rw_visit* tally = (rw_visit*)malloc(sizeof(rw_visit) * (size_t)n_steps);
  if (!pos_of || !visited || !tally) { free(pos_of); free(visited); free(tally); return COOPREF_E_NOMEM; }
  for (int64_t v = 0; v < n_vertices; ++v) pos_of[v] = -1;
  for (int64_t i = 0; i < n_seeds; ++i) {
    if (seeds[i] < 0 || seeds[i] >= n_vertices) { free(pos_of); free(visited); free(tally); return COOPREF_E_RANGE; }
    if (pos_of[seeds[i]] >= 0) { free(pos_of); free(visited); free(tally); return COOPREF_E_DUPSEED; }
    pos_of[seeds[i]] = 1;
  }
  for (int64_t i = 0; i < n_seeds; ++i) pos_of[seeds[i]] = -1;

  const uint64_t P = rw_restart_threshold(restart_p);
  const int32_t* dst = seeds; int64_t n_dst = n_seeds;
  int rc = COOPREF_OK;
  for (int l = 0; l < L && rc == COOPREF_OK; ++l) {
    coopref_block* blk = &blocks_out[l];
    const int32_t k = fanouts[l];
    uint32_t K[4];
    coopref_layer_keys(seed, COOPREF_RW, l, iter, K);
    const int64_t cap = n_dst * (int64_t)(k < n_steps ? k : n_steps);
    blk->n_dst = n_dst;
    blk->dst_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_dst > 0 ? n_dst : 1));
    blk->indptr = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_dst + 1));
    blk->col_global = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap > 0 ? cap : 1));
    blk->eid = (int64_t*)malloc(sizeof(int64_t) * (size_t)(cap > 0 ? cap : 1));
    if (!blk->dst_ids || !blk->indptr || !blk->col_global || !blk->eid) { rc = COOPREF_E_NOMEM; break; }
    memcpy(blk->dst_ids, dst, sizeof(int32_t) * (size_t)n_dst);
    int64_t m = 0;
    for (int64_t i = 0; i < n_dst; ++i) {
      const uint32_t s = (uint32_t)dst[i];
      const int64_t s_beg = g_indptr[s], s_d = g_indptr[s + 1] - s_beg;
      blk->indptr[i] = m;
      if (s_d == 0) continue;
      int64_t n_vis = 0;
      for (int32_t w = 0; w < n_walks; ++w) {
        uint32_t cur = s;
        for (int32_t step = 0; step < walk_length; ++step) {
          const uint32_t c = 2u * (uint32_t)(w * walk_length + step);
          int restart = step == 0 || (uint64_t)rw_draw(K, c + 1u, s) < P; /* the first step leaves from s */
          const uint32_t base = restart ? s : cur;
          const int64_t beg = g_indptr[base], d = g_indptr[base + 1] - beg;
          if (d == 0) break; /* dead end: the walk ends */
          const uint64_t pick = ((uint64_t)rw_draw(K, c, s) * (uint64_t)d) >> 32;
          cur = (uint32_t)g_indices[beg + (int64_t)pick];
          visited[n_vis++] = (int32_t)cur;
        }
      }
      /* tally: sort the visits by id, run lengths are the counts */
      qsort(visited, (size_t)n_vis, sizeof(int32_t), i32_cmp);
      int64_t n_t = 0;
      for (int64_t q = 0; q < n_vis; ++q) {
        if (n_t > 0 && tally[n_t - 1].v == visited[q]) tally[n_t - 1].count += 1;
        else { tally[n_t].v = visited[q]; tally[n_t].count = 1; ++n_t; }
      }
      qsort(tally, (size_t)n_t, sizeof(rw_visit), rw_visit_cmp);
      for (int64_t q = 0; q < n_t && q < k; ++q) {
        blk->col_global[m] = tally[q].v; blk->eid[m] = tally[q].count; ++m;
      }
    }
    blk->indptr[n_dst] = m;
    blk->n_edges = m;
    rc = finish_block(dst, n_dst, blk, pos_of);
    dst = blk->src_ids; n_dst = blk->n_src;
  }
  if (rc != COOPREF_OK) coopref_free_blocks(blocks_out, L);
  free(pos_of); free(visited); free(tally);
  return rc;
}

/* Feature loading of Algorithm 1: out[i,:] = feat[ids[i],:], rows are opaque bytes. */
int coopref_gather(const void* feat, int64_t n_rows, int64_t row_bytes, const int32_t* ids,
                   int64_t n_ids, void* out) {
  if (!feat || (!ids && n_ids > 0) || (!out && n_ids > 0)) return COOPREF_E_NULL;
  if (row_bytes <= 0 || n_ids < 0) return COOPREF_E_ARG;
  for (int64_t i = 0; i < n_ids; ++i) {
    if (ids[i] < 0 || ids[i] >= n_rows) return COOPREF_E_RANGE;
    memcpy((char*)out + i * row_bytes, (const char*)feat + (int64_t)ids[i] * row_bytes, (size_t)row_bytes);
  }
  return COOPREF_OK;
}

/* Sec. 3.1 / Algorithm 1: the vertices of a frontier grouped by the PE that owns them, in their original order within
 * each group.  scheme 0: PE p owns a contiguous range, owner(v) = floor(v P / |V|); scheme 1: a random partition,
 * owner(v) = floor(mix32(v ^ key) P / 2^32) with key = the low word of seed xor its high word.  ids_out and origin_out
 * (the position that each entry had in ids) get n entries, offsets_out P + 1: group p is [offsets[p], offsets[p+1]). */
int coopref_bucket_by_owner(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, uint64_t seed,
                            int32_t* ids_out, int32_t* origin_out, int64_t* offsets_out) {
  if ((!ids && n > 0) || !offsets_out) return COOPREF_E_NULL;
  if (n < 0 || n_vertices < 1 || n_parts < 1 || (scheme != 0 && scheme != 1)) return COOPREF_E_ARG;
  const uint32_t key = (uint32_t)(seed ^ (seed >> 32));
  int64_t at = 0;
  for (int p = 0; p < n_parts; ++p) {       /* one sweep over the list per PE: group p is what the sweep finds */
    offsets_out[p] = at;
    for (int64_t i = 0; i < n; ++i) {
      if (ids[i] < 0 || ids[i] >= n_vertices) return COOPREF_E_RANGE;
      const uint64_t v = (uint64_t)ids[i];
      const uint64_t owner = scheme == 0 ? (v * (uint64_t)n_parts) / (uint64_t)n_vertices
                                         : ((uint64_t)coopref_mix32((uint32_t)v ^ key) * (uint64_t)n_parts) >> 32;
      if (owner == (uint64_t)p) {
        ids_out[at] = ids[i];
        origin_out[at] = (int32_t)i;
        ++at;
      }
    }
  }
  offsets_out[n_parts] = at;
  return COOPREF_OK;
}

/* IEEE binary16 -> double, from the bit fields (no compiler half type needed). */
static double half_to_double(uint16_t h) {
  int sign = h >> 15, ex = (h >> 10) & 31, man = h & 1023;
  double v;
  if (ex == 0) v = ldexp((double)man, -24);                    /* subnormal or zero */
  else if (ex == 31) v = man ? NAN : INFINITY;
  else v = ldexp((double)(man | 1024), ex - 25);
  return sign ? -v : v;
}

/* Neighbour mean of Eq. (1) with a mean aggregator over one sampled block:
 * out[i, c] = (1/deg_i) sum_{e in [indptr[i], indptr[i+1])} feat[col[e], c] in binary64 (0 when deg_i = 0).
 * dtype: 0 = float rows, 1 = binary16 rows. */
int coopref_gather_mean(const void* feat, int64_t n_rows, int32_t dim, int dtype, const int64_t* indptr,
                        const int32_t* col, int64_t n_dst, double* out) {
  if (!feat || !indptr || (!out && n_dst > 0)) return COOPREF_E_NULL;
  if (dim < 1 || (dtype != 0 && dtype != 1) || n_dst < 0) return COOPREF_E_ARG;
  for (int64_t i = 0; i < n_dst; ++i) {
    int64_t beg = indptr[i], end = indptr[i + 1];
    for (int32_t c = 0; c < dim; ++c) {
      double acc = 0.0;
      for (int64_t e = beg; e < end; ++e) {
        int64_t t = col[e];
        if (t < 0 || t >= n_rows) return COOPREF_E_RANGE;
        acc += dtype == 0 ? (double)((const float*)feat)[t * dim + c]
                          : half_to_double(((const uint16_t*)feat)[t * dim + c]);
      }
      out[i * dim + c] = end > beg ? acc / (double)(end - beg) : 0.0;
    }
  }
  return COOPREF_OK;
}

/* ------------------------------------------------------------------------- */
/* LRU vertex cache (Sec. 4.2 names "an LRU cache" and nothing more).          */
/* Reading: a textbook LRU (recency list + membership map, one access at a     */
/* time) fed, per batch A of distinct ids, first the ids of A that are cached  */
/* when the batch starts (in A order), then the ids that are not (in A order). */
/* Serving hits first means a batch never evicts a row it is about to read.    */
/* ------------------------------------------------------------------------- */
typedef struct {
  int64_t capacity, n_vertices, size;
  int32_t head, tail;    /* least / most recently used vertex, -1 when empty */
  int32_t* prev;         /* [n_vertices] towards the LRU end; -2 = not cached */
  int32_t* next;         /* [n_vertices] towards the MRU end */
} coopref_cache;

coopref_cache* coopref_cache_create(int64_t capacity, int64_t n_vertices) {
  coopref_cache* c = (coopref_cache*)calloc(1, sizeof(coopref_cache));
  if (!c) return NULL;
  c->capacity = capacity; c->n_vertices = n_vertices; c->size = 0; c->head = c->tail = -1;
  size_t n = (size_t)(n_vertices > 0 ? n_vertices : 1);
  c->prev = (int32_t*)malloc(sizeof(int32_t) * n);
  c->next = (int32_t*)malloc(sizeof(int32_t) * n);
  if (!c->prev || !c->next) { free(c->prev); free(c->next); free(c); return NULL; }
  for (int64_t v = 0; v < n_vertices; ++v) { c->prev[v] = -2; c->next[v] = -2; }
  return c;
}
void coopref_cache_free(coopref_cache* c) { if (c) { free(c->prev); free(c->next); free(c); } }
int64_t coopref_cache_size(const coopref_cache* c) { return c->size; }
int coopref_cache_contains(const coopref_cache* c, int32_t v) { return c->prev[v] != -2; }

static void lru_unlink(coopref_cache* c, int32_t v) {
  int32_t p = c->prev[v], n = c->next[v];
  if (p >= 0) c->next[p] = n; else c->head = n;
  if (n >= 0) c->prev[n] = p; else c->tail = p;
  c->prev[v] = -2; c->next[v] = -2; c->size--;
}
static void lru_push_mru(coopref_cache* c, int32_t v) {
  c->prev[v] = c->tail; c->next[v] = -1;
  if (c->tail >= 0) c->next[c->tail] = v; else c->head = v;
  c->tail = v; c->size++;
}
/* one textbook access; returns 1 on a hit */
static int lru_access(coopref_cache* c, int32_t v) {
  if (c->prev[v] != -2) { lru_unlink(c, v); lru_push_mru(c, v); return 1; }
  if (c->capacity == 0) return 0;
  if (c->size >= c->capacity) lru_unlink(c, c->head);
  lru_push_mru(c, v);
  return 0;
}

/* Processes one batch of distinct ids; hit_out[i] = 1 if ids[i] was cached when the
 * batch started.  Returns the number of misses, or a negative error code. */
int64_t coopref_cache_access(coopref_cache* c, const int32_t* ids, int64_t n_ids, uint8_t* hit_out) {
  if (!c || (!ids && n_ids > 0)) return COOPREF_E_NULL;
  for (int64_t i = 0; i < n_ids; ++i)
    if (ids[i] < 0 || ids[i] >= c->n_vertices) return COOPREF_E_RANGE;
  uint8_t* hit = (uint8_t*)malloc((size_t)(n_ids > 0 ? n_ids : 1));
  if (!hit) return COOPREF_E_NOMEM;
  int64_t n_miss = 0;
  for (int64_t i = 0; i < n_ids; ++i) { hit[i] = c->prev[ids[i]] != -2; n_miss += !hit[i]; }
  for (int64_t i = 0; i < n_ids; ++i) if (hit[i]) lru_access(c, ids[i]);
  for (int64_t i = 0; i < n_ids; ++i) if (!hit[i]) lru_access(c, ids[i]);
  if (hit_out) memcpy(hit_out, hit, (size_t)n_ids);
  free(hit);
  return n_miss;
}
