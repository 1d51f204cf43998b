// Feature loading step of Algorithm 1: out[i, :] = feat[ids[i], :], an exact copy of bits.
//
// HBM-bound row gather.  A row of `vecs` vectors (16, 8, 4, 2 or 1 bytes each, the widest that the row size and
// the base addresses allow) is moved by `lpr` adjacent lanes (a power of two), so one wave64 load instruction
// covers 64 / lpr rows and each row is read with full-width, coalesced accesses.  Every thread keeps kUnroll rows
// in flight to cover the latency of the random row reads.  Loads and stores are non-temporal: a row is used once.
#include <hip/hip_fp16.h>

#include <mutex>

#include "coop_internal.h"
#include "device_utils.h"

namespace coop {

constexpr int kGatherUnroll = 4;

template <typename V>
__global__ __launch_bounds__(kBlock) void k_gather(const V* __restrict__ feat, int64_t n_rows, int32_t vecs, int lpr_log2,
                                                   const int32_t* __restrict__ ids, int64_t n_ids, V* __restrict__ out,
                                                   int32_t* __restrict__ bad) {
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kBlock >> lpr_log2;
  const int sub = threadIdx.x & (lpr - 1);
  const int64_t row0 = ((int64_t)blockIdx.x * kGatherUnroll) * rows_per_block + (threadIdx.x >> lpr_log2);

  int64_t src_row[kGatherUnroll];
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const int64_t r = row0 + (int64_t)u * rows_per_block;
    int64_t id = -1;
    if (r < n_ids) {
      id = ids[r];
      if ((uint64_t)id >= (uint64_t)n_rows) {
        if (sub == 0) atomicOr(bad, 1);
        id = -2;
      }
    }
    src_row[u] = id;
  }
  for (int32_t v = sub; v < vecs; v += lpr) {
    V x[kGatherUnroll];
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
      if (src_row[u] >= 0) x[u] = __builtin_nontemporal_load(feat + src_row[u] * vecs + v);
      else x[u] = V{};
    }
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
      const int64_t r = row0 + (int64_t)u * rows_per_block;
      if (src_row[u] != -1) __builtin_nontemporal_store(x[u], out + r * vecs + v);
    }
  }
}

// ---- neighbour mean fused with the feature load ------------------------------------------------------------------
// out[i, :] = mean over the sampled in-edges e of destination i of feat[col[e], :]  (Eq. 1 with a mean aggregator,
// the first thing a GCN / GraphSAGE layer does with the loaded rows), 0 for a destination without edges.  The rows
// are read straight from the feature table and never written out individually: the kernel moves m rows in and
// n_dst rows out.  Accumulation is fp32, one lane per column group, edges in adjacency order (deterministic).
constexpr int kMeanUnroll = 4;

template <typename V, bool F16>
struct MeanAcc {
  static constexpr int kN = F16 ? (int)(sizeof(V) / 2) : (int)(sizeof(V) / 4);
  float a[kN];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int i = 0; i < kN; ++i) a[i] = 0.f;
  }
  __device__ __forceinline__ void add(const V& x) {
    if constexpr (F16) {
      const __half* h = reinterpret_cast<const __half*>(&x);
#pragma unroll
      for (int i = 0; i < kN; ++i) a[i] += __half2float(h[i]);
    } else {
      const float* f = reinterpret_cast<const float*>(&x);
#pragma unroll
      for (int i = 0; i < kN; ++i) a[i] += f[i];
    }
  }
  __device__ __forceinline__ V mean(float count) const {
    V r;
    if constexpr (F16) {
      __half* h = reinterpret_cast<__half*>(&r);
#pragma unroll
      for (int i = 0; i < kN; ++i) h[i] = __float2half_rn(a[i] / count);
    } else {
      float* f = reinterpret_cast<float*>(&r);
#pragma unroll
      for (int i = 0; i < kN; ++i) f[i] = a[i] / count;
    }
    return r;
  }
};

template <typename V, bool F16>
__global__ __launch_bounds__(kBlock) void k_gather_mean(const V* __restrict__ feat, int64_t n_rows, int32_t vecs, int lpr_log2,
                                                        const int64_t* __restrict__ indptr, const int32_t* __restrict__ col,
                                                        int64_t n_dst, V* __restrict__ out, int32_t* __restrict__ bad) {
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kBlock >> lpr_log2;
  const int sub = threadIdx.x & (lpr - 1);
  const int64_t i = (int64_t)blockIdx.x * rows_per_block + (threadIdx.x >> lpr_log2);
  if (i >= n_dst) return;
  const int64_t beg = indptr[i], end = indptr[i + 1];
  for (int32_t v = sub; v < vecs; v += lpr) {
    MeanAcc<V, F16> acc;
    acc.clear();
    for (int64_t e = beg; e < end; e += kMeanUnroll) {
      V x[kMeanUnroll];
      bool ok[kMeanUnroll];
#pragma unroll
      for (int u = 0; u < kMeanUnroll; ++u) {
        ok[u] = false;
        if (e + u < end) {
          const int64_t id = col[e + u];
          ok[u] = (uint64_t)id < (uint64_t)n_rows;
          if (ok[u]) x[u] = feat[id * vecs + v];
          else if (sub == 0 && v == sub) atomicOr(bad, 1);
        }
      }
#pragma unroll
      for (int u = 0; u < kMeanUnroll; ++u)
        if (ok[u]) acc.add(x[u]);
    }
    const int64_t cnt = end - beg;
    __builtin_nontemporal_store(cnt > 0 ? acc.mean((float)cnt) : V{}, out + i * vecs + v);
  }
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_bad_mu;
// Sticky "an id was out of range" word.  A device variable of this library's code object (zero when the code object is
// loaded): every GPU has its own copy at its own address, which hipGetSymbolAddress gives for the current device.
// Nothing is allocated for it, so the entry points that promise not to allocate can report through it as well.
static __device__ int32_t g_bad_word;
int32_t* g_bad_flag[kMaxDevices] = {};  // per device: the address of that device's copy

}  // namespace

// the current device's flag word (its address is looked up on first use and kept for the life of the process)
int32_t* bad_flag() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lk(g_bad_mu);
  if (!g_bad_flag[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_bad_word)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_bad_flag[dev] = (int32_t*)p;
  }
  return g_bad_flag[dev];
}

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename V>
void launch_gather(const void* feat, int64_t n_rows, int64_t row_bytes, const int32_t* ids, int64_t n_ids, void* out,
                   int32_t* bad, hipStream_t s) {
  const int32_t vecs = (int32_t)(row_bytes / (int64_t)sizeof(V));
  int lpr_log2 = 0;
  while ((1 << lpr_log2) < vecs && lpr_log2 < 8) ++lpr_log2;
  const int rows_per_block = kBlock >> lpr_log2;
  const int64_t rows_per_launch_block = (int64_t)rows_per_block * kGatherUnroll;
  const unsigned grid = (unsigned)((n_ids + rows_per_launch_block - 1) / rows_per_launch_block);
  COOP_LAUNCH(K_GATHER, k_gather<V>, dim3(grid), dim3(kBlock), 0, s, (const V*)feat, n_rows, vecs, lpr_log2, ids, n_ids, (V*)out,
              bad);
}
}  // namespace

}  // namespace coop

using namespace coop;

extern "C" int coop_gather(const void* feat, int64_t n_rows, int32_t dim, int dtype, const int32_t* ids, int64_t n_ids, void* out,
                           void* stream) {
  if (dtype != COOP_F32 && dtype != COOP_F16) return COOP_E_ARG;
  if (dim < 1 || n_rows < 0 || n_ids < 0) return COOP_E_ARG;
  if (n_ids == 0) return COOP_OK;
  if (!feat || !ids || !out) return COOP_E_NULL;
  const int64_t row_bytes = (int64_t)dim * (dtype == COOP_F32 ? 4 : 2);
  if ((n_ids + 255) / 256 > 0x7FFFFFFF) return COOP_E_ARG;
  int32_t* bad = bad_flag();
  if (!bad) return COOP_E_HIP;
  hipStream_t s = (hipStream_t)stream;
  const uintptr_t align = (uintptr_t)feat | (uintptr_t)out | (uintptr_t)row_bytes;
  if (align % 16 == 0) launch_gather<u32x4>(feat, n_rows, row_bytes, ids, n_ids, out, bad, s);
  else if (align % 8 == 0) launch_gather<u32x2>(feat, n_rows, row_bytes, ids, n_ids, out, bad, s);
  else if (align % 4 == 0) launch_gather<uint32_t>(feat, n_rows, row_bytes, ids, n_ids, out, bad, s);
  else if (align % 2 == 0) launch_gather<uint16_t>(feat, n_rows, row_bytes, ids, n_ids, out, bad, s);
  else return COOP_E_ARG;  // fp16 / fp32 tables are at least 2-byte aligned
  if (hipGetLastError() != hipSuccess) return COOP_E_HIP;
  return COOP_OK;
}

namespace {
template <typename V, bool F16>
void launch_mean(const void* feat, int64_t n_rows, int64_t row_bytes, const int64_t* indptr, const int32_t* col, int64_t n_dst,
                 void* out, int32_t* bad, hipStream_t s) {
  const int32_t vecs = (int32_t)(row_bytes / (int64_t)sizeof(V));
  int lpr_log2 = 0;
  while ((1 << lpr_log2) < vecs && lpr_log2 < 8) ++lpr_log2;
  const int rows_per_block = kBlock >> lpr_log2;
  const unsigned grid = (unsigned)((n_dst + rows_per_block - 1) / rows_per_block);
  COOP_LAUNCH(K_GATHER_MEAN, (k_gather_mean<V, F16>), dim3(grid), dim3(kBlock), 0, s, (const V*)feat, n_rows, vecs, lpr_log2, indptr, col,
              n_dst, (V*)out, bad);
}
}  // namespace

extern "C" int coop_gather_mean(const void* feat, int64_t n_rows, int32_t dim, int dtype, const int64_t* indptr,
                                const int32_t* col_global, int64_t n_dst, void* out, void* stream) {
  if (dtype != COOP_F32 && dtype != COOP_F16) return COOP_E_ARG;
  if (dim < 1 || n_rows < 0 || n_dst < 0) return COOP_E_ARG;
  if (n_dst == 0) return COOP_OK;
  if (!feat || !indptr || !out) return COOP_E_NULL;  // col_global may be NULL only if there are no edges; not checkable here
  if ((n_dst + 255) / 256 > 0x7FFFFFFF) return COOP_E_ARG;
  const int64_t row_bytes = (int64_t)dim * (dtype == COOP_F32 ? 4 : 2);
  int32_t* bad = bad_flag();
  if (!bad) return COOP_E_HIP;
  hipStream_t s = (hipStream_t)stream;
  const uintptr_t align = (uintptr_t)feat | (uintptr_t)out | (uintptr_t)row_bytes;
  if (dtype == COOP_F16) {
    if (align % 16 == 0) launch_mean<u32x4, true>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else if (align % 8 == 0) launch_mean<u32x2, true>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else if (align % 4 == 0) launch_mean<uint32_t, true>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else if (align % 2 == 0) launch_mean<uint16_t, true>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else return COOP_E_ARG;
  } else {
    if (align % 16 == 0) launch_mean<u32x4, false>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else if (align % 8 == 0) launch_mean<u32x2, false>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else if (align % 4 == 0) launch_mean<uint32_t, false>(feat, n_rows, row_bytes, indptr, col_global, n_dst, out, bad, s);
    else return COOP_E_ARG;
  }
  if (hipGetLastError() != hipSuccess) return COOP_E_HIP;
  return COOP_OK;
}

extern "C" int coop_gather_status(void* stream) {
  int32_t* bad = bad_flag();
  if (!bad) return COOP_E_HIP;
  hipStream_t s = (hipStream_t)stream;
  int32_t h = 0;
  COOP_HIP_TRY(hipMemcpyAsync(&h, bad, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  COOP_HIP_TRY(hipStreamSynchronize(s));
  if (h) {
    COOP_HIP_TRY(hipMemsetAsync(bad, 0, sizeof(int32_t), s));
    COOP_HIP_TRY(hipStreamSynchronize(s));
    return COOP_E_RANGE;
  }
  return COOP_OK;
}
