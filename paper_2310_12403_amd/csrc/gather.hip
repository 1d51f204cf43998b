// Feature loading step of Algorithm 1: out[i, :] = feat[ids[i], :], an exact copy of bits.
//
// HBM-bound row gather.  A row of `vecs` vectors (16, 8, 4, 2 or 1 bytes each, the widest that the row size and
// the base addresses allow) is moved by `lpr` adjacent lanes (a power of two), so one wave64 load instruction
// covers 64 / lpr rows and each row is read with full-width, coalesced accesses.  Every thread keeps kUnroll rows
// in flight to cover the latency of the random row reads.  Loads and stores are non-temporal: a row is used once.
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

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_bad_mu;
int32_t* g_bad_flag[kMaxDevices] = {};  // per device: a device word, sticky "an id was out of range"

// the current device's flag word, created on first use (a few bytes, kept for the life of the process)
int32_t* bad_flag() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lk(g_bad_mu);
  if (!g_bad_flag[dev]) {
    int32_t* p = nullptr;
    if (hipMalloc((void**)&p, sizeof(int32_t)) != hipSuccess) return nullptr;
    if (hipMemset(p, 0, sizeof(int32_t)) != hipSuccess) { (void)hipFree(p); return nullptr; }
    g_bad_flag[dev] = p;
  }
  return g_bad_flag[dev];
}

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
