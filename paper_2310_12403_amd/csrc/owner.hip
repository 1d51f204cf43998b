// The local half of the id redistribution of Algorithm 1 (Sec. 3.1: vertices are partitioned over the PEs, and every PE
// sends the vertices of its frontier to their owners): a stable counting sort of an id list by owner.  One GPU can show
// this much of the redistribution; the all-to-all that follows it needs a second one.
//
// Every wave owns a contiguous stretch of the list.  Pass 1 counts the stretch's ids per owner (a column of the matrix
// [owner][wave]); the exclusive scan of the matrix in row-major order gives every (owner, wave) its place in the output;
// pass 2 walks the stretch again, 64 ids at a time, and places each id behind the ids of the same owner that precede it.
#include <mutex>

#include "coop_internal.h"
#include "device_utils.h"
#include "variates.h"

namespace coop {
namespace {

constexpr int kMaxParts = 64;        // one lane per owner holds that owner's running place
constexpr int64_t kMaxWaves = 8192;  // columns of the matrix
constexpr int64_t kMinStretch = 512; // ids per wave, at least

struct OwnerRule {
  int scheme;           // COOP_OWNER_RANGE / COOP_OWNER_HASH
  uint32_t n_parts;
  uint64_t n_vertices;
  uint32_t key;         // COOP_OWNER_HASH
};

__device__ __forceinline__ uint32_t owner_of(const OwnerRule& r, uint32_t v) {
  if (r.scheme == COOP_OWNER_RANGE) return (uint32_t)(((uint64_t)v * r.n_parts) / r.n_vertices);
  return (uint32_t)(((uint64_t)mix32(v ^ r.key) * r.n_parts) >> 32);
}

struct Stretch { int64_t beg, end; };
__device__ __forceinline__ Stretch stretch_of(int64_t n, int64_t n_waves, int64_t w) {
  const int64_t len = ((n + n_waves - 1) / n_waves + kWave - 1) & ~(int64_t)(kWave - 1);  // a multiple of 64
  const int64_t beg = w * len;
  return Stretch{beg < n ? beg : n, beg + len < n ? beg + len : n};
}

__global__ __launch_bounds__(kBlock) void k_owner_count(const int32_t* __restrict__ ids, int64_t n, int64_t n_waves, OwnerRule rule,
                                                        uint32_t* __restrict__ matrix, int32_t* bad) {
  __shared__ uint32_t cnt[kWavesPerBlock][kMaxParts];
  const int wib = uniform_wave_in_block();
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + wib;
  if (w >= n_waves) return;
  const int lane = lane_id();
  cnt[wib][lane] = 0;
  __builtin_amdgcn_wave_barrier();
  const Stretch st = stretch_of(n, n_waves, w);
  bool out_of_range = false;
  for (int64_t i = st.beg + lane; i < st.end; i += kWave) {
    const uint32_t v = (uint32_t)ids[i];
    if ((uint64_t)v >= rule.n_vertices) { out_of_range = true; continue; }  // (left out of every group; reported)
    atomicAdd(&cnt[wib][owner_of(rule, v)], 1u);
  }
  if (out_of_range) atomicOr(bad, 1);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  if ((uint32_t)lane < rule.n_parts) matrix[(int64_t)lane * n_waves + w] = cnt[wib][lane];
}

__global__ __launch_bounds__(kBlock) void k_owner_scatter(const int32_t* __restrict__ ids, int64_t n, int64_t n_waves, OwnerRule rule,
                                                          const uint32_t* __restrict__ place, int32_t* __restrict__ ids_out,
                                                          int32_t* __restrict__ origin_out, int64_t* __restrict__ offsets_out) {
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + uniform_wave_in_block();
  if (w >= n_waves) return;
  const uint32_t lane = (uint32_t)lane_id();
  if (w == 0) {  // group boundaries; place[n_parts * n_waves] is the number of ids in range
    if (lane < rule.n_parts) offsets_out[lane] = place[(int64_t)lane * n_waves];
    if (lane == 0) offsets_out[rule.n_parts] = place[(int64_t)rule.n_parts * n_waves];
  }
  uint32_t run = lane < rule.n_parts ? place[(int64_t)lane * n_waves + w] : 0u;  // lane p: next place of owner p
  const Stretch st = stretch_of(n, n_waves, w);
  for (int64_t base = st.beg; base < st.end; base += kWave) {
    const int64_t i = base + lane;
    uint32_t v = 0;
    bool valid = false;
    if (i < st.end) {
      v = (uint32_t)ids[i];
      valid = (uint64_t)v < rule.n_vertices;
    }
    const uint32_t o = valid ? owner_of(rule, v) : 0xFFFFFFFFu;
    uint64_t todo = ballot64(valid);
    while (todo != 0) {  // one round per owner present among the 64 ids
      const int leader = __builtin_ctzll(todo);
      const uint32_t ol = (uint32_t)__builtin_amdgcn_readlane((int)o, leader);
      const uint64_t same = ballot64(o == ol);
      const uint32_t first = (uint32_t)__builtin_amdgcn_readlane((int)run, (int)ol);
      if (o == ol) {
        const uint32_t at = first + lanes_below(same);
        ids_out[at] = (int32_t)v;
        if (origin_out != nullptr) origin_out[at] = (int32_t)i;
      }
      if (lane == ol) run += (uint32_t)__popcll(same);
      todo &= ~same;
    }
  }
}

}  // namespace
}  // namespace coop

using namespace coop;

extern "C" size_t coop_bucket_workspace_bytes(int64_t n, int n_parts) {
  if (n < 0 || n_parts < 1 || n_parts > kMaxParts) return 0;
  const int64_t cells = (int64_t)n_parts * kMaxWaves + 1;
  return (size_t)(2 * cells) * sizeof(uint32_t) + scan_tmp_bytes(cells) + 512;
}

namespace {
// the checks and launches shared by the two entry points; `workspace` holds coop_bucket_workspace_bytes(n, n_parts) bytes
int bucket_launch(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, uint64_t seed, int32_t* ids_out,
                  int32_t* origin_out, int64_t* offsets_out, void* workspace, hipStream_t s) {
  int32_t* bad = bad_flag();
  if (!bad) return COOP_E_HIP;
  int64_t n_waves = (n + kMinStretch - 1) / kMinStretch;
  n_waves = n_waves < 1 ? 1 : n_waves > kMaxWaves ? kMaxWaves : n_waves;
  const int64_t cells = (int64_t)n_parts * n_waves;
  uint32_t* matrix = (uint32_t*)workspace;
  uint32_t* place = matrix + (((cells + 1) + 1) & ~(int64_t)1);  // [cells + 1], 8-byte aligned
  void* scan_tmp = place + (((cells + 1) + 1) & ~(int64_t)1);
  const OwnerRule rule{scheme, (uint32_t)n_parts, (uint64_t)n_vertices, (uint32_t)(seed ^ (seed >> 32))};
  const dim3 grid((unsigned)((n_waves + kWavesPerBlock - 1) / kWavesPerBlock));
  COOP_LAUNCH(K_OWNER_COUNT, k_owner_count, grid, dim3(kBlock), 0, s, ids, n, n_waves, rule, matrix, bad);
  scan_u32_to_u32(matrix, cells, place, scan_tmp, s);
  COOP_LAUNCH(K_OWNER_SCATTER, k_owner_scatter, grid, dim3(kBlock), 0, s, ids, n, n_waves, rule, (const uint32_t*)place, ids_out, origin_out,
              offsets_out);
  if (hipGetLastError() != hipSuccess) return COOP_E_HIP;
  return COOP_OK;
}

int bucket_check(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, const int32_t* ids_out,
                 const int64_t* offsets_out) {
  if (n < 0 || n >= ((int64_t)1 << 31) || n_vertices < 1 || n_vertices >= ((int64_t)1 << 31)) return COOP_E_ARG;
  if (n_parts < 1 || n_parts > kMaxParts || (scheme != COOP_OWNER_RANGE && scheme != COOP_OWNER_HASH)) return COOP_E_ARG;
  if (!offsets_out || (n > 0 && (!ids || !ids_out))) return COOP_E_NULL;
  return COOP_OK;
}

// ---- the workspace of coop_bucket_by_owner_static ---------------------------------------------------------------------
// The counter matrix, its scan and the scan's tile sums for the largest call (64 owners): 4 MiB and a little, a device
// array of this library's code object.  Every GPU holds its own copy at its own address until the process ends; the
// name below is only the host-side handle by which hipGetSymbolAddress finds the current device's copy.
constexpr size_t kStaticScratchBytes = (size_t)4 * 1024 * 1024 + 65536;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};  // per device: the device address of that device's `scratch`

// device address of the current device's scratch array (looked up once per device; allocates nothing)
int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return COOP_E_HIP;
  if (dev < 0 || dev >= kMaxDevices) return COOP_E_CAPACITY;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return COOP_E_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return COOP_OK;
}
}  // namespace

extern "C" int coop_bucket_by_owner(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, uint64_t seed,
                                    int32_t* ids_out, int32_t* origin_out, int64_t* offsets_out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  const int rc = bucket_check(ids, n, n_vertices, n_parts, scheme, ids_out, offsets_out);
  if (rc != COOP_OK) return rc;
  if (!workspace) return COOP_E_NULL;
  if (workspace_bytes < coop_bucket_workspace_bytes(n, n_parts) || ((uintptr_t)workspace & 7) != 0) return COOP_E_ARG;
  return bucket_launch(ids, n, n_vertices, n_parts, scheme, seed, ids_out, origin_out, offsets_out, workspace, (hipStream_t)stream);
}

extern "C" int coop_bucket_by_owner_static(const int32_t* ids, int64_t n, int64_t n_vertices, int n_parts, int scheme, uint64_t seed,
                                           int32_t* ids_out, int32_t* origin_out, int64_t* offsets_out, void* stream) {
  const int rc = bucket_check(ids, n, n_vertices, n_parts, scheme, ids_out, offsets_out);
  if (rc != COOP_OK) return rc;
  // (a call whose workspace would not fit the array is refused; with the limits above, 64 owners and 2^31 - 1 ids, none is)
  if (coop_bucket_workspace_bytes(n, n_parts) > kStaticScratchBytes) return COOP_E_CAPACITY;
  void* ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs != COOP_OK) return rs;
  // Nothing in the workspace has to start at zero: the first kernel stores every cell of the matrix that the scan reads,
  // the scan stores every tile sum and every place that the second kernel reads.
  return bucket_launch(ids, n, n_vertices, n_parts, scheme, seed, ids_out, origin_out, offsets_out, ws, (hipStream_t)stream);
}
