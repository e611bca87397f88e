// tc_merge_noalloc: Stage II (Section 3.3.2) for callers that cannot allocate.  Same kernels as
// tc_merge; the scratch they need (row norms, the similarity matrix, the merge list) lives in a
// file-scope device array instead of a caller-supplied workspace.
#include <mutex>

#include "tc_internal.h"

namespace tc {

// One copy of this array exists on every GPU the library runs on, from the first use of the library on
// that GPU until the process ends.  Host code never uses the array's name as an address: the device
// address is looked up once per device with hipGetSymbolAddress and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[TC_NOALLOC_SCRATCH_BYTES];

static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64];  // per device; nullptr until looked up

// Device address of `scratch` on the current device (nullptr on failure).
static void* scratch_address() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// The merge list is the one region whose entries are only written for tokens that are merged: it starts
// at zero (source 0, destination 0) so that a malformed `order` cannot leave stale indices of an earlier
// call in it.  A plain kernel rather than a memset, so that the call can be captured into a HIP graph.
__global__ __launch_bounds__(256) void noalloc_clear(int32_t* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = 0;
}

}  // namespace tc

using namespace tc;

extern "C" int tc_merge_noalloc(const tc_params* p, const void* X, const void* metric, const int32_t* order, void* X_out,
                                int32_t* kept_idx, int32_t* merge_dst, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;
  if (!X || !metric || !order || !X_out || !kept_idx || !merge_dst) return TC_ERR_NULL;
  if (misaligned(X) || misaligned(metric) || misaligned(order) || misaligned(X_out) || misaligned(kept_idx) ||
      misaligned(merge_dst))
    return TC_ERR_ALIGN;
  // the three regions tc_merge takes from its workspace, laid out back to back
  const size_t n_rnorm = (size_t)pl.B * pl.kp, n_sim = (size_t)pl.B * pl.nB * (pl.nA > 0 ? pl.nA : 1),
               n_mlist = (size_t)pl.B * (pl.m > 0 ? pl.m : 1) * 2;
  const size_t off_rnorm = 0, off_sim = align256(n_rnorm * 4), off_mlist = off_sim + align256(n_sim * 4),
               total = off_mlist + align256(n_mlist * 4);
  if (total > (size_t)TC_NOALLOC_SCRATCH_BYTES) return TC_ERR_SCRATCH;
  char* base = static_cast<char*>(scratch_address());
  if (!base) return TC_ERR_HIP;
  hipStream_t st = (hipStream_t)stream;
  int32_t* mlist = reinterpret_cast<int32_t*>(base + off_mlist);
  const int blocks = (int)((n_mlist + 255) / 256 < 64 ? (n_mlist + 255) / 256 : 64);
  noalloc_clear<<<blocks, 256, 0, st>>>(mlist, n_mlist);
  return launch_merge(pl, p->dtype, X, metric, order, X_out, kept_idx, merge_dst, reinterpret_cast<float*>(base + off_rnorm),
                      reinterpret_cast<float*>(base + off_sim), mlist, st);
}
