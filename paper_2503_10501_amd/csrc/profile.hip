// Per-kernel timing with HIP events, used only by tc_profile_compress (a measurement aid).
#include <vector>

#include "tc_internal.h"

namespace tc {

struct ProfRecord { int kind, tag; hipEvent_t start, stop; };
struct Profiler { std::vector<ProfRecord> recs; };
static thread_local Profiler* g_prof = nullptr;

bool profiling_active() { return g_prof != nullptr; }

void prof_begin(int kind, int tag, hipStream_t st) {
  if (!g_prof) return;
  // A record is pushed even when its events could not be created (both stay null): prof_end() always
  // pairs with the record of its own prof_begin() and never stamps an older one.
  ProfRecord r{kind, tag, nullptr, nullptr};
  if (hipEventCreate(&r.start) != hipSuccess) r.start = nullptr;
  if (r.start && hipEventCreate(&r.stop) != hipSuccess) {
    (void)hipEventDestroy(r.start);
    r.start = r.stop = nullptr;
  }
  if (r.start) (void)hipEventRecord(r.start, st);
  g_prof->recs.push_back(r);
}

void prof_end(hipStream_t st) {
  if (!g_prof || g_prof->recs.empty()) return;
  if (g_prof->recs.back().stop) (void)hipEventRecord(g_prof->recs.back().stop, st);
}

}  // namespace tc

using namespace tc;

extern "C" int tc_profile_compress(const tc_params* p, const void* Q, const void* K, const void* V, const void* X,
                                   void* X_out, int32_t* kept_idx, int32_t* merge_dst, int32_t* info, void* ws,
                                   size_t ws_bytes, void* stream, float* ms_by_kind, int32_t* launches_by_kind,
                                   float* jacobi_update_ms_by_sweep, int32_t max_sweeps_out,
                                   int64_t* jacobi_work) {
  if (!ms_by_kind || !launches_by_kind) return TC_ERR_NULL;
  Profiler prof;
  g_prof = &prof;
  const int rc = tc_compress(p, Q, K, V, X, X_out, kept_idx, merge_dst, nullptr, nullptr, nullptr, info, ws, ws_bytes,
                             stream);
  g_prof = nullptr;
  const hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  for (int k = 0; k < TC_PROF_KINDS; k++) { ms_by_kind[k] = 0.f; launches_by_kind[k] = 0; }
  if (jacobi_update_ms_by_sweep)
    for (int s = 0; s < max_sweeps_out; s++) jacobi_update_ms_by_sweep[s] = 0.f;
  for (auto& r : prof.recs) {
    float ms = 0.f;
    if (!r.start) continue;  // its events could not be created: not timed
    if (e == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      ms_by_kind[r.kind] += ms;
      launches_by_kind[r.kind] += 1;
      if (r.kind == PK_JUPDATE && jacobi_update_ms_by_sweep && r.tag < max_sweeps_out)
        jacobi_update_ms_by_sweep[r.tag] += ms;
    }
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  if (rc != TC_OK) return rc;
  if (e != hipSuccess) return TC_ERR_HIP;
  if (jacobi_work) {  // the solver state of every image is still in the workspace
    jacobi_work[0] = jacobi_work[1] = 0;
    Plan pl;
    if (make_plan(p, &pl) == TC_OK && pl.B > 0) {
      std::vector<EigState> host((size_t)pl.B);
      if (hipMemcpy(host.data(), at<EigState>(ws, pl.off_state), host.size() * sizeof(EigState), hipMemcpyDeviceToHost) != hipSuccess)
        return TC_ERR_HIP;
      for (const EigState& st : host) {
        jacobi_work[0] += st.tiles;
        for (unsigned v : st.rot_steps) jacobi_work[1] += v;
      }
    }
  }
  return TC_OK;
}
