// What the files of the C boundary share: the profiling hooks around a launch, the checks of a device
// tensor, the RoPE frequency table, and the two helpers that run the re-encode and RoPE pre-pass kernels
// over a list of blocks or segments.  Defined in ba_api.hip.
#pragma once

#include <mutex>
#include <vector>

#include "../../include/ba.h"
#include "ba_internal.h"
#include "ba_plan.h"

namespace ba {
namespace api {

// ---- optional per-kernel timing (ba_profile_begin / ba_profile_end) ------------------------
struct Profiler {
  std::mutex mu;
  bool on = false;
  int max_records = 0;
  std::vector<hipEvent_t> start[BA_PROFILE_CLASSES], stop[BA_PROFILE_CLASSES];
};
extern Profiler g_prof;

// Brackets one kernel launch with two events on its stream while profiling is on.
struct ProfileScope {
  hipStream_t stream;
  int cls;
  bool active = false;
  hipEvent_t stop_event = nullptr;  // this scope's own: another thread may open a scope of the class meanwhile
  ProfileScope(int cls_, hipStream_t s) : stream(s), cls(cls_) {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (!g_prof.on || (int)g_prof.start[cls].size() >= g_prof.max_records) return;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return;
    if (hipEventCreate(&e1) != hipSuccess) {
      (void)hipEventDestroy(e0);
      return;
    }
    g_prof.start[cls].push_back(e0);
    g_prof.stop[cls].push_back(e1);
    (void)hipEventRecord(e0, stream);
    stop_event = e1;
    active = true;
  }
  ~ProfileScope() {
    if (!active) return;
    // (under the lock: ba_profile_end destroys the events, and must not do so between the
    // constructor and this record)
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (g_prof.on) (void)hipEventRecord(stop_event, stream);
  }
};


size_t elt_size(int32_t dtype);
// pointer, dtype, alignment and strides of a device tensor; BA_OK or a status with ba_last_error() set
int32_t check_tensor(const ba_tensor *t, const char *name, bool allow_f32, int32_t D, int32_t n_heads);
// theta_j / (2 pi) as a Q0.64 fraction, from extended-precision host arithmetic
void build_rope_table(const ba_heads *h, RopeTable *rt);
float scale_log2e(const ba_heads *h);  // softmax scale * log2(e)
int32_t run_reencode(ReencParams p, const RopeTable &rt, int n_blocks, const int32_t *src_off, const int32_t *dst_off,
                     const int32_t *len, const int32_t *pos_old, const int32_t *pos_new, hipStream_t stream);
// Rotate fresh Q (into q_rot, packed, pre-scaled) and fresh K (into k_rot) for segments
// [seg0, seg0 + n) given by start offsets and first positions.
int32_t run_rope_prepass(const ba_heads *h, const RopeTable &rt, const ba_tensor *q, uint16_t *q_rot, const ba_tensor *k,
                         const ba_tensor *k_rot, int n, const int32_t *start, const int32_t *pos0, hipStream_t stream,
                         const RopeRots *rots = nullptr, const RopeRotsSmall *rots_small = nullptr, float *rot_dst = nullptr,
                         int n_rot = 0, float *q_table = nullptr, bool rows_too = false,
                         int table_rows = 0);

}  // namespace api
}  // namespace ba
