// Calibration and diagnostics of the Block-attention library: the relative speed of the device's XCDs
// under the attention core's load (ba_heads.xcd_speed), where the time of one final-block launch goes,
// and the MFMA rate the device sustains.  Each runs kernels of the library on synthetic data in a
// caller's workspace and synchronises the stream: not hot-path calls.
#include <string.h>

#include <algorithm>
#include <vector>

#include "../../include/ba.h"
#include "ba_internal.h"
#include "ba_plan.h"

namespace {
using ba::align256;
using ba::device_fail;
using ba::fail;
using ba::num_cus;
}  // namespace

// ------------------------------------------------------------------------------------------
// Calibration: relative XCD speeds under the attention core's load (ba_heads.xcd_speed).
namespace {
constexpr int kProbeCtx = 31744, kProbeLq = 256, kProbeHq = 32, kProbeHkv = 8, kProbeD = 128;
constexpr int kProbeWarmRuns = 3, kProbeRuns = 4;  // launches to reach the steady clock, then launches that are read
constexpr int kProbeMaxWg = 4096;
ba_heads probe_heads() {
  ba_heads h;
  memset(&h, 0, sizeof(h));
  h.n_q_heads = kProbeHq;
  h.n_kv_heads = kProbeHkv;
  h.head_dim = kProbeD;
  h.rope_base = 500000.0;
  h.rope_layout = BA_ROPE_INTERLEAVED;
  return h;
}
struct ProbeLayout {
  size_t kv_bytes, q_bytes, kvf_bytes, clock_bytes, final_bytes;
  size_t total() const { return 2 * kv_bytes + 2 * q_bytes + 2 * kvf_bytes + clock_bytes + final_bytes; }
};
ProbeLayout probe_layout() {
  ProbeLayout l;
  l.kv_bytes = align256((size_t)kProbeCtx * kProbeHkv * kProbeD * 2);
  l.q_bytes = align256((size_t)kProbeLq * kProbeHq * kProbeD * 2);
  l.kvf_bytes = align256((size_t)kProbeLq * kProbeHkv * kProbeD * 2);
  l.clock_bytes = align256((size_t)kProbeMaxWg * ba::kProbeRecord * sizeof(unsigned long long) * kProbeRuns);
  const ba_heads h = probe_heads();
  const int32_t cu_q[2] = {0, kProbeLq}, cu_ctx[2] = {0, kProbeCtx};
  l.final_bytes = align256(ba_final_block_attention_workspace_bytes(&h, 1, cu_q, cu_ctx, BA_ROPE_NONE, 0));
  return l;
}
}  // namespace

extern "C" size_t ba_measure_xcd_speed_workspace_bytes(void) { return probe_layout().total(); }

namespace {
// Runs the probe launches and reads the workgroups' records back: kProbeRuns launches' worth, one
// after the other in *rec (the clocks of the XCDs drift by a few per cent from launch to launch, so
// one launch alone is a noisy sample).  Empty: the launch has a shape there is nothing to learn from.
// Synchronises the stream.
int32_t run_probe(void *ws, size_t ws_bytes, void *stream_, const float *xcd_speed, std::vector<unsigned long long> *rec,
                  int64_t *n_wg_out) {
  hipStream_t stream = (hipStream_t)stream_;
  rec->clear();
  *n_wg_out = 0;
  const ProbeLayout l = probe_layout();
  if (!ws || ws_bytes < l.total() || ((uintptr_t)ws & 255))
    return fail(BA_ERR_WORKSPACE, "final-block probe: 256-byte aligned workspace of %zu bytes needed, %zu given", l.total(),
                ws_bytes);
  char *wp = (char *)ws;
  ba_heads h = probe_heads();
  h.xcd_speed = xcd_speed;
  auto tensor = [&](size_t bytes, int heads_n) {
    ba_tensor t;
    t.ptr = wp;
    t.stride_head = kProbeD;
    t.stride_tok = (int64_t)heads_n * kProbeD;
    t.dtype = BA_DTYPE_BF16;
    wp += bytes;
    return t;
  };
  const ba_tensor kc = tensor(l.kv_bytes, kProbeHkv), vc = tensor(l.kv_bytes, kProbeHkv);
  const ba_tensor q = tensor(l.q_bytes, kProbeHq), o = tensor(l.q_bytes, kProbeHq);
  const ba_tensor kf = tensor(l.kvf_bytes, kProbeHkv), vf = tensor(l.kvf_bytes, kProbeHkv);
  unsigned long long *clk = (unsigned long long *)wp;
  wp += l.clock_bytes;
  // keys, values and queries with the bit activity of real data (the clock a part sustains depends on it)
  hipError_t e = ba::launch_fill_random_bf16((uint16_t *)kc.ptr, (2 * l.kv_bytes + l.q_bytes) / 2, 0x9e3779b9u, stream);
  if (e == hipSuccess)
    e = ba::launch_fill_random_bf16((uint16_t *)kf.ptr, 2 * l.kvf_bytes / 2, 0x85ebca6bu, stream);
  if (e == hipSuccess) e = hipMemsetAsync(clk, 0, l.clock_bytes, stream);
  if (e != hipSuccess) return device_fail(e, "final-block probe: fill");
  const int32_t cu_q[2] = {0, kProbeLq}, cu_ctx[2] = {0, kProbeCtx};
  int32_t rc = BA_OK;
  ba::FinalPlan pl;
  if ((rc = ba::plan_final(&h, 1, cu_q, cu_ctx, BA_ROPE_NONE, false, num_cus(), &pl))) return rc;
  const int64_t n_wg = pl.total_tiles * kProbeHkv * pl.n_splits;
  const bool readable = n_wg >= ba::kNumXcds && n_wg <= kProbeMaxWg;
  const size_t per_run = (size_t)n_wg * ba::kProbeRecord;
  if (readable) rec->resize(per_run * kProbeRuns);
  // (back to back, as a caller's layers run: a pause between launches lets the clocks recover and
  // shows a faster part than the one that does the work; every measured launch has records of its own)
  for (int run = 0; run < kProbeWarmRuns + kProbeRuns && rc == BA_OK; ++run) {
    ba::probe_clock() = run >= kProbeWarmRuns && readable ? clk + per_run * (run - kProbeWarmRuns) : nullptr;
    rc = ba_final_block_attention(&h, &q, &kc, &vc, &kf, &vf, &o, nullptr, 1, cu_q, cu_ctx, nullptr, BA_ROPE_NONE, wp,
                                  l.final_bytes, stream_);
    ba::probe_clock() = nullptr;
  }
  if (rc) return rc;
  if ((e = hipStreamSynchronize(stream)) != hipSuccess) return device_fail(e, "final-block probe: synchronize");
  if (!readable) return BA_OK;
  if ((e = hipMemcpy(rec->data(), clk, rec->size() * sizeof(unsigned long long), hipMemcpyDeviceToHost)) != hipSuccess)
    return device_fail(e, "final-block probe: read-back");
  *n_wg_out = n_wg;
  return BA_OK;
}
}  // namespace

extern "C" int32_t ba_measure_xcd_speed(float speed_out[8], void *ws, size_t ws_bytes, void *stream_) {
  if (!speed_out) return fail(BA_ERR_INVALID_ARG, "speed_out: null");
  float speed[ba::kNumXcds];
  for (int x = 0; x < ba::kNumXcds; ++x) speed_out[x] = speed[x] = 1.0f;
  // Two passes: equal splits first, then splits sized by the first pass's figures, whose residual
  // corrects them.  What is measured is how long an XCD's workgroups take from entry to the end of
  // their walk (not its clock alone: cycles per tile differ between XCDs too, with the place of their
  // keys in memory and with the causal tiles of the last split); a split's share is scaled by
  // mean / own, which equalises those times where time is proportional to tiles.
  for (int pass = 0; pass < 2; ++pass) {
    std::vector<unsigned long long> rec;
    int64_t n_wg = 0;
    if (int32_t rc = run_probe(ws, ws_bytes, stream_, pass ? speed : nullptr, &rec, &n_wg)) return rc;
    if (n_wg == 0) return BA_OK;  // nothing to learn from such a launch: equal speeds
    double sum[ba::kNumXcds] = {0}, total = 0.0;
    int cnt[ba::kNumXcds] = {0};
    for (int64_t i = 0; i < n_wg * kProbeRuns; ++i) {
      const unsigned long long *r = &rec[(size_t)i * ba::kProbeRecord];
      const int x = ba::xcd_of_workgroup((unsigned)(i % n_wg));
      if ((int)r[0] != x || r[5] <= r[2]) return BA_OK;  // not the mapping the planner assumes: equal speeds
      sum[x] += (double)(r[5] - r[2]);
      ++cnt[x];
    }
    for (int x = 0; x < ba::kNumXcds; ++x) {
      if (!cnt[x]) return BA_OK;
      sum[x] /= cnt[x];
      total += sum[x];
    }
    double next[ba::kNumXcds], norm = 0.0;
    for (int x = 0; x < ba::kNumXcds; ++x) {
      next[x] = (double)speed[x] * (total / ba::kNumXcds) / sum[x];
      norm += next[x];
    }
    for (int x = 0; x < ba::kNumXcds; ++x) {
      const double v = next[x] * ba::kNumXcds / norm;
      if (!(v >= 0.5 && v <= 2.0)) return BA_OK;  // implausible: keep equal speeds
      speed[x] = (float)v;
    }
  }
  for (int x = 0; x < ba::kNumXcds; ++x) speed_out[x] = speed[x];
  return BA_OK;
}

extern "C" int32_t ba_diag_final_block_phases(double phases_us[BA_DIAG_PHASES], const float *xcd_speed, void *ws,
                                              size_t ws_bytes, void *stream_) {
  if (!phases_us) return fail(BA_ERR_INVALID_ARG, "phases_us: null");
  for (int i = 0; i < BA_DIAG_PHASES; ++i) phases_us[i] = 0.0;
  std::vector<unsigned long long> rec;
  int64_t n_wg = 0;
  if (int32_t rc = run_probe(ws, ws_bytes, stream_, xcd_speed, &rec, &n_wg)) return rc;
  if (n_wg == 0) return fail(BA_ERR_UNSUPPORTED, "final-block phases: this device's launch is not the shape the probe times");
  // means over the launches that were read; per launch: its own first entry and last store
  const double tick_us = 0.01;  // the real-time counter runs at 100 MHz
  for (int run = 0; run < kProbeRuns; ++run) {
    const unsigned long long *base = &rec[(size_t)run * n_wg * ba::kProbeRecord];
    unsigned long long first = ~0ull, last = 0;
    double longest_walk = 0.0;
    for (int64_t wg = 0; wg < n_wg; ++wg) {
      const unsigned long long *r = base + (size_t)wg * ba::kProbeRecord;
      if (!(r[2] <= r[3] && r[3] <= r[6] && r[6] <= r[7] && r[7] <= r[5] && r[5] <= r[8] && r[8] <= r[9]))
        return fail(BA_ERR_DEVICE, "final-block phases: workgroup %lld left marks out of order", (long long)wg);
      first = std::min(first, r[2]);
      last = std::max(last, r[9]);
      phases_us[0] += (double)(r[3] - r[2]);
      phases_us[1] += (double)(r[6] - r[3]);
      phases_us[2] += (double)(r[7] - r[6]);
      phases_us[3] += (double)(r[5] - r[7]);
      phases_us[4] += (double)(r[9] - r[5]);
      phases_us[5] += (double)(r[9] - r[2]);
      longest_walk = std::max(longest_walk, (double)(r[5] - r[7]));
    }
    phases_us[6] += (double)(last - first) * (double)n_wg;  // (scaled like the sums above)
    phases_us[7] += longest_walk * (double)n_wg;
  }
  for (int i = 0; i < BA_DIAG_PHASES; ++i) phases_us[i] *= tick_us / ((double)n_wg * kProbeRuns);
  return BA_OK;
}

// ------------------------------------------------------------------------------------------
// Diagnostic: the MFMA rate the device sustains on data-like operands (see diag.hip).
extern "C" size_t ba_diag_mfma_ceiling_workspace_bytes(void) { return align256(ba::diag_mfma_workspace_bytes(num_cus())); }

extern "C" int32_t ba_diag_mfma_ceiling(int32_t lds_reads_per_two_mfma, double *tflops, double *clock_ghz,
                                        double *pipe_busy, void *ws, size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (lds_reads_per_two_mfma < 0 || lds_reads_per_two_mfma > 2)
    return fail(BA_ERR_INVALID_ARG, "lds_reads_per_two_mfma: 0, 1 or 2");
  const int n_wg = num_cus(), iters = 6000, runs = 5;
  const size_t need = ba_diag_mfma_ceiling_workspace_bytes();
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 255))
    return fail(BA_ERR_WORKSPACE, "MFMA diagnostic: 256-byte aligned workspace of %zu bytes needed, %zu given", need, ws_bytes);
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return device_fail(e, "MFMA diagnostic: event");
  if ((e = hipEventCreate(&e1)) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return device_fail(e, "MFMA diagnostic: event");
  }
  e = ba::launch_mfma_ceiling(lds_reads_per_two_mfma, n_wg, iters, ws, 1u, stream);  // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, stream);
  for (int r = 0; r < runs && e == hipSuccess; ++r) e = ba::launch_mfma_ceiling(lds_reads_per_two_mfma, n_wg, iters, ws, 7u + r, stream);
  if (e == hipSuccess) e = hipEventRecord(e1, stream);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  std::vector<unsigned long long> clk((size_t)n_wg * 8 * 2);
  if (e == hipSuccess) e = hipMemcpy(clk.data(), ws, clk.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return device_fail(e, "MFMA diagnostic");
  // Per workgroup, the wave that ran longest: the two waves of a SIMD do not share its matrix pipe
  // evenly (one may issue most of its loop before the other), so a single wave's time understates
  // how long the pipe was in use.
  double cyc = 0.0, ticks = 0.0, cyc_longest = 0.0;
  for (int wg = 0; wg < n_wg; ++wg) {
    unsigned long long longest = 0;
    for (int w = 0; w < 8; ++w) {
      const unsigned long long c = clk[((size_t)wg * 8 + w) * 2];
      cyc += (double)c;
      ticks += (double)clk[((size_t)wg * 8 + w) * 2 + 1];
      longest = std::max(longest, c);
    }
    cyc_longest += (double)longest;
  }
  const double waves = (double)n_wg * 8, mfma_per_wave = (double)iters * 16;
  if (tflops) *tflops = runs * waves * mfma_per_wave * 32768.0 / (ms * 1e-3) / 1e12;
  if (clock_ghz) *clock_ghz = ticks > 0 ? cyc / (10.0 * ticks) : 0.0;
  // two waves share a SIMD's matrix pipe, an MFMA of this shape occupies it for 32 cycles
  if (pipe_busy) *pipe_busy = cyc_longest > 0 ? mfma_per_wave * 32.0 * 2.0 / (cyc_longest / n_wg) : 0.0;
  return BA_OK;
}
