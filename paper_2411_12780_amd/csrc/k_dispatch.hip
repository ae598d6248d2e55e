// Kernel selection: the MFMA kernels take the bf16 shapes they are built for,
// everything else goes to the run-time-typed kernels.  Also holds the optional
// per-launch timing of a block's contraction kernels used by the benchmark.
#include <vector>

#include "common.h"

namespace ppll {

namespace {
thread_local LaunchTimes* t_times = nullptr;

hipEvent_t pooled_event(LaunchTimes& t) {
  if (!t.pool.empty()) { hipEvent_t e = t.pool.back(); t.pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

void profile_bind(LaunchTimes* t) { t_times = t; }
bool profile_enabled() { return t_times != nullptr; }

// Adds the elapsed time of every bracketed launch since the last drain, per kind (0: GEMM, 1: convolution).
int profile_drain(LaunchTimes& t) {
  for (TimedLaunch& l : t.timed) {
    PPLL_HIP(hipEventSynchronize(l.b));
    float dt = 0.f;
    PPLL_HIP(hipEventElapsedTime(&dt, l.a, l.b));
    t.ms[l.kind] += dt; t.units[l.kind] += l.units; ++t.launches[l.kind];
    t.pool.push_back(l.a); t.pool.push_back(l.b);
  }
  t.timed.clear();
  return PPLL_OK;
}

void profile_destroy(LaunchTimes& t) {
  for (TimedLaunch& l : t.timed) { (void)hipEventDestroy(l.a); (void)hipEventDestroy(l.b); }
  for (hipEvent_t e : t.pool) (void)hipEventDestroy(e);
  t.timed.clear(); t.pool.clear();
}

// Brackets one kernel launch with a pair of events when the calling thread has a record bound.
int profile_begin(hipStream_t s, double units, void** token, int kind) {
  *token = nullptr;
  if (!t_times) return PPLL_OK;
  TimedLaunch tl{pooled_event(*t_times), pooled_event(*t_times), units, kind};
  if (!tl.a || !tl.b) { set_error("hipEventCreate failed"); return PPLL_ERR_HIP; }
  PPLL_HIP(hipEventRecord(tl.a, s));
  t_times->timed.push_back(tl);
  *token = (void*)(uintptr_t)t_times->timed.size();
  return PPLL_OK;
}
int profile_end(hipStream_t s, void* token) {
  if (!token || !t_times) return PPLL_OK;
  PPLL_HIP(hipEventRecord(t_times->timed[(size_t)(uintptr_t)token - 1].b, s));
  return PPLL_OK;
}

int launch_gemm(hipStream_t s, const GemmArgs& g) {
  if (gemm_rows_supported(g)) return launch_gemm_rows(s, g);   // few output rows: latency, not throughput
  return gemm_mfma_supported(g) ? launch_gemm_mfma(s, g, g.splitk_ws, g.splitk_floats) : launch_gemm_generic(s, g);
}

bool gemm_group_in_one_launch(const GemmArgs* gs, int n) {
  bool all = n > 1;
  for (int j = 0; j < n && all; ++j) all = gemm_mfma_groupable(gs[j]);
  return all;
}

// use_workspace: the grouped launch may pass divided tiles through the products' split-K scratch (gs[0].splitk_ws);
// only for a launch that is the sole user of that scratch while it runs.
int launch_gemm_group(hipStream_t s, const GemmArgs* gs, int n, bool one_launch, bool use_workspace) {
  if (n <= 0) return PPLL_OK;
  bool all = n > 1;
  long tiles = 0;
  for (int j = 0; j < n && all; ++j) {
    all = gemm_mfma_groupable(gs[j]);
    tiles += (long)((gs[j].M + 127) / 128) * ((gs[j].N + 127) / 128);
  }
  // one launch when the products together have enough output tiles for the chip; a small set runs
  // product by product, each with split-K (their reduction index is the long one)
  if (all && (tiles >= 128 || one_launch))
    return launch_gemm_mfma_grouped(s, gs, n, use_workspace ? gs[0].splitk_ws : nullptr, use_workspace ? gs[0].splitk_floats : 0);
  for (int j = 0; j < n; ++j) {
    const bool fused = gemm_fuses_colsum(gs[j]);
    if (gs[j].colsum && !fused) { set_error("launch_gemm_group: column sums need the MFMA kernel"); return PPLL_ERR_CONFIG; }
    PPLL_TRY(launch_gemm(s, gs[j]));
  }
  return PPLL_OK;
}

int launch_attention_fwd(hipStream_t s, const void* qkv, int dt, int B, int T, int H, int dh, void* out, float* lse) {
  if (attention_mfma_supported(dt, T, H, dh, qkv, out, nullptr, nullptr)) return launch_attention_fwd_mfma(s, qkv, B, T, H, out, lse);
  return launch_attention_fwd_generic(s, qkv, dt, B, T, H, dh, out, lse);
}

int launch_attention_bwd(hipStream_t s, const void* qkv, const void* out, const void* dout, const float* lse, int dt,
                         int B, int T, int H, int dh, void* dqkv) {
  if (attention_mfma_supported(dt, T, H, dh, qkv, out, dout, dqkv))
    return launch_attention_bwd_mfma(s, qkv, out, dout, lse, B, T, H, dqkv);
  return launch_attention_bwd_generic(s, qkv, out, dout, lse, dt, B, T, H, dh, dqkv);
}

}  // namespace ppll
