// Kernel selection: the MFMA kernels take the bf16 shapes they are built for,
// everything else goes to the run-time-typed kernels.
#include "common.h"

namespace ppll {

int launch_gemm(hipStream_t s, const GemmArgs& g) { return launch_gemm_generic(s, g); }

int launch_attention_fwd(hipStream_t s, const void* qkv, int dt, int B, int T, int H, int dh, void* out, float* lse) {
  return launch_attention_fwd_generic(s, qkv, dt, B, T, H, dh, out, lse);
}

int launch_attention_bwd(hipStream_t s, const void* qkv, const void* out, const void* dout, const float* lse, int dt,
                         int B, int T, int H, int dh, void* dqkv) {
  return launch_attention_bwd_generic(s, qkv, out, dout, lse, dt, B, T, H, dh, dqkv);
}

}  // namespace ppll
