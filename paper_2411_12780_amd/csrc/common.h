// Shared declarations of the HIP implementation: element types, error plumbing
// and the launcher interface between the block engine and the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <vector>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ppll.h"

namespace ppll {

// Element type of a buffer as seen by a kernel.
enum DType : int { F32 = 0, BF16 = 1 };
inline size_t dtype_size(int dt) { return dt == BF16 ? 2 : 4; }

void set_error(const char* fmt, ...);

#define PPLL_HIP(expr)                                                              \
  do {                                                                              \
    hipError_t e__ = (expr);                                                        \
    if (e__ != hipSuccess) {                                                        \
      ::ppll::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__),     \
                        __FILE__, __LINE__);                                        \
      return PPLL_ERR_HIP;                                                          \
    }                                                                               \
  } while (0)

#define PPLL_TRY(expr)                \
  do {                                \
    int s__ = (expr);                 \
    if (s__ != PPLL_OK) return s__;   \
  } while (0)

#ifdef __HIPCC__
// bf16 <-> fp32 by bit manipulation, round to nearest even.
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
// float -> bf16, round to nearest even: gfx950's v_cvt_pk_bf16_f32 (one instruction for two values)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const bf16x2_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float ld_f(const void* p, size_t i, int dt) {
  return dt == BF16 ? bf16_to_f32(((const uint16_t*)p)[i]) : ((const float*)p)[i];
}
__device__ __forceinline__ void st_f(void* p, size_t i, float v, int dt) {
  if (dt == BF16) ((uint16_t*)p)[i] = f32_to_bf16(v);
  else ((float*)p)[i] = v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Orders LDS traffic between the lanes of one wave (writes before, reads after).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// Exact-form GELU through the rational erf approximation of Abramowitz & Stegun 7.1.26
// (|error| < 1.5e-7, far below bf16 resolution); erf(h/sqrt 2) and the normal density share
// one exponential: e^{-z^2} with z = h/sqrt 2 is e^{-h^2/2}.
__device__ __forceinline__ void cdf_pdf(float h, float& cdf, float& pdf) {
  const float z = fabsf(h) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * z);
  const float ex = __expf(-z * z);
  const float poly = ((((1.061405429f * t - 1.453152027f) * t + 1.421413741f) * t - 0.284496736f) * t + 0.254829592f) * t;
  const float erf_abs = 1.0f - poly * ex;
  cdf = 0.5f * (1.0f + copysignf(erf_abs, h));
  pdf = 0.39894228040143268f * ex;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
#endif

// ---------------------------------------------------------------- GEMM
// C[m,n] = sum_k A(m,k) B(k,n), fp32 accumulation, element strides for both
// operands so that one routine covers Y = X W, dX = dY W^T and dW = X^T dY.
enum Epilogue : int {
  EPI_NONE = 0,   // C = acc (+bias) (+residual)
  // GELU of h = acc + bias: C2 = gelu(h) and C = gelu'(h), the factor the backward pass multiplies by (h itself is
  // needed nowhere else, and the forward has the normal CDF and density at hand anyway)
  EPI_GELU = 1,
  EPI_DGELU = 2   // C = acc * aux   (aux = the gelu'(h) saved by EPI_GELU)
};
struct GemmArgs {
  const void* A; int a_dt; long a_sm, a_sk;   // A(m,k) = A[m*a_sm + k*a_sk]
  const void* B; int b_dt; long b_sk, b_sn;   // B(k,n) = B[k*b_sk + n*b_sn]
  void* C; int c_dt; long ldc;                // row-major output
  int M, N, K;
  const float* bias;                          // [N] fp32 or null
  const void* residual; int r_dt; long ldr;   // [M,N] or null
  int epilogue;
  void* C2;                                   // EPI_GELU second output (c_dt, ldc)
  const void* aux; int aux_dt; long ldaux;    // EPI_DGELU: the saved GELU derivative
  float* splitk_ws; size_t splitk_floats;     // optional scratch for split-K partial sums
  float* colsum;                              // optional: out[n] = sum_k B(k,n) (bias gradient of a dW product);
                                              // honoured only by the MFMA kernel, see gemm_fuses_colsum()
};
int launch_gemm(hipStream_t s, const GemmArgs& g);          // picks the MFMA kernel when the shape allows
int launch_gemm_generic(hipStream_t s, const GemmArgs& g);
// Products with few output rows (the class-token rows of a pruned auxiliary layer): see k_gemm_rows.hip
bool gemm_rows_supported(const GemmArgs& g);
int launch_gemm_rows(hipStream_t s, const GemmArgs& g);
bool gemm_mfma_supported(const GemmArgs& g);
inline bool gemm_fuses_colsum(const GemmArgs& g) { return g.colsum && gemm_mfma_supported(g); }
size_t gemm_mfma_partial_floats(int M, int N, int K);
int launch_gemm_mfma(hipStream_t s, const GemmArgs& g, float* partial, size_t partial_floats);
bool gemm_mfma_groupable(const GemmArgs& g);
// every product must be groupable; ws (gemm_mfma_balanced_floats() floats or more), when given, lets the launch deal
// the k-steps out evenly over the compute units (parts of divided tiles pass through it)
int launch_gemm_mfma_grouped(hipStream_t s, const GemmArgs* gs, int n, float* ws = nullptr, size_t ws_floats = 0);
size_t gemm_mfma_balanced_floats();
// A set of independent products; one launch when all of them are groupable, else one by one.
// `one_launch`: take the grouped kernel whenever all products allow it, however few tiles they have
int launch_gemm_group(hipStream_t s, const GemmArgs* gs, int n, bool one_launch = false, bool use_workspace = false);
bool gemm_group_in_one_launch(const GemmArgs* gs, int n);   // every product fits the grouped kernel (n > 1)
// Per-launch timing of the contraction kernels (a measurement aid, off unless a block asks for it).  A block that
// times its launches binds its record to the calling thread for the duration of a step; the launch functions
// below the block engine then bracket each contraction launch with a pair of events on its stream.
// kind 0: GEMM over a token matrix (units = flops), 1: convolution (units = bytes), 2: GEMM with fewer than 256 output rows
// (the class-token products of the pruned auxiliary layer; units = flops)
struct TimedLaunch { hipEvent_t a, b; double units; int kind; };
struct LaunchTimes {
  std::vector<TimedLaunch> timed;
  std::vector<hipEvent_t> pool;
  double ms[3] = {0, 0, 0}, units[3] = {0, 0, 0};
  long long launches[3] = {0, 0, 0};
};
void profile_bind(LaunchTimes* t);     // null: launches of this thread are not timed
bool profile_enabled();                // a record is bound to this thread
int profile_begin(hipStream_t s, double units, void** token, int kind = 0);
int profile_end(hipStream_t s, void* token);
int profile_drain(LaunchTimes& t);     // waits for the recorded events and adds them to t.ms / t.units / t.launches
void profile_destroy(LaunchTimes& t);
int reduce_partials(hipStream_t s, const float* partial, int chunks, int N, long stride, float scale, float* out);

// Second stage of the two-stage (ordered, atomic-free) reductions.  A first-stage kernel asks for
// room for its partial sums: from the arena, if there is one with space left, and then the second
// stage is only queued and all queued ones run as one launch in flush() (parameter gradients are
// not needed before the optimizer update); otherwise from the shared scratch buffer, and the
// second stage runs at once.  The summation order is the same either way.
struct ReduceJob { const float* src; float* dst; int chunks, N; long stride; float scale; };
struct ReduceQueue {
  float* scratch = nullptr;            // shared by all reductions that finish at once
  float* arena = nullptr;              // private room for the queued ones, handed out front to back
  size_t arena_floats = 0, used = 0;
  std::vector<ReduceJob> jobs;
  float* space(size_t floats, bool* queued);
  int reduce(hipStream_t s, bool queued, const float* src, int chunks, int N, long stride, float scale, float* out);
  int flush(hipStream_t s);
  void reset() { used = 0; jobs.clear(); }
};
int colsum_mode(hipStream_t s, const void* x, int dt, int rows, int N, int mode, const float* shift, float scale,
                ReduceQueue& rq, float* out);

// ---------------------------------------------------------------- row-wise ops
int launch_layernorm_fwd(hipStream_t s, const void* x, int dt, long x_row_stride, int rows, int D,
                         const float* g, const float* b, float eps, void* y, float* mean, float* rstd);
// dx_out = dres + LN'(dy) (either may be null); partial sums of dg/db ([nchunks][2][D]) are
// reduced into dg, db through the queue.
int launch_layernorm_bwd(hipStream_t s, const void* dy, const void* x, int dt, long x_row_stride, int rows,
                         int D, const float* g, const float* mean, const float* rstd, const void* dres,
                         void* dx_out, ReduceQueue& rq, float* dg, float* db);
int layernorm_bwd_partial_floats(int rows, int D);

// out[n] = sum over rows of x[r, n]  (two-stage, deterministic)
int launch_colsum(hipStream_t s, const void* x, int dt, int rows, int N, ReduceQueue& rq, float* out);
int colsum_partial_floats(int rows, int N);

// mean softmax cross-entropy and its gradient; loss2 (optional) receives a copy of the loss, dbias (optional)
// the column sums of dlogits
int launch_cross_entropy(hipStream_t s, const float* logits, const int32_t* labels, int B, int C,
                         float* loss, float* loss2, float* dlogits, float* dbias, int* flag);

// ViT auxiliary head in one launch: z = LN(x[:, 0, :]), logits = z W + b, mean cross-entropy, and back to
// dcls = dL/dx[:, 0, :]; the batch sums (loss, dW, db, LayerNorm dg / db) go through the reduction queue.
size_t vit_head_partial_floats(int B, int D, int C);
bool vit_head_fused_ok(int D, int C);
int launch_vit_head(hipStream_t s, const void* x, int dt, long x_row_stride, int B, int D, int C, const float* ln_g,
                    const float* ln_b, float eps, const float* W, const float* bias, const int32_t* labels, void* dcls,
                    ReduceQueue& rq, float* d_ln_g, float* d_ln_b, float* dW, float* dbias, float* loss, float* loss2,
                    int* flag);

// ---------------------------------------------------------------- ViT pieces
int launch_patchify(hipStream_t s, const void* img, int dt, int B, int H, int W, int C, int P, void* patches);
int launch_assemble_tokens(hipStream_t s, const void* E, int dt, const float* cls, const float* pos, int B,
                           int T, int D, void* x0);
// dpos[t,d] = sum_b dx[b,t,d]; dcls[d] = dpos[0,d]; dE = dx[:,1:,:] gathered
int launch_embed_bwd(hipStream_t s, const void* dx, int dt, int B, int T, int D, ReduceQueue& rq, float* dpos,
                     float* dcls, void* dE);
int embed_bwd_partial_floats(int B, int T, int D);
// dx[b,0,:] = dcls[b,:], every other row 0
int launch_scatter_cls(hipStream_t s, const void* dcls, int dt, int B, int T, int D, void* dx);

int launch_attention_fwd(hipStream_t s, const void* qkv, int dt, int B, int T, int H, int dh, void* out,
                         float* lse);
int launch_attention_bwd(hipStream_t s, const void* qkv, const void* out, const void* dout, const float* lse,
                         int dt, int B, int T, int H, int dh, void* dqkv);
bool attention_mfma_supported(int dt, int T, int H, int dh, const void* a, const void* b, const void* c,
                              const void* d);
int launch_attention_fwd_mfma(hipStream_t s, const void* qkv, int B, int T, int H, void* out, float* lse);
int launch_attention_bwd_mfma(hipStream_t s, const void* qkv, const void* out, const void* dout, const float* lse,
                              int B, int T, int H, void* dqkv);
int launch_attention_fwd_generic(hipStream_t s, const void* qkv, int dt, int B, int T, int H, int dh, void* out,
                                 float* lse);
int launch_attention_bwd_generic(hipStream_t s, const void* qkv, const void* out, const void* dout,
                                 const float* lse, int dt, int B, int T, int H, int dh, void* dqkv);

// Attention of the class token's query alone against all keys and values of its (batch, head): q, out, dq, dout are
// [B, H*dh], kv and dkv [B*T, 2*H*dh] (keys then values), prob [B, H, T] fp32 (saved by the forward).
size_t attention_cls_lds_bytes(int T, int dh);
int launch_attention_cls_fwd(hipStream_t s, const void* q, const void* kv, int dt, int B, int T, int H, int dh, void* out,
                             float* prob);
int launch_attention_cls_bwd(hipStream_t s, const void* q, const void* kv, const float* prob, const void* dout, int dt, int B,
                             int T, int H, int dh, void* dq, void* dkv);
// dst[r * dst_stride + d] += src[r * D + d] for r < rows
int launch_add_rows(hipStream_t s, void* dst, long dst_stride, const void* src, int rows, int D, int dt);

// ---------------------------------------------------------------- optimizers
// `shadow` (nullable): bf16 copy of the updated parameters, same offsets
int launch_sgd(hipStream_t s, float* p, const float* g, float* buf, uint16_t* shadow, size_t n, float lr,
               float momentum, int nesterov, float wd, int first);
int launch_adamw(hipStream_t s, float* p, const float* g, float* m, float* v, uint16_t* shadow, size_t n, float lr,
                 float b1, float b2, float eps, float wd, float bias_corr1, float bias_corr2);
int launch_refresh_shadow(hipStream_t s, const float* p, uint16_t* shadow, size_t n);
int launch_fill_zero(hipStream_t s, void* p, size_t bytes);
int launch_copy_probe(hipStream_t s, const void* src, void* dst, size_t bytes);

// ---------------------------------------------------------------- ResNet pieces
// stat / stat_blocks (nullable): room for the sums a BatchNorm over y needs (bn_partial_floats of y's shape); on
// return *stat_blocks is the number of partial rows the convolution wrote there itself (0: none, the BatchNorm
// has to make its own pass)
int launch_conv3x3_fwd(hipStream_t s, const void* x, const void* w, int wdt, int dt, int B, int H, int W, int Ci,
                       int Co, int stride, void* y, float* stat = nullptr, int* stat_blocks = nullptr);
// dx = dgrad(dy, w) (+ dres * (ymask > 0) when dres != null)
// The BatchNorm whose output gradient a convolution's input gradient dx is: output y (ReLU mask), input x, saved
// statistics, and room for the partial sums of its backward pass (bn_partial_floats of its shape).
struct BnBwdSums { const void* y; const void* x; const float* mean; const float* rstd; float* partials; };
// bn / stat_blocks (nullable): on return *stat_blocks is the number of partial rows of that BatchNorm's two backward
// sums that the convolution wrote to bn->partials itself (0: none, launch_bn_bwd has to make its own pass)
int launch_conv3x3_dgrad(hipStream_t s, const void* dy, const void* w, int wdt, int dt, int B, int H, int W, int Ci,
                         int Co, int stride, const void* dres, const void* ymask, void* dx, const BnBwdSums* bn = nullptr,
                         int* stat_blocks = nullptr);
// dw [9][ci_keep][Co]: the gradient for the first ci_keep input channels (all of them by default; fewer when
// the caller padded x with zero channels)
int launch_conv3x3_wgrad(hipStream_t s, const void* x, const void* dy, int dt, int B, int H, int W, int Ci,
                         int Co, int stride, ReduceQueue& rq, float* dw, int ci_keep = -1);
// weight gradients of n convolutions of one shape (x [B,H,W,Ci], dy [B,Ho,Wo,Co] each): one launch where the
// matrix-core kernel takes the shape, else one launch per convolution
struct ConvWgradJob { const void* x; const void* dy; float* dw; };
int launch_conv3x3_wgrad_group(hipStream_t s, const ConvWgradJob* jobs, int n, int dt, int B, int H, int W, int Ci, int Co,
                               int stride, ReduceQueue& rq);
int launch_conv3x3_wgrad_group_bf16(hipStream_t s, const ConvWgradJob* jobs, int n, int B, int H, int W, int Ci, int Co,
                                    int stride, ReduceQueue& rq, bool* done);
// second stage of a convolution weight gradient: adds `rows` partial filters [9][Ci][Co] into dw [9][keep][Co]
int reduce_conv_filters(hipStream_t s, ReduceQueue& rq, bool queued, const float* partials, int rows, int Ci, int Co,
                        int keep, float* dw);
// x [P, c] -> y [P, 16] with zero channels appended (c < 16); w [9][c][Co] (fp32 master) -> wp [9][16][Co] bf16
int launch_pad_channels16(hipStream_t s, const void* x, size_t P, int c, void* y);
int launch_pad_filter16(hipStream_t s, const float* w, int c, int Co, void* wp);
int conv3x3_wgrad_partial_floats(int B, int H, int W, int Ci, int Co, int stride);
// shortcut of a downsampling basic block: y = every stride-th pixel of x [B,H,W,Ci] with Co - Ci zero channels
// appended; its transpose adds dy * (ymask > 0) into dx
int launch_shortcut_fwd(hipStream_t s, const void* x, int dt, int B, int H, int W, int Ci, int Co, int stride, void* y);
int launch_shortcut_bwd(hipStream_t s, const void* dy, const void* ymask, int dt, int B, int H, int W, int Ci, int Co,
                        int stride, void* dx);
// training-mode statistics over rows of x [rows, C]; also updates running stats
int launch_bn_stats(hipStream_t s, const void* x, int dt, int rows, int C, float eps, float momentum,
                    float* partials, float* mean, float* rstd, float* run_mean, float* run_var);
// statistics of x, running-statistics update and y = relu(bn(x) (+ res)): the BatchNorm of a training step
// ready_blocks: rows of `partials` the producing convolution has already filled (see launch_conv3x3_fwd), else 0
int launch_bn_train_fwd(hipStream_t s, const void* x, int dt, int rows, int C, float eps, float momentum, float* partials,
                        float* mean, float* rstd, float* run_mean, float* run_var, const float* g, const float* b,
                        const void* res, void* y, int ready_blocks = 0);
// y = relu(bn(x) (+ res))
int launch_bn_running_stats(hipStream_t s, const float* run_mean, const float* run_var, int C, float eps, float* mean,
                            float* rstd);
int launch_bn_apply(hipStream_t s, const void* x, int dt, int rows, int C, const float* mean, const float* rstd,
                    const float* g, const float* b, const void* res, void* y);
// dyh = dy * (y > 0); dx = bn'(dyh); dg = sum dyh*xhat; db = sum dyh
// ready_blocks: rows of `partials` the convolution that produced dy has already filled (see launch_conv3x3_dgrad), else 0
int launch_bn_bwd(hipStream_t s, const void* dy, const void* y, const void* x, int dt, int rows, int C,
                  const float* mean, const float* rstd, const float* g, float* partials, float* dg,
                  float* db, void* dx, int ready_blocks = 0);
int bn_partial_floats(int rows, int C);
// bf16 fast path (k_resnet_bf16.hip)
bool conv_bf16_supported(int dt, int wdt, int Ci, int Co, const void* a, const void* b, const void* c);
bool conv_pixels_fit(int B, int H, int W);
bool conv_fwd_bf16_ok(int Ci, int Co);
bool conv_dgrad_bf16_ok(int Ci, int Co);
bool conv_wgrad_bf16_ok(int Ci, int Co);
// stat (nullable): the kernel also writes per-workgroup per-channel sums of its stored outputs there
// ([*stat_blocks][2][Co] floats: what the BatchNorm behind the convolution reduces)
int launch_conv3x3_fwd_bf16(hipStream_t s, const void* x, const void* w, int B, int H, int W, int Ci, int Co,
                            int stride, void* y, float* stat = nullptr, int* stat_blocks = nullptr);
int launch_conv3x3_dgrad_bf16(hipStream_t s, const void* dy, const void* w, int B, int H, int W, int Ci, int Co,
                              int stride, const void* dres, const void* ymask, void* dx, const BnBwdSums* bn = nullptr,
                              int* stat_blocks = nullptr);
int launch_conv3x3_wgrad_bf16(hipStream_t s, const void* x, const void* dy, int B, int H, int W, int Ci, int Co,
                              int stride, ReduceQueue& rq, float* dw, int ci_keep);
size_t conv3x3_wgrad_bf16_partial_floats(int B, int H, int W, int Ci, int Co, int stride);
bool eltwise_bf16_ok(int dt, size_t elems, int C0, int C1, const void* a, const void* b, const void* c);
int launch_gap_bwd_bf16(hipStream_t s, const void* dpooled, int B, int HW, int C, void* dx);
bool gap_fwd_bf16_ok(int dt, int C, const void* x, const void* pooled);
int launch_gap_fwd_bf16(hipStream_t s, const void* x, int B, int HW, int C, void* pooled);
int launch_shortcut_fwd_bf16(hipStream_t s, const void* x, int B, int H, int W, int Ci, int Co, int stride, void* y);
int launch_shortcut_bwd_bf16(hipStream_t s, const void* dy, const void* ymask, int B, int H, int W, int Ci, int Co, int stride,
                             void* dx);
bool bn_bf16_supported(int dt, int rows, int C, const void* a, const void* b, const void* c, const void* d);
size_t bn_bf16_partial_floats(int rows, int C);
int launch_bn_stats_bf16(hipStream_t s, const void* x, int rows, int C, float eps, float momentum, float* partials,
                         float* mean, float* rstd, float* run_mean, float* run_var);
int launch_bn_train_fwd_bf16(hipStream_t s, const void* x, int rows, int C, float eps, float momentum, float* partials,
                             float* mean, float* rstd, float* run_mean, float* run_var, const float* g, const float* b,
                             const void* res, void* y, int ready_blocks = 0);
int launch_bn_apply_bf16(hipStream_t s, const void* x, int rows, int C, const float* mean, const float* rstd,
                         const float* g, const float* b, const void* res, void* y);
int launch_bn_bwd_bf16(hipStream_t s, const void* dy, const void* y, const void* x, int rows, int C, const float* mean,
                       const float* rstd, const float* g, float* partials, float* dg, float* db, void* dx, int ready_blocks = 0);
int launch_gap_fwd(hipStream_t s, const void* x, int dt, int B, int HW, int C, void* pooled);
int launch_gap_bwd(hipStream_t s, const void* dpooled, int dt, int B, int HW, int C, void* dx);

}  // namespace ppll
