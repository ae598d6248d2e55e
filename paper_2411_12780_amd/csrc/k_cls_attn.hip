// Attention of one query per (batch, head): the class token's.  In the last encoder layer of an auxiliary network
// only the class-token row of the layer output is read (the head takes LayerNorm -> class token -> Linear), so of
// that layer's attention only the class token's query is needed, against the keys and values of all tokens.
// One workgroup per (batch, head); run-time typed (fp32 or bf16 tensors), fp32 arithmetic.
//   forward:   p = softmax_j(q . k_j / sqrt(dh)),  o = sum_j p_j v_j
//   backward:  dp_j = do . v_j,  ds_j = p_j (dp_j - sum_i p_i dp_i),  dq = sum_j ds_j k_j / sqrt(dh),
//              dk_j = ds_j q / sqrt(dh),  dv_j = p_j do
// Layouts: q, o, dq, do are [B, H*dh]; kv and dkv are [B*T, 2*H*dh] with the keys in the first H*dh columns.
#include "common.h"

namespace ppll {

namespace {
constexpr int CLS_THREADS = 256;
// K and V rows of one head staged in LDS as fp32, one padding float per row (lanes on different rows then hit
// different banks); all threads of the workgroup copy, eight independent loads in flight each
// VEC: bf16 tensors whose rows are multiples of 8 elements at 16-byte aligned addresses: one 16-byte load per 8 elements
template <bool VEC>
__device__ __forceinline__ void stage_head(const void* src, int dt, size_t first, long row_stride, int T, int dh, int tid,
                                           float* dst) {
  if (VEC) {
    const int gpr = dh >> 3, n = T * gpr;     // 16-byte granules per row, in all
    const uint16_t* p = (const uint16_t*)src + first;
#pragma unroll 4
    for (int i = tid; i < n; i += CLS_THREADS) {
      const int j = i / gpr, g = i - j * gpr;
      const uint4 w = *reinterpret_cast<const uint4*>(p + (size_t)j * row_stride + 8 * g);
      float* o = dst + j * (dh + 1) + 8 * g;
      o[0] = __uint_as_float(w.x << 16); o[1] = __uint_as_float(w.x & 0xffff0000u);
      o[2] = __uint_as_float(w.y << 16); o[3] = __uint_as_float(w.y & 0xffff0000u);
      o[4] = __uint_as_float(w.z << 16); o[5] = __uint_as_float(w.z & 0xffff0000u);
      o[6] = __uint_as_float(w.w << 16); o[7] = __uint_as_float(w.w & 0xffff0000u);
    }
    return;
  }
  const int n = T * dh;
#pragma unroll 8
  for (int i = tid; i < n; i += CLS_THREADS) {
    const int j = i / dh, d = i - j * dh;
    dst[j * (dh + 1) + d] = ld_f(src, first + (size_t)j * row_stride + d, dt);
  }
}
// sum / maximum over the workgroup through LDS (red: CLS_THREADS / 64 floats), same order for every thread
__device__ __forceinline__ float block_sum(float v, float* red, int tid) {
  v = wave_sum(v);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < CLS_THREADS / 64; ++w) t += red[w];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red, int tid) {
  v = wave_max(v);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int w = 1; w < CLS_THREADS / 64; ++w) t = fmaxf(t, red[w]);
  return t;
}

// one workgroup per (batch, head): a thread per token for the scores, a thread per feature for the output
template <bool VEC>
__global__ __launch_bounds__(CLS_THREADS) void attn_cls_fwd_kernel(const void* q, const void* kv, int dt, int T, int H, int dh,
                                                                   void* out, float* prob) {
  extern __shared__ float sm[];
  float* Ks = sm;                          // [T][dh + 1]
  float* Vs = Ks + (size_t)T * (dh + 1);   // [T][dh + 1]
  float* qs = Vs + (size_t)T * (dh + 1);   // [dh]
  float* ps = qs + dh;                     // [T]
  float* red = ps + T;                     // [4]
  const int b = blockIdx.x / H, h = blockIdx.x % H, D = H * dh, tid = threadIdx.x;
  const float scale = rsqrtf((float)dh);
  const size_t k0 = (size_t)b * T * 2 * D + (size_t)h * dh;   // key row of token 0; values D further
  stage_head<VEC>(kv, dt, k0, 2L * D, T, dh, tid, Ks);
  stage_head<VEC>(kv, dt, k0 + D, 2L * D, T, dh, tid, Vs);
  for (int d = tid; d < dh; d += CLS_THREADS) qs[d] = ld_f(q, (size_t)b * D + h * dh + d, dt) * scale;
  __syncthreads();
  float sc = -INFINITY;
  if (tid < T) {
    float s = 0.f;
    for (int d = 0; d < dh; ++d) s = fmaf(qs[d], Ks[tid * (dh + 1) + d], s);
    sc = s;
  }
  const float mx = block_max(sc, red, tid);
  const float e = tid < T ? __expf(sc - mx) : 0.f;
  const float sum = block_sum(e, red, tid);
  if (tid < T) { const float p = e / sum; ps[tid] = p; prob[(size_t)blockIdx.x * T + tid] = p; }
  __syncthreads();
  for (int d = tid; d < dh; d += CLS_THREADS) {
    float o = 0.f;
    for (int j = 0; j < T; ++j) o = fmaf(ps[j], Vs[j * (dh + 1) + d], o);
    st_f(out, (size_t)b * D + h * dh + d, o, dt);
  }
}

template <bool VEC>
__global__ __launch_bounds__(CLS_THREADS) void attn_cls_bwd_kernel(const void* q, const void* kv, const float* prob,
                                                                   const void* dout, int dt, int T, int H, int dh, void* dq,
                                                                   void* dkv) {
  extern __shared__ float sm[];
  float* Ks = sm;                          // [T][dh + 1]
  float* Vs = Ks + (size_t)T * (dh + 1);   // [T][dh + 1]
  float* dos = Vs + (size_t)T * (dh + 1);  // [dh]   (the forward's qs)
  float* ps = dos + dh;                    // [T]
  float* red = ps + T;                     // [4]
  float* ds = red + 4;                     // [T]
  float* qs = ds + T;                      // [dh]  scaled query
  const int b = blockIdx.x / H, h = blockIdx.x % H, D = H * dh, tid = threadIdx.x;
  const float scale = rsqrtf((float)dh);
  const size_t k0 = (size_t)b * T * 2 * D + (size_t)h * dh;
  stage_head<VEC>(kv, dt, k0, 2L * D, T, dh, tid, Ks);
  stage_head<VEC>(kv, dt, k0 + D, 2L * D, T, dh, tid, Vs);
  for (int d = tid; d < dh; d += CLS_THREADS) {
    dos[d] = ld_f(dout, (size_t)b * D + h * dh + d, dt);
    qs[d] = ld_f(q, (size_t)b * D + h * dh + d, dt) * scale;
  }
  __syncthreads();
  float p = 0.f, dp = 0.f;
  if (tid < T) {
    for (int d = 0; d < dh; ++d) dp = fmaf(dos[d], Vs[tid * (dh + 1) + d], dp);
    p = prob[(size_t)blockIdx.x * T + tid];
  }
  const float delta = block_sum(p * dp, red, tid);
  if (tid < T) { ps[tid] = p; ds[tid] = p * (dp - delta); }
  __syncthreads();
  for (int d = tid; d < dh; d += CLS_THREADS) {
    float acc = 0.f;
    for (int j = 0; j < T; ++j) acc = fmaf(ds[j], Ks[j * (dh + 1) + d], acc);
    st_f(dq, (size_t)b * D + h * dh + d, acc * scale, dt);
  }
  if (VEC) {
    const int gpr = dh >> 3, n = T * gpr;
    uint16_t* o = (uint16_t*)dkv + k0;
#pragma unroll 2
    for (int i = tid; i < n; i += CLS_THREADS) {
      const int j = i / gpr, d = 8 * (i - j * gpr);
      const float a = ds[j], c = ps[j];
      *reinterpret_cast<uint4*>(o + (size_t)j * 2 * D + d) =
          make_uint4(f32x2_to_bf16x2(a * qs[d], a * qs[d + 1]), f32x2_to_bf16x2(a * qs[d + 2], a * qs[d + 3]),
                     f32x2_to_bf16x2(a * qs[d + 4], a * qs[d + 5]), f32x2_to_bf16x2(a * qs[d + 6], a * qs[d + 7]));
      *reinterpret_cast<uint4*>(o + (size_t)j * 2 * D + D + d) =
          make_uint4(f32x2_to_bf16x2(c * dos[d], c * dos[d + 1]), f32x2_to_bf16x2(c * dos[d + 2], c * dos[d + 3]),
                     f32x2_to_bf16x2(c * dos[d + 4], c * dos[d + 5]), f32x2_to_bf16x2(c * dos[d + 6], c * dos[d + 7]));
    }
    return;
  }
  const int n = T * dh;
  for (int i = tid; i < n; i += CLS_THREADS) {
    const int j = i / dh, d = i - j * dh;
    const size_t kj = k0 + (size_t)j * 2 * D + d;
    st_f(dkv, kj, ds[j] * qs[d], dt);
    st_f(dkv, kj + D, ps[j] * dos[d], dt);
  }
}

// dst[r * dst_stride + d] += src[r * D + d]
__global__ __launch_bounds__(256) void add_rows_kernel(void* dst, long dst_stride, const void* src, int rows, int D, int dt) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)rows * D) return;
  const size_t r = i / D, d = i % D, o = r * dst_stride + d;
  st_f(dst, o, ld_f(dst, o, dt) + ld_f(src, i, dt), dt);
}

bool cls_vec_ok(int dt, int H, int dh, const void* a, const void* b) {
  return dt == BF16 && !(dh & 7) && !((((uintptr_t)a) | ((uintptr_t)b)) & 15) && H >= 1;
}
int opt_in_lds(const void* fn, size_t bytes, const char* what) {
  if (bytes > 160 * 1024) { set_error("%s: %zu bytes of LDS exceed 160 KB", what, bytes); return PPLL_ERR_CONFIG; }
  if (bytes > 64 * 1024) PPLL_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return PPLL_OK;
}
}  // namespace

size_t attention_cls_lds_bytes(int T, int dh) { return (2 * (size_t)T * (dh + 1) + 2 * (size_t)dh + 2 * (size_t)T + 4) * sizeof(float); }

int launch_attention_cls_fwd(hipStream_t s, const void* q, const void* kv, int dt, int B, int T, int H, int dh, void* out,
                             float* prob) {
  const size_t lds = attention_cls_lds_bytes(T, dh);
  if (cls_vec_ok(dt, H, dh, kv, nullptr)) {
    PPLL_TRY(opt_in_lds((const void*)attn_cls_fwd_kernel<true>, lds, "class-token attention"));
    hipLaunchKernelGGL(attn_cls_fwd_kernel<true>, dim3(B * H), dim3(CLS_THREADS), lds, s, q, kv, dt, T, H, dh, out, prob);
  } else {
    PPLL_TRY(opt_in_lds((const void*)attn_cls_fwd_kernel<false>, lds, "class-token attention"));
    hipLaunchKernelGGL(attn_cls_fwd_kernel<false>, dim3(B * H), dim3(CLS_THREADS), lds, s, q, kv, dt, T, H, dh, out, prob);
  }
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_attention_cls_bwd(hipStream_t s, const void* q, const void* kv, const float* prob, const void* dout, int dt, int B,
                             int T, int H, int dh, void* dq, void* dkv) {
  const size_t lds = attention_cls_lds_bytes(T, dh);
  if (cls_vec_ok(dt, H, dh, kv, dkv)) {
    PPLL_TRY(opt_in_lds((const void*)attn_cls_bwd_kernel<true>, lds, "class-token attention"));
    hipLaunchKernelGGL(attn_cls_bwd_kernel<true>, dim3(B * H), dim3(CLS_THREADS), lds, s, q, kv, prob, dout, dt, T, H, dh, dq, dkv);
  } else {
    PPLL_TRY(opt_in_lds((const void*)attn_cls_bwd_kernel<false>, lds, "class-token attention"));
    hipLaunchKernelGGL(attn_cls_bwd_kernel<false>, dim3(B * H), dim3(CLS_THREADS), lds, s, q, kv, prob, dout, dt, T, H, dh, dq, dkv);
  }
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_add_rows(hipStream_t s, void* dst, long dst_stride, const void* src, int rows, int D, int dt) {
  const size_t total = (size_t)rows * D;
  hipLaunchKernelGGL(add_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, dst, dst_stride, src, rows, D, dt);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

}  // namespace ppll
