// ResNet stage kernels (element type chosen at run time): direct 3x3
// convolution forward / input gradient / weight gradient on NHWC activations
// with [ky,kx,Cin,Cout] filters, training-mode BatchNorm (+ReLU, +skip) forward
// and backward, and global average pooling.  Reductions are two-stage and
// ordered, never atomic.
#include "common.h"

namespace ppll {

namespace {
__device__ __forceinline__ int out_dim(int in, int stride) { return (in - 1) / stride + 1; }   // pad 1, 3x3

// y[b,oy,ox,co] = sum_{ky,kx,ci} x[b, oy*s+ky-1, ox*s+kx-1, ci] w[ky,kx,ci,co]
__global__ __launch_bounds__(256) void conv3x3_fwd_kernel(const void* x, const void* w, int wdt, int dt, int B, int H,
                                                          int W, int Ci, int Co, int stride, void* y) {
  int Ho = out_dim(H, stride), Wo = out_dim(W, stride);
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)B * Ho * Wo * Co) return;
  int co = i % Co; size_t pix = i / Co;
  int ox = pix % Wo, oy = (pix / Wo) % Ho; int b = pix / ((size_t)Wo * Ho);
  float acc = 0.f;
  for (int ky = 0; ky < 3; ++ky) {
    int iy = oy * stride + ky - 1;
    if (iy < 0 || iy >= H) continue;
    for (int kx = 0; kx < 3; ++kx) {
      int ix = ox * stride + kx - 1;
      if (ix < 0 || ix >= W) continue;
      size_t xb = (((size_t)b * H + iy) * W + ix) * Ci;
      size_t wb = ((size_t)(ky * 3 + kx) * Ci) * Co + co;
      for (int ci = 0; ci < Ci; ++ci) acc = fmaf(ld_f(x, xb + ci, dt), ld_f(w, wb + (size_t)ci * Co, wdt), acc);
    }
  }
  st_f(y, i, acc, dt);
}

// dx[b,iy,ix,ci] = sum_{ky,kx,co} dy[b,oy,ox,co] w[ky,kx,ci,co] over the (oy,ox)
// with oy*s+ky-1 = iy, ox*s+kx-1 = ix; optionally + dres * (ymask > 0).
__global__ __launch_bounds__(256) void conv3x3_dgrad_kernel(const void* dy, const void* w, int wdt, int dt, int B, int H,
                                                            int W, int Ci, int Co, int stride, const void* dres,
                                                            const void* ymask, void* dx) {
  int Ho = out_dim(H, stride), Wo = out_dim(W, stride);
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)B * H * W * Ci) return;
  int ci = i % Ci; size_t pix = i / Ci;
  int ix = pix % W, iy = (pix / W) % H; int b = pix / ((size_t)W * H);
  float acc = 0.f;
  for (int ky = 0; ky < 3; ++ky) {
    int ty = iy + 1 - ky;
    if (ty < 0 || ty % stride) continue;
    int oy = ty / stride;
    if (oy >= Ho) continue;
    for (int kx = 0; kx < 3; ++kx) {
      int tx = ix + 1 - kx;
      if (tx < 0 || tx % stride) continue;
      int ox = tx / stride;
      if (ox >= Wo) continue;
      size_t yb = (((size_t)b * Ho + oy) * Wo + ox) * Co;
      size_t wb = ((size_t)(ky * 3 + kx) * Ci + ci) * Co;
      for (int co = 0; co < Co; ++co) acc = fmaf(ld_f(dy, yb + co, dt), ld_f(w, wb + co, wdt), acc);
    }
  }
  if (dres && ld_f(ymask, i, dt) > 0.f) acc += ld_f(dres, i, dt);
  st_f(dx, i, acc, dt);
}

// partial[chunk][tap,ci,co] = sum over the chunk's output pixels of x(...) dy(...)
constexpr int WG_PIX = 64;
__global__ __launch_bounds__(256) void conv3x3_wgrad_kernel(const void* x, const void* dy, int dt, int B, int H, int W,
                                                            int Ci, int Co, int stride, float* partial) {
  int Ho = out_dim(H, stride), Wo = out_dim(W, stride);
  size_t npix = (size_t)B * Ho * Wo;
  size_t p0 = (size_t)blockIdx.x * WG_PIX, p1 = min(npix, p0 + WG_PIX);
  int nw = 9 * Ci * Co;
  for (int e = threadIdx.x; e < nw; e += 256) {
    int co = e % Co, ci = (e / Co) % Ci, tap = e / (Co * Ci);
    int ky = tap / 3, kx = tap % 3;
    float acc = 0.f;
    for (size_t p = p0; p < p1; ++p) {
      int ox = p % Wo, oy = (p / Wo) % Ho; int b = p / ((size_t)Wo * Ho);
      int iy = oy * stride + ky - 1, ix = ox * stride + kx - 1;
      if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
      acc = fmaf(ld_f(x, (((size_t)b * H + iy) * W + ix) * Ci + ci, dt), ld_f(dy, p * Co + co, dt), acc);
    }
    partial[(size_t)blockIdx.x * nw + e] = acc;
  }
}

__global__ __launch_bounds__(256) void bn_finalize_kernel(const float* var_in, int C, int rows, float eps,
                                                          float momentum, const float* mean, float* rstd,
                                                          float* run_mean, float* run_var) {
  int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  float var = var_in[c];
  rstd[c] = 1.0f / sqrtf(var + eps);
  run_mean[c] = (1.f - momentum) * run_mean[c] + momentum * mean[c];
  run_var[c] = (1.f - momentum) * run_var[c] + momentum * var * ((float)rows / (float)(rows - 1));
}

__global__ __launch_bounds__(256) void bn_apply_kernel(const void* x, int dt, size_t total, int C, const float* mean,
                                                       const float* rstd, const float* g, const float* b,
                                                       const void* res, void* y) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  int c = i % C;
  float v = (ld_f(x, i, dt) - mean[c]) * rstd[c] * g[c] + b[c];
  if (res) v += ld_f(res, i, dt);
  st_f(y, i, fmaxf(v, 0.f), dt);
}

constexpr int BN_ROWS = 64;
// partial[chunk][0][c] = sum dyh, partial[chunk][1][c] = sum dyh*xhat, dyh = dy * (y > 0)
__global__ __launch_bounds__(256) void bn_bwd_partial_kernel(const void* dy, const void* y, const void* x, int dt,
                                                             int rows, int C, const float* mean, const float* rstd,
                                                             float* partial) {
  int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  int r0 = blockIdx.y * BN_ROWS, r1 = min(rows, r0 + BN_ROWS);
  float mu = mean[c], rs = rstd[c], s1 = 0.f, s2 = 0.f;
  for (int r = r0; r < r1; ++r) {
    size_t i = (size_t)r * C + c;
    float d = ld_f(y, i, dt) > 0.f ? ld_f(dy, i, dt) : 0.f;
    s1 += d;
    s2 += d * (ld_f(x, i, dt) - mu) * rs;
  }
  partial[((size_t)blockIdx.y * 2) * C + c] = s1;
  partial[((size_t)blockIdx.y * 2 + 1) * C + c] = s2;
}

// dx = (g rstd / N) (N dyh - sum dyh - xhat sum dyh*xhat); db = sum dyh, dg = sum dyh*xhat
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const void* dy, const void* y, const void* x, int dt,
                                                           size_t total, int C, int rows, const float* mean,
                                                           const float* rstd, const float* g, const float* dg,
                                                           const float* db, void* dx) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  int c = i % C;
  float d = ld_f(y, i, dt) > 0.f ? ld_f(dy, i, dt) : 0.f;
  float xh = (ld_f(x, i, dt) - mean[c]) * rstd[c];
  float n = (float)rows;
  st_f(dx, i, g[c] * rstd[c] / n * (n * d - db[c] - xh * dg[c]), dt);
}

__global__ __launch_bounds__(256) void gap_fwd_kernel(const void* x, int dt, int B, int HW, int C, void* pooled) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B * C) return;
  int c = i % C, b = i / C;
  float acc = 0.f;
  for (int p = 0; p < HW; p += 8) {   // eight loads in flight; added in pixel order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p + u < HW ? ld_f(x, ((size_t)b * HW + p + u) * C + c, dt) : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  st_f(pooled, i, acc / HW, dt);
}

// one workgroup per image; 256 / C thread groups split the pixels, and are added in group order
__global__ __launch_bounds__(256) void gap_fwd_image_kernel(const void* x, int dt, int HW, int C, void* pooled) {
  __shared__ float red[256];
  const int b = blockIdx.x, c = threadIdx.x % C, g = threadIdx.x / C, G = 256 / C;
  const int per = (HW + G - 1) / G, p0 = g * per, p1 = min(HW, p0 + per);
  float acc = 0.f;
  for (int p = p0; p < p1; p += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p + u < p1 ? ld_f(x, ((size_t)b * HW + p + u) * C + c, dt) : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (g == 0) {
    float t = 0.f;
    for (int k = 0; k < G; ++k) t += red[k * C + c];
    st_f(pooled, (size_t)b * C + c, t / HW, dt);
  }
}

__global__ __launch_bounds__(256) void gap_bwd_kernel(const void* dpooled, int dt, int B, int HW, int C, void* dx) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)B * HW * C) return;
  int c = i % C; int b = i / ((size_t)HW * C);
  st_f(dx, i, ld_f(dpooled, (size_t)b * C + c, dt) / HW, dt);
}

// Parameter-free shortcut of a basic block that shrinks the map and widens it (the CIFAR ResNet of
// Section 4.1): y[b,oy,ox,c] = x[b, oy*stride, ox*stride, c] for c < Ci, 0 for the appended channels.
__global__ __launch_bounds__(256) void shortcut_fwd_kernel(const void* x, int dt, int B, int H, int W, int Ci, int Co,
                                                           int stride, void* y) {
  int Ho = out_dim(H, stride), Wo = out_dim(W, stride);
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)B * Ho * Wo * Co) return;
  int c = i % Co; size_t pix = i / Co;
  int ox = pix % Wo, oy = (pix / Wo) % Ho; int b = pix / ((size_t)Wo * Ho);
  float v = c < Ci ? ld_f(x, (((size_t)b * H + oy * stride) * W + ox * stride) * Ci + c, dt) : 0.f;
  st_f(y, i, v, dt);
}

// Its transpose added into dx: dx[b, oy*stride, ox*stride, c] += dy[b,oy,ox,c] * (ymask[b,oy,ox,c] > 0), c < Ci.
// Every thread owns one element of dx.
__global__ __launch_bounds__(256) void shortcut_bwd_kernel(const void* dy, const void* ymask, int dt, int B, int H, int W,
                                                           int Ci, int Co, int stride, void* dx) {
  int Ho = out_dim(H, stride), Wo = out_dim(W, stride);
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)B * Ho * Wo * Ci) return;
  int c = i % Ci; size_t pix = i / Ci;
  int ox = pix % Wo, oy = (pix / Wo) % Ho; int b = pix / ((size_t)Wo * Ho);
  size_t yi = pix * Co + c;
  if (!(ld_f(ymask, yi, dt) > 0.f)) return;
  size_t xi = (((size_t)b * H + oy * stride) * W + ox * stride) * Ci + c;
  st_f(dx, xi, ld_f(dx, xi, dt) + ld_f(dy, yi, dt), dt);
}

// x [P, c] -> y [P, 16] bf16 with zero channels appended; one pixel per thread
__global__ __launch_bounds__(256) void pad_channels16_kernel(const uint16_t* x, size_t P, int c, uint16_t* y) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= P) return;
  uint16_t v[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = j < c ? x[i * c + j] : (uint16_t)0;
  uint4* out = reinterpret_cast<uint4*>(y + i * 16);
  out[0] = *reinterpret_cast<const uint4*>(v);
  out[1] = *reinterpret_cast<const uint4*>(v + 8);
}
// w [9][c][Co] fp32 -> wp [9][16][Co] bf16, zero rows appended
__global__ __launch_bounds__(256) void pad_filter16_kernel(const float* w, int c, int Co, uint16_t* wp) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 9 * 16 * Co) return;
  const int co = i % Co, ci = (i / Co) % 16, tap = i / (16 * Co);
  wp[i] = ci < c ? f32_to_bf16(w[((size_t)tap * c + ci) * Co + co]) : (uint16_t)0;
}
}  // namespace

int launch_pad_channels16(hipStream_t s, const void* x, size_t P, int c, void* y) {
  hipLaunchKernelGGL(pad_channels16_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, (const uint16_t*)x, P, c,
                     (uint16_t*)y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
int launch_pad_filter16(hipStream_t s, const float* w, int c, int Co, void* wp) {
  hipLaunchKernelGGL(pad_filter16_kernel, dim3((9 * 16 * Co + 255) / 256), dim3(256), 0, s, w, c, Co, (uint16_t*)wp);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_shortcut_fwd(hipStream_t s, const void* x, int dt, int B, int H, int W, int Ci, int Co, int stride, void* y) {
  if (eltwise_bf16_ok(dt, (size_t)B * H * W * Ci, Ci, Co, x, y, nullptr))
    return launch_shortcut_fwd_bf16(s, x, B, H, W, Ci, Co, stride, y);
  size_t total = (size_t)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1) * Co;
  hipLaunchKernelGGL(shortcut_fwd_kernel, dim3((total + 255) / 256), dim3(256), 0, s, x, dt, B, H, W, Ci, Co, stride, y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
int launch_shortcut_bwd(hipStream_t s, const void* dy, const void* ymask, int dt, int B, int H, int W, int Ci, int Co,
                        int stride, void* dx) {
  if (eltwise_bf16_ok(dt, (size_t)B * H * W * Ci, Ci, Co, dy, ymask, dx))
    return launch_shortcut_bwd_bf16(s, dy, ymask, B, H, W, Ci, Co, stride, dx);
  size_t total = (size_t)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1) * Ci;
  hipLaunchKernelGGL(shortcut_bwd_kernel, dim3((total + 255) / 256), dim3(256), 0, s, dy, ymask, dt, B, H, W, Ci, Co, stride,
                     dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_conv3x3_fwd(hipStream_t s, const void* x, const void* w, int wdt, int dt, int B, int H, int W, int Ci,
                       int Co, int stride, void* y, float* stat, int* stat_blocks) {
  if (stat_blocks) *stat_blocks = 0;
  if (conv_bf16_supported(dt, wdt, Ci, Co, x, w, y) && conv_fwd_bf16_ok(Ci, Co) && conv_pixels_fit(B, H, W)) {
    // the sums are only of use to the bf16 BatchNorm kernels (same partial layout); they refuse fewer than 2 rows
    const long rows = (long)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
    const bool want = stat && stat_blocks && rows >= 2 && bn_bf16_supported(dt, (int)rows, Co, y, nullptr, nullptr, nullptr);
    return launch_conv3x3_fwd_bf16(s, x, w, B, H, W, Ci, Co, stride, y, want ? stat : nullptr, stat_blocks);
  }
  size_t total = (size_t)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1) * Co;
  hipLaunchKernelGGL(conv3x3_fwd_kernel, dim3((total + 255) / 256), dim3(256), 0, s, x, w, wdt, dt, B, H, W, Ci, Co,
                     stride, y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_conv3x3_dgrad(hipStream_t s, const void* dy, const void* w, int wdt, int dt, int B, int H, int W, int Ci,
                         int Co, int stride, const void* dres, const void* ymask, void* dx, const BnBwdSums* bn,
                         int* stat_blocks) {
  if (stat_blocks) *stat_blocks = 0;
  if (conv_bf16_supported(dt, wdt, Ci, Co, dy, w, dx) && conv_dgrad_bf16_ok(Ci, Co) && conv_pixels_fit(B, H, W) && stride <= 2 &&
      !((((uintptr_t)dres) | ((uintptr_t)ymask)) & 15)) {
    // the sums are only of use to the bf16 BatchNorm kernels (same partial layout)
    const long rows = (long)B * H * W;
    const bool want = bn && stat_blocks && rows >= 2 && bn_bf16_supported(dt, (int)rows, Ci, dx, bn->y, bn->x, nullptr);
    return launch_conv3x3_dgrad_bf16(s, dy, w, B, H, W, Ci, Co, stride, dres, ymask, dx, want ? bn : nullptr, stat_blocks);
  }
  size_t total = (size_t)B * H * W * Ci;
  hipLaunchKernelGGL(conv3x3_dgrad_kernel, dim3((total + 255) / 256), dim3(256), 0, s, dy, w, wdt, dt, B, H, W, Ci,
                     Co, stride, dres, ymask, dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

static size_t wgrad_chunks(int B, int H, int W, int stride) {
  size_t npix = (size_t)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
  return (npix + WG_PIX - 1) / WG_PIX;
}
int conv3x3_wgrad_partial_floats(int B, int H, int W, int Ci, int Co, int stride) {
  size_t a = wgrad_chunks(B, H, W, stride) * 9 * Ci * Co, b = conv3x3_wgrad_bf16_partial_floats(B, H, W, Ci, Co, stride);
  return (int)(a > b ? a : b);
}
int reduce_conv_filters(hipStream_t s, ReduceQueue& rq, bool queued, const float* partials, int rows, int Ci, int Co,
                        int keep, float* dw) {
  const int nw = 9 * Ci * Co;
  if (keep == Ci) return rq.reduce(s, queued, partials, rows, nw, nw, 1.0f, dw);
  for (int tap = 0; tap < 9; ++tap)   // the leading `keep` input channels of every tap
    PPLL_TRY(rq.reduce(s, queued, partials + (size_t)tap * Ci * Co, rows, keep * Co, nw, 1.0f, dw + (size_t)tap * keep * Co));
  return PPLL_OK;
}

int launch_conv3x3_wgrad(hipStream_t s, const void* x, const void* dy, int dt, int B, int H, int W, int Ci, int Co,
                         int stride, ReduceQueue& rq, float* dw, int ci_keep) {
  if (ci_keep < 0 || ci_keep > Ci) ci_keep = Ci;
  if (conv_bf16_supported(dt, BF16, Ci, Co, x, dy, dw) && conv_wgrad_bf16_ok(Ci, Co) && conv_pixels_fit(B, H, W))
    return launch_conv3x3_wgrad_bf16(s, x, dy, B, H, W, Ci, Co, stride, rq, dw, ci_keep);
  int chunks = (int)wgrad_chunks(B, H, W, stride), nw = 9 * Ci * Co;
  bool queued;
  float* partials = rq.space((size_t)chunks * nw, &queued);
  hipLaunchKernelGGL(conv3x3_wgrad_kernel, dim3(chunks), dim3(256), 0, s, x, dy, dt, B, H, W, Ci, Co, stride, partials);
  PPLL_HIP(hipGetLastError());
  return reduce_conv_filters(s, rq, queued, partials, chunks, Ci, Co, ci_keep, dw);
}

int launch_conv3x3_wgrad_group(hipStream_t s, const ConvWgradJob* jobs, int n, int dt, int B, int H, int W, int Ci, int Co,
                               int stride, ReduceQueue& rq) {
  bool fast = conv_wgrad_bf16_ok(Ci, Co) && conv_pixels_fit(B, H, W);
  for (int j = 0; j < n && fast; ++j) fast = conv_bf16_supported(dt, BF16, Ci, Co, jobs[j].x, jobs[j].dy, jobs[j].dw);
  if (fast && n > 1) {
    bool done = false;
    PPLL_TRY(launch_conv3x3_wgrad_group_bf16(s, jobs, n, B, H, W, Ci, Co, stride, rq, &done));
    if (done) return PPLL_OK;
  }
  for (int j = 0; j < n; ++j) PPLL_TRY(launch_conv3x3_wgrad(s, jobs[j].x, jobs[j].dy, dt, B, H, W, Ci, Co, stride, rq, jobs[j].dw));
  return PPLL_OK;
}

int bn_partial_floats(int rows, int C) {
  int a = colsum_partial_floats(rows, C), b = ((rows + BN_ROWS - 1) / BN_ROWS) * 2 * C;
  int c = (C % 8 == 0 && C >= 8 && C <= 128 && 256 % (C / 8) == 0) ? (int)bn_bf16_partial_floats(rows, C) : 0;
  a = a > b ? a : b;
  return (a > c ? a : c) + C;
}

int launch_bn_stats(hipStream_t s, const void* x, int dt, int rows, int C, float eps, float momentum, float* partials,
                    float* mean, float* rstd, float* run_mean, float* run_var) {
  if (rows < 2) { set_error("batchnorm needs at least 2 rows per channel"); return PPLL_ERR_CONFIG; }
  if (bn_bf16_supported(dt, rows, C, x, nullptr, nullptr, nullptr))
    return launch_bn_stats_bf16(s, x, rows, C, eps, momentum, partials, mean, rstd, run_mean, run_var);
  float* var = partials;            // [C], then the chunk partials
  float* part = partials + C;
  ReduceQueue now;   // no arena: both reductions finish at once (the second one reads the first one's result)
  now.scratch = part;
  PPLL_TRY(colsum_mode(s, x, dt, rows, C, 0, nullptr, 1.0f / rows, now, mean));
  PPLL_TRY(colsum_mode(s, x, dt, rows, C, 1, mean, 1.0f / rows, now, var));
  hipLaunchKernelGGL(bn_finalize_kernel, dim3((C + 255) / 256), dim3(256), 0, s, var, C, rows, eps, momentum, mean, rstd,
                     run_mean, run_var);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_bn_train_fwd(hipStream_t s, const void* x, int dt, int rows, int C, float eps, float momentum, float* partials,
                        float* mean, float* rstd, float* run_mean, float* run_var, const float* g, const float* b,
                        const void* res, void* y, int ready_blocks) {
  if (rows >= 2 && bn_bf16_supported(dt, rows, C, x, res, y, nullptr))
    return launch_bn_train_fwd_bf16(s, x, rows, C, eps, momentum, partials, mean, rstd, run_mean, run_var, g, b, res, y,
                                    ready_blocks);
  PPLL_TRY(launch_bn_stats(s, x, dt, rows, C, eps, momentum, partials, mean, rstd, run_mean, run_var));
  return launch_bn_apply(s, x, dt, rows, C, mean, rstd, g, b, res, y);
}

int launch_bn_apply(hipStream_t s, const void* x, int dt, int rows, int C, const float* mean, const float* rstd,
                    const float* g, const float* b, const void* res, void* y) {
  if (bn_bf16_supported(dt, rows, C, x, res, y, nullptr))
    return launch_bn_apply_bf16(s, x, rows, C, mean, rstd, g, b, res, y);
  size_t total = (size_t)rows * C;
  hipLaunchKernelGGL(bn_apply_kernel, dim3((total + 255) / 256), dim3(256), 0, s, x, dt, total, C, mean, rstd, g, b, res, y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_bn_bwd(hipStream_t s, const void* dy, const void* y, const void* x, int dt, int rows, int C,
                  const float* mean, const float* rstd, const float* g, float* partials, float* dg,
                  float* db, void* dx, int ready_blocks) {
  if (bn_bf16_supported(dt, rows, C, dy, y, x, dx))
    return launch_bn_bwd_bf16(s, dy, y, x, rows, C, mean, rstd, g, partials, dg, db, dx, ready_blocks);
  int chunks = (rows + BN_ROWS - 1) / BN_ROWS;
  size_t total = (size_t)rows * C;
  hipLaunchKernelGGL(bn_bwd_partial_kernel, dim3((C + 255) / 256, chunks), dim3(256), 0, s, dy, y, x, dt, rows, C, mean,
                     rstd, partials);
  PPLL_HIP(hipGetLastError());
  PPLL_TRY(reduce_partials(s, partials, chunks, C, 2L * C, 1.0f, db));
  PPLL_TRY(reduce_partials(s, partials + C, chunks, C, 2L * C, 1.0f, dg));
  hipLaunchKernelGGL(bn_bwd_apply_kernel, dim3((total + 255) / 256), dim3(256), 0, s, dy, y, x, dt, total, C, rows, mean,
                     rstd, g, dg, db, dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

namespace {
__global__ __launch_bounds__(256) void bn_running_stats_kernel(const float* run_mean, const float* run_var, int C, float eps,
                                                               float* mean, float* rstd) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  mean[c] = run_mean[c];
  rstd[c] = 1.0f / sqrtf(run_var[c] + eps);
}
}  // namespace

// evaluation mode: the (mean, 1/sqrt(var + eps)) pair BatchNorm normalises with, from its running statistics
int launch_bn_running_stats(hipStream_t s, const float* run_mean, const float* run_var, int C, float eps, float* mean,
                            float* rstd) {
  hipLaunchKernelGGL(bn_running_stats_kernel, dim3((C + 255) / 256), dim3(256), 0, s, run_mean, run_var, C, eps, mean, rstd);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_gap_fwd(hipStream_t s, const void* x, int dt, int B, int HW, int C, void* pooled) {
  if (gap_fwd_bf16_ok(dt, C, x, pooled)) return launch_gap_fwd_bf16(s, x, B, HW, C, pooled);
  if (C <= 256 && 256 % C == 0)
    hipLaunchKernelGGL(gap_fwd_image_kernel, dim3(B), dim3(256), 0, s, x, dt, HW, C, pooled);
  else
    hipLaunchKernelGGL(gap_fwd_kernel, dim3((B * C + 255) / 256), dim3(256), 0, s, x, dt, B, HW, C, pooled);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
int launch_gap_bwd(hipStream_t s, const void* dpooled, int dt, int B, int HW, int C, void* dx) {
  if (eltwise_bf16_ok(dt, (size_t)B * HW * C, C, C, dpooled, dx, nullptr)) return launch_gap_bwd_bf16(s, dpooled, B, HW, C, dx);
  size_t total = (size_t)B * HW * C;
  hipLaunchKernelGGL(gap_bwd_kernel, dim3((total + 255) / 256), dim3(256), 0, s, dpooled, dt, B, HW, C, dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

}  // namespace ppll
