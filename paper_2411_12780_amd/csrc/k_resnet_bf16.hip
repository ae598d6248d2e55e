// bf16 fast path of the ResNet blocks (channel counts 16, 32, 48, 64):
//  * 3x3 convolution forward and input gradient as an implicit GEMM on the
//    matrix cores: a lane owns one output pixel, reads its 3x3 neighbourhood
//    straight from the NHWC tensor in MFMA fragment order (8 consecutive
//    channels = 16 bytes), the filter sits in LDS (forward: as in memory, read
//    with transposing LDS reads; input gradient: [in channel][tap, out channel]);
//    the product is issued filter-first so that a lane ends up with 4 consecutive
//    output channels of its pixel (8-byte stores).
//  * weight gradient on the matrix cores with the output pixel as reduction index
//    (images transposed in LDS; stride 1 and 2, up to 16 convolutions of one shape per
//    launch); shapes it refuses: 64 output pixels per workgroup, their nine shifted
//    input vectors and dy staged in LDS, fp32 accumulators per thread.  Partial sums
//    per workgroup, added in a fixed order by the queued second stage.
//  * BatchNorm statistics / backward sums: 8 channels per thread (16-byte loads),
//    per-workgroup partials, added in workgroup order either by a one-workgroup launch
//    or, on small tensors, by every workgroup of the kernel that applies them (a
//    last-arrival scheme in one launch was slower: device-scope fences cost more).
//  * the elementwise pieces: shortcut of a downsampling block, global average pooling.
#include "common.h"

namespace ppll {

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float lo_bf(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack2(float a, float b) { return f32x2_to_bf16x2(a, b); }
__device__ __forceinline__ int out_dim(int in, int stride) { return (in - 1) / stride + 1; }

// Raw buffer access: a load whose byte offset lies beyond the buffer returns 0, so a tap outside the image needs
// no branch, only the offset CONV_OOB (buffers here stay below 2^30 bytes, checked by the launcher).
typedef __attribute__((ext_vector_type(4))) uint32_t conv_u32x4;
constexpr int CONV_OOB = 0x7fffffff;
__device__ __forceinline__ uint4 conv_buf_load16(__amdgpu_buffer_rsrc_t r, int off) {
  const conv_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Transposing LDS read of 16-bit elements: lane r of a 16-lane group hands in the address of 4 elements and receives
// element r % 4 from the addresses of lanes r / 4, r / 4 + 4, r / 4 + 8, r / 4 + 12 of its group.
typedef __attribute__((ext_vector_type(4))) short conv_s16x4;
__device__ __forceinline__ uint2 conv_lds_read_tr(const char* p) {
  const conv_s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) conv_s16x4*)p);
  return __builtin_bit_cast(uint2, v);
}

struct ConvArgs {
  const uint16_t* src;     // forward: x [B,H,W,Ci]; input gradient: dy [B,Ho,Wo,Co]
  const uint16_t* w;       // [9][Ci][Co]
  uint16_t* dst;           // forward: y [B,Ho,Wo,Co]; input gradient: dx [B,H,W,Ci]
  int B, H, W, Ci, Co, stride;
  const uint16_t* dres;    // input gradient only: dx += dres * (ymask > 0)
  const uint16_t* ymask;
  float* stat;             // STAT: [workgroups][2][channels produced] partial sums for the BatchNorm next in line:
                           //  forward: sum and sum of squares of the stored outputs;
                           //  input gradient: the two backward sums of the BatchNorm whose output gradient dx is
                           //  (sum dyh, sum dyh * xhat with dyh = dx * (bn_y > 0), xhat = (bn_x - bn_mean) * bn_rstd)
  const uint16_t* bn_y; const uint16_t* bn_x; const float* bn_mean; const float* bn_rstd;
};

// One halving step of a butterfly sum over lanes `step` apart: of the N values a lane holds, it keeps one half
// (the upper one if `up`), hands the other to its partner and adds what the partner hands over.
template <int N>
__device__ __forceinline__ void butterfly_halve(float* v, bool up, int step) {
#pragma unroll
  for (int i = 0; i < N / 2; ++i) {
    const float send = up ? v[i] : v[i + N / 2], keep = up ? v[i + N / 2] : v[i];
    v[i] = keep + __shfl_xor(send, step, 64);
  }
}
// Sums NV (16 or 32) per-lane values over the 32 lanes of a half-wave in a fixed order: afterwards v[0] of lane li holds
// the total of value index li >> 1 (NV = 16) or li (NV = 32).
template <int NV>
__device__ __forceinline__ void halfwave_sums(float (&v)[NV], int li) {
  static_assert(NV == 16 || NV == 32, "16 or 32 values per lane");
  if (NV == 32) {
    butterfly_halve<32>(v, (li & 16) != 0, 16);
    butterfly_halve<16>(v, (li & 8) != 0, 8);
    butterfly_halve<8>(v, (li & 4) != 0, 4);
    butterfly_halve<4>(v, (li & 2) != 0, 2);
    butterfly_halve<2>(v, (li & 1) != 0, 1);
  } else {
    butterfly_halve<16>(v, (li & 16) != 0, 16);
    butterfly_halve<8>(v, (li & 8) != 0, 8);
    butterfly_halve<4>(v, (li & 4) != 0, 4);
    butterfly_halve<2>(v, (li & 2) != 0, 2);
    v[0] += __shfl_xor(v[0], 1, 64);
  }
}
// the forward convolution sums its outputs for the BatchNorm behind it up to this many workgroups; the input gradient
// the backward sums of the BatchNorm before it up to fewer (at 512, 1024 x 8 x 8 x 64, it measured 5 % of the step slower)
constexpr long CONV_STAT_MAX_BLOCKS = 512, CONV_BWD_STAT_MAX_BLOCKS = 256;
constexpr int CONV_STAT_LDS = 4 * 2 * 2 * 32 * 4;   // [wave][sum kind][lane half][32] floats behind the filter

// MODE 0: forward.  MODE 1: input gradient.  NO = channels produced, KC = 16 * K16 channels reduced.
// GRP: how many of a pixel's nine tap loads are issued before the first product waits for one
// (0: one, 1: the three of a filter row, 3: all nine; a filter row measured best).
// LIN (forward, and input gradient at stride 1): a tap's source is the centre pixel's plus a constant,
// so a tap costs one offset addition and one select between that offset and "out of range".
// STAT (forward): the workgroup also writes the per-channel sum and sum of squares of the values it stored (as
// stored: after rounding to bf16), which is what the BatchNorm behind the convolution needs of its input; the sums
// run per lane over the workgroup's tiles, then over the lanes of a half-wave, then over the four waves.
template <int MODE, int K16, int NT, int GRP, bool LIN, bool STAT>
__global__ __launch_bounds__(256) void conv3x3_mfma_kernel(ConvArgs p) {
  // The filter in LDS.  Input gradient: [produced channel ci][tap, co] with rows RSW bytes apart (co, the reduced
  // index, is the contiguous one in memory: a fragment is one 16-byte read).  Forward: as in memory, [tap, ci][co]
  // with rows of PB bytes (the produced channels rounded up to 32); a fragment, 8 consecutive (tap, ci) of one co,
  // comes out of two transposing LDS reads.
  extern __shared__ __align__(16) char wl[];
  constexpr int KC = 16 * K16;
  const int NO = MODE == 0 ? p.Co : p.Ci;
  constexpr int RSW = 18 * KC + 16;
  const int PB = (NO + 31) / 32 * 64;
  const int Ho = out_dim(p.H, p.stride), Wo = out_dim(p.W, p.stride);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, hh = lane >> 5;
  // filter -> LDS; 8 output channels per 16-byte load, four loads in flight per thread
  {
    const int nvec = 9 * p.Ci * p.Co / 8;
    for (int v0 = tid; v0 < nvec; v0 += 4 * 256) {
      uint4 wv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int v = v0 + 256 * u;
        wv[u] = make_uint4(0, 0, 0, 0);
        if (v < nvec) wv[u] = *reinterpret_cast<const uint4*>(p.w + (size_t)v * 8);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int v = v0 + 256 * u;
        if (v >= nvec) break;
        const int e = v * 8, co = e % p.Co, ci = (e / p.Co) % p.Ci, tap = e / (p.Co * p.Ci);
        if (MODE == 0) {       // row (tap, ci), 8 consecutive co: a plain copy
          *reinterpret_cast<uint4*>(wl + (tap * KC + ci) * PB + 2 * co) = wv[u];
        } else {               // one row (ci), 8 consecutive k
          *reinterpret_cast<uint4*>(wl + ci * RSW + 2 * (tap * KC + co)) = wv[u];
        }
      }
    }
  }
  __syncthreads();
  // forward: lane part of a fragment address: (tap, ci) row 8 (lane/32) + (lane%16)/4, co 16 ((lane/16)%2) + 4 (lane%4)
  const int tr_lane = (8 * hh + ((lane & 15) >> 2)) * PB + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
  const int OH = MODE == 0 ? Ho : p.H, OW = MODE == 0 ? Wo : p.W;      // output spatial size
  const int SH = MODE == 0 ? p.H : Ho, SW = MODE == 0 ? p.W : Wo;      // source spatial size
  const long P = (long)p.B * OH * OW, ntiles = (P + 127) / 128;
  // NT = tiles of 32 produced channels (NO = 16: the upper half of the one tile is never stored)
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.src), 0, (int)((long)p.B * SH * SW * KC * 2), 0x00020000);
  constexpr int NV = NT * 16;
  float st0[STAT ? NV : 1], st1[STAT ? NV : 1];
  if (STAT) {
#pragma unroll
    for (int j = 0; j < NV; ++j) { st0[j] = 0.f; st1[j] = 0.f; }
  }
  // the workgroup keeps its filter for several tiles of 128 pixels
  for (long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    // 32-bit index arithmetic (the launcher checks that the pixel count fits): 64-bit division costs more than the tile
    const uint32_t pix = (uint32_t)tile * 128 + wave * 32 + li;
    const bool live = pix < (uint32_t)P;
    const uint32_t prow = pix / (uint32_t)OW;
    const int ox = (int)(pix - prow * (uint32_t)OW), oy = (int)(prow % (uint32_t)OH), b = (int)(prow / (uint32_t)OH);
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    constexpr int NG = GRP == 0 ? 9 : (GRP == 1 ? 3 : 1), TG = 9 / NG;   // groups of taps whose loads are in flight together
    // LIN: centre source pixel (cy, cx); tap (ky, kx) reads (cy + sg (ky-1), cx + sg (kx-1)), sg = +1 forward, -1 gradient
    const int sg = MODE == 0 ? 1 : -1;
    const int cy = MODE == 0 ? oy * p.stride : oy, cx = MODE == 0 ? ox * p.stride : ox;
    const int base = (((b * SH + cy) * SW + cx) * KC + 8 * hh) * 2;
    bool rowok[3], colok[3];
#pragma unroll
    for (int d = 0; d < 3; ++d) {
      rowok[d] = live && (unsigned)(cy + sg * (d - 1)) < (unsigned)SH;
      colok[d] = (unsigned)(cx + sg * (d - 1)) < (unsigned)SW;
    }
    auto tap_load = [&](const int grp, uint4 (&xv)[TG][K16]) {
#pragma unroll
      for (int j = 0; j < TG; ++j) {
        const int tap = grp * TG + j, ky = tap / 3, kx = tap % 3;
        if (LIN) {
          // ky is uniform (GRP = 1: ky = grp, kx = j): the row test is picked with scalar selects
          const bool ok = (ky == 0 ? rowok[0] : (ky == 1 ? rowok[1] : rowok[2])) && (kx == 0 ? colok[0] : (kx == 1 ? colok[1] : colok[2]));
          const int off = base + sg * (((ky - 1) * SW + (kx - 1)) * KC * 2);
#pragma unroll
          for (int c16 = 0; c16 < K16; ++c16) xv[j][c16] = conv_buf_load16(rsrc, ok ? off + 32 * c16 : CONV_OOB);
        } else {
          int sy, sx;
          bool ok = live;
          if (MODE == 0) {
            sy = oy * p.stride + ky - 1; sx = ox * p.stride + kx - 1;
          } else {
            // stride is 1 or 2 (checked by the launcher): mask and shift instead of a division per tap
            const int ty = oy + 1 - ky, tx = ox + 1 - kx, sm1 = p.stride - 1;
            ok = ok && ty >= 0 && tx >= 0 && !((ty | tx) & sm1);
            sy = ty >> sm1; sx = tx >> sm1;
          }
          ok = ok && sy >= 0 && sy < SH && sx >= 0 && sx < SW;
          const uint16_t* sp = p.src + (((long)b * SH + sy) * SW + sx) * KC + 8 * hh;
#pragma unroll
          for (int c16 = 0; c16 < K16; ++c16) {
            xv[j][c16] = make_uint4(0, 0, 0, 0);
            if (ok) xv[j][c16] = *reinterpret_cast<const uint4*>(sp + 16 * c16);
          }
        }
      }
    };
    auto tap_mma = [&](const int grp, const uint4 (&xv)[TG][K16]) {
#pragma unroll
      for (int j = 0; j < TG; ++j) {
        const int tap = grp * TG + j;
        const char* wrow = wl + 2 * (tap * KC + 8 * hh);
#pragma unroll
        for (int c16 = 0; c16 < K16; ++c16) {
          const bf16x8 xf = __builtin_bit_cast(bf16x8, xv[j][c16]);
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            bf16x8 wf;
            if (MODE == 0) {
              const char* fp = wl + tr_lane + (tap * KC + 16 * c16) * PB + 64 * t;
              const uint2 lo = conv_lds_read_tr(fp), hi = conv_lds_read_tr(fp + 4 * PB);
              wf = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
            } else {
              wf = *reinterpret_cast<const bf16x8*>(wrow + (t * 32 + li) * RSW + 32 * c16);
            }
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[t], 0, 0, 0);
          }
        }
      }
    };
    // Up to 32 reduced channels: the loads of a tap group are in flight while the group before it is multiplied (two
    // register sets); with three groups of three taps (GRP = 1) that leaves one load latency per tile exposed instead
    // of three (7.1 -> 6.4 us for the 32 -> 32 forward at 128 x 16 x 16).  With 48 or 64 reduced channels the second
    // register set (96 registers at 64 channels) spills, and the rolled loop over the groups measured faster
    // (0.92 against 0.97 ms per step at the 8 x 8 stage of ResNet-32).
    if constexpr (NG == 3 && K16 <= 2) {
      uint4 xa[TG][K16], xb[TG][K16];
      tap_load(0, xa);
      tap_load(1, xb);
      tap_mma(0, xa);
      tap_load(2, xa);
      tap_mma(1, xb);
      tap_mma(2, xa);
    } else {
#pragma unroll 1
      for (int grp = 0; grp < NG; ++grp) {
        uint4 xv[TG][K16];
        tap_load(grp, xv);
        tap_mma(grp, xv);
      }
    }
    if (!live) continue;
    // acc[t][4q+e] = out[pix][32t + 8q + 4hh + e]
    uint16_t* drow = p.dst + (size_t)pix * NO;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = 32 * t + 8 * q + 4 * hh;
          if (c >= NO) continue;
          float v[4] = {acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
          if (MODE == 1 && p.dres) {
            const uint2 m = *reinterpret_cast<const uint2*>(p.ymask + (size_t)pix * NO + c);
            const uint2 r = *reinterpret_cast<const uint2*>(p.dres + (size_t)pix * NO + c);
            if (lo_bf(m.x) > 0.f) v[0] += lo_bf(r.x);
            if (hi_bf(m.x) > 0.f) v[1] += hi_bf(r.x);
            if (lo_bf(m.y) > 0.f) v[2] += lo_bf(r.y);
            if (hi_bf(m.y) > 0.f) v[3] += hi_bf(r.y);
          }
          const uint2 o = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
          *reinterpret_cast<uint2*>(drow + c) = o;
          if (STAT) {
            const float r[4] = {lo_bf(o.x), hi_bf(o.x), lo_bf(o.y), hi_bf(o.y)};
            if (MODE == 0) {
#pragma unroll
              for (int e = 0; e < 4; ++e) { st0[16 * t + 4 * q + e] += r[e]; st1[16 * t + 4 * q + e] += r[e] * r[e]; }
            } else {
              const uint2 by = *reinterpret_cast<const uint2*>(p.bn_y + (size_t)pix * NO + c);
              const uint2 bx = *reinterpret_cast<const uint2*>(p.bn_x + (size_t)pix * NO + c);
              const float4 mu = *reinterpret_cast<const float4*>(p.bn_mean + c), rs = *reinterpret_cast<const float4*>(p.bn_rstd + c);
              const float yv[4] = {lo_bf(by.x), hi_bf(by.x), lo_bf(by.y), hi_bf(by.y)};
              const float xv[4] = {lo_bf(bx.x), hi_bf(bx.x), lo_bf(bx.y), hi_bf(bx.y)};
              const float mv[4] = {mu.x, mu.y, mu.z, mu.w}, rv[4] = {rs.x, rs.y, rs.z, rs.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const float d = yv[e] > 0.f ? r[e] : 0.f;
                st0[16 * t + 4 * q + e] += d;
                st1[16 * t + 4 * q + e] += d * (xv[e] - mv[e]) * rv[e];
              }
            }
          }
        }
      }
  }
  if constexpr (STAT) {
    // value index j = 16 t + 4 q + e of lane half hh is channel 32 t + 8 q + 4 hh + e
    float* red = reinterpret_cast<float*>(wl + (size_t)((NO + 31) / 32 * 32) * RSW);
    halfwave_sums<NV>(st0, li);
    halfwave_sums<NV>(st1, li);
    if (NV == 32 || !(li & 1)) {
      const int j = NV == 32 ? li : li >> 1;
      red[((wave * 2 + 0) * 2 + hh) * 32 + j] = st0[0];
      red[((wave * 2 + 1) * 2 + hh) * 32 + j] = st1[0];
    }
    __syncthreads();
    if (tid < 2 * NO) {
      const int which = tid / NO, c = tid % NO, j = 16 * (c >> 5) + 4 * ((c & 31) >> 3) + (c & 3), h2 = (c & 7) >> 2;
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) tot += red[((w * 2 + which) * 2 + h2) * 32 + j];
      p.stat[(size_t)blockIdx.x * 2 * NO + tid] = tot;
    }
  }
}

// Input gradient at stride 2 (H and W even, no fused shortcut gradient).  An input pixel (y, x) receives from
// the taps ky with (y + 1 - ky) even only: one tap per axis for even y (ky = 1), two for odd y (ky = 0, 2).  The
// pixels are therefore taken class by class (y parity, x parity): a tile of 128 pixels is of one class, and
// its 1, 2 or 4 live taps are the only ones loaded and multiplied (2.25 on average instead of 9).
template <int K16, int NT>
__global__ __launch_bounds__(256) void conv3x3_dgrad_s2_kernel(ConvArgs p) {
  extern __shared__ __align__(16) char wl[];        // [Ci rounded up to 32][9*Co] bf16, row stride RSW bytes
  constexpr int KC = 16 * K16, RSW = 18 * KC + 16;
  const int NO = p.Ci;
  const int Ho = p.H / 2, Wo = p.W / 2;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, hh = lane >> 5;
  {
    const int nvec = 9 * p.Ci * p.Co / 8;           // the filter row of an input channel: 8 consecutive output channels per copy
    for (int v = tid; v < nvec; v += 256) {
      const int e = v * 8, co = e % p.Co, ci = (e / p.Co) % p.Ci, tap = e / (p.Co * p.Ci);
      *reinterpret_cast<uint4*>(wl + ci * RSW + 2 * (tap * KC + co)) = *reinterpret_cast<const uint4*>(p.w + (size_t)v * 8);
    }
  }
  __syncthreads();
  const uint32_t Pc = (uint32_t)p.B * Ho * Wo, tpc = (Pc + 127) / 128;    // pixels and tiles per class
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.src), 0, (int)(Pc * KC * 2), 0x00020000);
  for (uint32_t tile = blockIdx.x; tile < 4 * tpc; tile += gridDim.x) {
    const int cls = (int)(tile / tpc), cy = cls >> 1, cx = cls & 1;
    const uint32_t q = (tile - cls * tpc) * 128 + wave * 32 + li;
    const bool live = q < Pc;
    const uint32_t qrow = q / (uint32_t)Wo;
    const int hx = (int)(q - qrow * (uint32_t)Wo), hy = (int)(qrow % (uint32_t)Ho), b = (int)(qrow / (uint32_t)Ho);
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    const int base = (((b * Ho + hy) * Wo + hx) * KC + 8 * hh) * 2;
    // axis parity 0: tap 1 reads source hy; parity 1: tap 0 reads hy + 1, tap 2 reads hy
#pragma unroll
    for (int iy = 0; iy < 2; ++iy) {
      if (iy > cy) break;
      const int ky = cy ? 2 * iy : 1, dy = (cy && iy == 0) ? 1 : 0;
#pragma unroll
      for (int ix = 0; ix < 2; ++ix) {
        if (ix > cx) break;
        const int kx = cx ? 2 * ix : 1, dx = (cx && ix == 0) ? 1 : 0;
        const bool ok = live && hy + dy < Ho && hx + dx < Wo;
        const int off = base + ((dy * Wo + dx) * KC) * 2;
        uint4 xv[K16];
#pragma unroll
        for (int c16 = 0; c16 < K16; ++c16) xv[c16] = conv_buf_load16(rsrc, ok ? off + 32 * c16 : CONV_OOB);
        const char* wrow = wl + 2 * ((ky * 3 + kx) * KC + 8 * hh);
#pragma unroll
        for (int c16 = 0; c16 < K16; ++c16) {
          const bf16x8 xf = __builtin_bit_cast(bf16x8, xv[c16]);
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const bf16x8 wf = *reinterpret_cast<const bf16x8*>(wrow + (t * 32 + li) * RSW + 32 * c16);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[t], 0, 0, 0);
          }
        }
      }
    }
    if (!live) continue;
    uint16_t* drow = p.dst + ((size_t)(b * p.H + 2 * hy + cy) * p.W + 2 * hx + cx) * NO;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int qq = 0; qq < 4; ++qq) {
        const int c = 32 * t + 8 * qq + 4 * hh;
        if (c >= NO) continue;
        *reinterpret_cast<uint2*>(drow + c) = make_uint2(pack2(acc[t][4 * qq], acc[t][4 * qq + 1]), pack2(acc[t][4 * qq + 2], acc[t][4 * qq + 3]));
      }
    }
  }
}

// Weight gradient.  CO = 32 or 64.  Thread (co = tid % CO, cig = tid / CO) owns
// dw[tap][cig*CPT .. +CPT-1][co], CPT = Ci / (256 / CO) input channels.
constexpr int WG_PIX_F = 64;
template <int CO, int CPT>
__global__ __launch_bounds__(256) void conv3x3_wgrad_bf16_kernel(const uint16_t* __restrict__ x,
                                                                 const uint16_t* __restrict__ dy, int B, int H, int W,
                                                                 int Ci, int stride, float* __restrict__ partial) {
  extern __shared__ __align__(16) char sm[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(sm);                 // [pixels][9][Ci]
  uint16_t* dys = xs + WG_PIX_F * 9 * Ci;                         // [pixels][CO]
  const int Ho = out_dim(H, stride), Wo = out_dim(W, stride);
  const long P = (long)B * Ho * Wo, p0 = (long)blockIdx.x * WG_PIX_F;
  const int tid = threadIdx.x;
  const int cpc = Ci / 8;                                         // 16-byte chunks per pixel vector
  for (int item = tid; item < WG_PIX_F * 9 * cpc; item += 256) {
    const int ch = item % cpc, tap = (item / cpc) % 9, lp = item / (cpc * 9);
    const long pp = p0 + lp;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (pp < P) {
      const uint32_t p32 = (uint32_t)pp, prow = p32 / (uint32_t)Wo;   // the launcher checks that the pixel count fits
      const int ox = (int)(p32 - prow * (uint32_t)Wo), oy = (int)(prow % (uint32_t)Ho), b = (int)(prow / (uint32_t)Ho);
      const int iy = oy * stride + tap / 3 - 1, ix = ox * stride + tap % 3 - 1;
      if (iy >= 0 && iy < H && ix >= 0 && ix < W)
        v = *reinterpret_cast<const uint4*>(x + (((long)b * H + iy) * W + ix) * Ci + 8 * ch);
    }
    *reinterpret_cast<uint4*>(xs + ((size_t)lp * 9 + tap) * Ci + 8 * ch) = v;
  }
  for (int item = tid; item < WG_PIX_F * (CO / 8); item += 256) {
    const int ch = item % (CO / 8), lp = item / (CO / 8);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (p0 + lp < P) v = *reinterpret_cast<const uint4*>(dy + (p0 + lp) * CO + 8 * ch);
    *reinterpret_cast<uint4*>(dys + (size_t)lp * CO + 8 * ch) = v;
  }
  __syncthreads();
  const int co = tid % CO, cig = tid / CO;
  float acc[9][CPT];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int j = 0; j < CPT; ++j) acc[t][j] = 0.f;
#pragma unroll 2
  for (int lp = 0; lp < WG_PIX_F; ++lp) {
    const float d = bf16_to_f32(dys[(size_t)lp * CO + co]);
    const uint16_t* xp = xs + (size_t)lp * 9 * Ci + cig * CPT;
    if constexpr (CPT == 1) {      // one input channel per thread: nine 16-bit reads
      uint16_t x1[9];
#pragma unroll
      for (int t = 0; t < 9; ++t) x1[t] = xp[t * Ci];
#pragma unroll
      for (int t = 0; t < 9; ++t) acc[t][0] = fmaf(bf16_to_f32(x1[t]), d, acc[t][0]);
    } else {
      uint32_t xv[9][CPT / 2];
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const uint32_t* xw = reinterpret_cast<const uint32_t*>(xp + t * Ci);
#pragma unroll
        for (int j = 0; j < CPT / 2; ++j) xv[t][j] = xw[j];
      }
#pragma unroll
      for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int j = 0; j < CPT / 2; ++j) {
          acc[t][2 * j] = fmaf(lo_bf(xv[t][j]), d, acc[t][2 * j]);
          acc[t][2 * j + 1] = fmaf(hi_bf(xv[t][j]), d, acc[t][2 * j + 1]);
        }
    }
  }
  float* out = partial + (size_t)blockIdx.x * 9 * Ci * CO;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int j = 0; j < CPT; ++j) out[((size_t)t * Ci + cig * CPT + j) * CO + co] = acc[t][j];
}

// ---------------------------------------------------------------- BatchNorm
// Per-channel sums over rows with 8 channels per thread.  KIND 0: (sum x, sum x^2) -> mean, rstd,
// running stats.  KIND 1: (sum dyh, sum dyh*xhat), dyh = dy*(y>0) -> dbeta, dgamma.
struct BnSumArgs {
  const uint16_t* x; const uint16_t* dy; const uint16_t* y;
  int rows, C;
  const float* mean; const float* rstd;        // KIND 1 inputs
  float* partial;                              // [blocks][2][C]
  float eps, momentum;
  float* out0; float* out1;                    // KIND 0: mean, rstd; KIND 1: dbeta, dgamma
  float* run_mean; float* run_var;
};

// Adds the workgroup partials [nblocks][2][C] in workgroup order and finishes mean / rstd / running
// statistics (KIND 0) or dbeta / dgamma (KIND 1).  One workgroup of NTHR threads.
// l0 / l1 (LDS, may be null) also receive the two results per channel; `global` says whether this
// workgroup writes them (and the running statistics) to memory.
template <int KIND, int NTHR>
__device__ __forceinline__ void bn_finish(const BnSumArgs& p, unsigned nblocks, float* red, float* l0, float* l1, bool global) {
  const int tid = threadIdx.x;
  // 2C values, four per thread (one 16-byte load per partial row); NTHR/(2C/4) thread groups take the workgroup
  // partials round-robin, eight loads in flight each, then one thread per value adds the groups in order
  // (at most 32 groups: the last stage adds them one after the other)
  const int nv = 2 * p.C, nq = nv / 4, parts = NTHR / nq < 32 ? NTHR / nq : 32;
  if (tid < nq * parts) {
    const int v4 = tid % nq, part = tid / nq;
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int U = 16;                                        // partial rows in flight per thread
    for (unsigned bk = part; bk < nblocks; bk += U * parts) {   // summed in workgroup order
      float4 q[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const unsigned bu = bk + u * parts;
        q[u] = bu < nblocks ? *reinterpret_cast<const float4*>(p.partial + (size_t)bu * nv + 4 * v4) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) { t.x += q[u].x; t.y += q[u].y; t.z += q[u].z; t.w += q[u].w; }
    }
    *reinterpret_cast<float4*>(red + part * nv + 4 * v4) = t;
  }
  __syncthreads();
  if (tid < p.C) {
    float s0 = 0.f, s1 = 0.f;
    for (int part = 0; part < parts; ++part) { s0 += red[part * nv + tid]; s1 += red[part * nv + p.C + tid]; }
    float v0 = s0, v1 = s1;
    if (KIND == 0) {
      const float n = (float)p.rows, m = s0 / n;
      const float var = fmaxf(s1 / n - m * m, 0.f);
      v0 = m;
      v1 = 1.0f / sqrtf(var + p.eps);
      if (global) {
        p.run_mean[tid] = (1.f - p.momentum) * p.run_mean[tid] + p.momentum * m;
        p.run_var[tid] = (1.f - p.momentum) * p.run_var[tid] + p.momentum * var * (n / (n - 1.f));
      }
    }
    if (global) { p.out0[tid] = v0; p.out1[tid] = v1; }
    if (l0) { l0[tid] = v0; l1[tid] = v1; }
  }
}

template <int KIND>
__global__ __launch_bounds__(256) void bn_sums_kernel(BnSumArgs p) {
  __shared__ float red[256][17];
  const int groups = p.C / 8;                   // channel groups of 8
  const int lanes = 256 / groups;               // row lanes per workgroup
  const int tid = threadIdx.x, cg = tid % groups, rl = tid / groups;
  float a0[8], a1[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { a0[j] = 0.f; a1[j] = 0.f; }
  float mu[8], rs[8];
  if (KIND == 1) {
#pragma unroll
    for (int j = 0; j < 8; ++j) { mu[j] = p.mean[8 * cg + j]; rs[j] = p.rstd[8 * cg + j]; }
  }
  if (rl < lanes) {
    // four rows per trip, their loads issued together; the sums of a lane still run in row order
    const int stride = gridDim.x * lanes;
    for (int r = blockIdx.x * lanes + rl; r < p.rows; r += 4 * stride) {
      uint4 xv[4], dv[4], yv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int ru = r + u * stride;
        xv[u] = dv[u] = yv[u] = make_uint4(0, 0, 0, 0);
        if (ru < p.rows) {
          const size_t off = (size_t)ru * p.C + 8 * cg;
          xv[u] = *reinterpret_cast<const uint4*>(p.x + off);
          if (KIND == 1) {
            dv[u] = *reinterpret_cast<const uint4*>(p.dy + off);
            yv[u] = *reinterpret_cast<const uint4*>(p.y + off);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (r + u * stride >= p.rows) break;
        const uint32_t* xw = reinterpret_cast<const uint32_t*>(&xv[u]);
        if (KIND == 0) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float a = lo_bf(xw[j]), b = hi_bf(xw[j]);
            a0[2 * j] += a; a0[2 * j + 1] += b; a1[2 * j] += a * a; a1[2 * j + 1] += b * b;
          }
        } else {
          const uint32_t* dw = reinterpret_cast<const uint32_t*>(&dv[u]);
          const uint32_t* yw = reinterpret_cast<const uint32_t*>(&yv[u]);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float d0 = lo_bf(yw[j]) > 0.f ? lo_bf(dw[j]) : 0.f, d1 = hi_bf(yw[j]) > 0.f ? hi_bf(dw[j]) : 0.f;
            a0[2 * j] += d0; a0[2 * j + 1] += d1;
            a1[2 * j] += d0 * (lo_bf(xw[j]) - mu[2 * j]) * rs[2 * j];
            a1[2 * j + 1] += d1 * (hi_bf(xw[j]) - mu[2 * j + 1]) * rs[2 * j + 1];
          }
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) { red[tid][j] = a0[j]; red[tid][8 + j] = a1[j]; }
  __syncthreads();
  // thread c < 2C adds the row lanes of its (sum kind, channel) in order
  if (tid < 2 * p.C) {
    const int which = tid / p.C, c = tid % p.C, g = c / 8, j = c % 8;
    float t = 0.f;
#pragma unroll 8
    for (int l = 0; l < lanes; ++l) t += red[l * groups + g][8 * which + j];
    p.partial[(size_t)blockIdx.x * 2 * p.C + tid] = t;
  }
}

template <int KIND>
__global__ __launch_bounds__(1024) void bn_finish_kernel(BnSumArgs p, unsigned nblocks) {
  __shared__ __align__(16) float red[4096];
  bn_finish<KIND, 1024>(p, nblocks, red, nullptr, nullptr, true);
}

// y = relu(bn(x) (+ res)), 8 channels per thread
__global__ __launch_bounds__(256) void bn_apply_bf16_kernel(const uint16_t* x, size_t chunks, int C, const float* mean,
                                                            const float* rstd, const float* g, const float* b,
                                                            const uint16_t* res, uint16_t* y) {
  const uint32_t i32 = blockIdx.x * 256 + threadIdx.x;     // fewer than 2^32 chunks (checked by the launcher)
  if (i32 >= chunks) return;
  const size_t i = i32;
  const int c0 = (int)(8 * (i32 % (uint32_t)(C / 8)));
  const uint4 xv = *reinterpret_cast<const uint4*>(x + i * 8);
  const uint32_t* xw = reinterpret_cast<const uint32_t*>(&xv);
  uint4 rv = make_uint4(0, 0, 0, 0);
  if (res) rv = *reinterpret_cast<const uint4*>(res + i * 8);
  const uint32_t* rw = reinterpret_cast<const uint32_t*>(&rv);
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = c0 + 2 * j;
    float u = (lo_bf(xw[j]) - mean[c]) * rstd[c] * g[c] + b[c] + lo_bf(rw[j]);
    float v = (hi_bf(xw[j]) - mean[c + 1]) * rstd[c + 1] * g[c + 1] + b[c + 1] + hi_bf(rw[j]);
    o[j] = pack2(fmaxf(u, 0.f), fmaxf(v, 0.f));
  }
  *reinterpret_cast<uint4*>(y + i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// dx = (g rstd / N) (N dyh - dbeta - xhat dgamma)
__global__ __launch_bounds__(256) void bn_bwd_apply_bf16_kernel(const uint16_t* dy, const uint16_t* y,
                                                                const uint16_t* x, size_t chunks, int C, int rows,
                                                                const float* mean, const float* rstd, const float* g,
                                                                const float* dg, const float* db, uint16_t* dx) {
  const uint32_t i32 = blockIdx.x * 256 + threadIdx.x;     // fewer than 2^32 chunks (checked by the launcher)
  if (i32 >= chunks) return;
  const size_t i = i32;
  const int c0 = (int)(8 * (i32 % (uint32_t)(C / 8)));
  const uint4 xv = *reinterpret_cast<const uint4*>(x + i * 8);
  const uint4 dv = *reinterpret_cast<const uint4*>(dy + i * 8);
  const uint4 yv = *reinterpret_cast<const uint4*>(y + i * 8);
  const uint32_t* xw = reinterpret_cast<const uint32_t*>(&xv);
  const uint32_t* dw = reinterpret_cast<const uint32_t*>(&dv);
  const uint32_t* yw = reinterpret_cast<const uint32_t*>(&yv);
  const float n = (float)rows;
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float r[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = c0 + 2 * j + h;
      const float yy = h ? hi_bf(yw[j]) : lo_bf(yw[j]), dd = h ? hi_bf(dw[j]) : lo_bf(dw[j]);
      const float xx = h ? hi_bf(xw[j]) : lo_bf(xw[j]);
      const float d = yy > 0.f ? dd : 0.f, xh = (xx - mean[c]) * rstd[c];
      r[h] = g[c] * rstd[c] / n * (n * d - db[c] - xh * dg[c]);
    }
    o[j] = pack2(r[0], r[1]);
  }
  *reinterpret_cast<uint4*>(dx + i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// Small tensors: the apply kernels add up the partial sums themselves (every workgroup, in the same order;
// workgroup 0 writes the results to memory), which saves the finishing launch.
__global__ __launch_bounds__(256) void bn_apply_fused_kernel(BnSumArgs p, unsigned nblocks, size_t chunks, const float* g,
                                                             const float* b, const uint16_t* res, uint16_t* y) {
  __shared__ __align__(16) float red[1024];
  __shared__ float s_mean[128], s_rstd[128];
  bn_finish<0, 256>(p, nblocks, red, s_mean, s_rstd, blockIdx.x == 0);
  __syncthreads();
  const uint32_t i32 = blockIdx.x * 256 + threadIdx.x;
  if (i32 >= chunks) return;
  const size_t i = i32;
  const int c0 = (int)(8 * (i32 % (uint32_t)(p.C / 8)));
  const uint4 xv = *reinterpret_cast<const uint4*>(p.x + i * 8);
  const uint32_t* xw = reinterpret_cast<const uint32_t*>(&xv);
  uint4 rv = make_uint4(0, 0, 0, 0);
  if (res) rv = *reinterpret_cast<const uint4*>(res + i * 8);
  const uint32_t* rw = reinterpret_cast<const uint32_t*>(&rv);
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = c0 + 2 * j;
    float u = (lo_bf(xw[j]) - s_mean[c]) * s_rstd[c] * g[c] + b[c] + lo_bf(rw[j]);
    float v = (hi_bf(xw[j]) - s_mean[c + 1]) * s_rstd[c + 1] * g[c + 1] + b[c + 1] + hi_bf(rw[j]);
    o[j] = pack2(fmaxf(u, 0.f), fmaxf(v, 0.f));
  }
  *reinterpret_cast<uint4*>(y + i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}
__global__ __launch_bounds__(256) void bn_bwd_apply_fused_kernel(BnSumArgs p, unsigned nblocks, size_t chunks, const float* g,
                                                                 uint16_t* dx) {
  __shared__ __align__(16) float red[1024];
  __shared__ float s_db[128], s_dg[128];
  bn_finish<1, 256>(p, nblocks, red, s_db, s_dg, blockIdx.x == 0);
  __syncthreads();
  const uint32_t i32 = blockIdx.x * 256 + threadIdx.x;
  if (i32 >= chunks) return;
  const size_t i = i32;
  const int c0 = (int)(8 * (i32 % (uint32_t)(p.C / 8)));
  const uint4 xv = *reinterpret_cast<const uint4*>(p.x + i * 8);
  const uint4 dv = *reinterpret_cast<const uint4*>(p.dy + i * 8);
  const uint4 yv = *reinterpret_cast<const uint4*>(p.y + i * 8);
  const uint32_t* xw = reinterpret_cast<const uint32_t*>(&xv);
  const uint32_t* dw = reinterpret_cast<const uint32_t*>(&dv);
  const uint32_t* yw = reinterpret_cast<const uint32_t*>(&yv);
  const float n = (float)p.rows;
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float r[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = c0 + 2 * j + h;
      const float yy = h ? hi_bf(yw[j]) : lo_bf(yw[j]), dd = h ? hi_bf(dw[j]) : lo_bf(dw[j]);
      const float xx = h ? hi_bf(xw[j]) : lo_bf(xw[j]);
      const float d = yy > 0.f ? dd : 0.f, xh = (xx - p.mean[c]) * p.rstd[c];
      r[h] = g[c] * p.rstd[c] / n * (n * d - s_db[c] - xh * s_dg[c]);
    }
    o[j] = pack2(r[0], r[1]);
  }
  *reinterpret_cast<uint4*>(dx + i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// Elementwise helpers of the stage, 8 channels (16 bytes) per thread, 32-bit index arithmetic.
// dx[b, p, c] = dpooled[b, c] / HW
__global__ __launch_bounds__(256) void gap_bwd_bf16_kernel(const uint16_t* dpooled, uint32_t HW, uint32_t C, uint32_t chunks,
                                                           uint16_t* dx) {
  const uint32_t i = blockIdx.x * 256 + threadIdx.x;
  if (i >= chunks) return;
  const uint32_t cpr = C / 8, cg = i % cpr, b = (i / cpr) / HW;
  const uint4 v = *reinterpret_cast<const uint4*>(dpooled + (size_t)b * C + 8 * cg);
  const uint32_t* w = reinterpret_cast<const uint32_t*>(&v);
  const float hw = (float)HW;
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) o[j] = pack2(lo_bf(w[j]) / hw, hi_bf(w[j]) / hw);
  *reinterpret_cast<uint4*>(dx + (size_t)i * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// pooled[b, c] = mean over the HW pixels of x[b, p, c]: one workgroup per image, thread (channel group of 8, pixel
// lane); the pixel lanes are added in order
__global__ __launch_bounds__(256) void gap_fwd_bf16_kernel(const uint16_t* x, int HW, int C, uint16_t* pooled) {
  __shared__ float red[256][9];
  const int groups = C / 8, lanes = 256 / groups, cg = threadIdx.x % groups, pl = threadIdx.x / groups;
  const uint16_t* xb = x + (size_t)blockIdx.x * HW * C + 8 * cg;
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (pl < lanes)
    for (int p0 = pl; p0 < HW; p0 += 4 * lanes) {     // four loads in flight
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int pp = p0 + u * lanes;
        v[u] = pp < HW ? *reinterpret_cast<const uint4*>(xb + (size_t)pp * C) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t* w = reinterpret_cast<const uint32_t*>(&v[u]);
#pragma unroll
        for (int j = 0; j < 4; ++j) { a[2 * j] += lo_bf(w[j]); a[2 * j + 1] += hi_bf(w[j]); }
      }
    }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[threadIdx.x][j] = a[j];
  __syncthreads();
  if (threadIdx.x < C) {
    const int g = threadIdx.x / 8, j = threadIdx.x % 8;
    float t = 0.f;
    for (int l = 0; l < lanes; ++l) t += red[l * groups + g][j];
    pooled[(size_t)blockIdx.x * C + threadIdx.x] = f32_to_bf16(t / HW);
  }
}

// y[b,oy,ox,c] = x[b, oy*stride, ox*stride, c] for c < Ci, 0 above
__global__ __launch_bounds__(256) void shortcut_fwd_bf16_kernel(const uint16_t* x, uint32_t H, uint32_t W, uint32_t Ci,
                                                                uint32_t Co, uint32_t stride, uint32_t Ho, uint32_t Wo,
                                                                uint32_t chunks, uint16_t* y) {
  const uint32_t i = blockIdx.x * 256 + threadIdx.x;
  if (i >= chunks) return;
  const uint32_t cpr = Co / 8, cg = i % cpr, pix = i / cpr, ox = pix % Wo, oy = (pix / Wo) % Ho, b = pix / (Wo * Ho);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (8 * cg < Ci) v = *reinterpret_cast<const uint4*>(x + ((size_t)(b * H + oy * stride) * W + ox * stride) * Ci + 8 * cg);
  *reinterpret_cast<uint4*>(y + (size_t)i * 8) = v;
}

// dx[b, oy*stride, ox*stride, c] += dy[b,oy,ox,c] * (ymask[b,oy,ox,c] > 0) for c < Ci
__global__ __launch_bounds__(256) void shortcut_bwd_bf16_kernel(const uint16_t* dy, const uint16_t* ymask, uint32_t H,
                                                                uint32_t W, uint32_t Ci, uint32_t Co, uint32_t stride,
                                                                uint32_t Ho, uint32_t Wo, uint32_t chunks, uint16_t* dx) {
  const uint32_t i = blockIdx.x * 256 + threadIdx.x;
  if (i >= chunks) return;
  const uint32_t cpr = Ci / 8, cg = i % cpr, pix = i / cpr, ox = pix % Wo, oy = (pix / Wo) % Ho, b = pix / (Wo * Ho);
  const size_t yi = (size_t)pix * Co + 8 * cg, xi = ((size_t)(b * H + oy * stride) * W + ox * stride) * Ci + 8 * cg;
  const uint4 dv = *reinterpret_cast<const uint4*>(dy + yi), mv = *reinterpret_cast<const uint4*>(ymask + yi);
  const uint4 xv = *reinterpret_cast<const uint4*>(dx + xi);
  const uint32_t* dw = reinterpret_cast<const uint32_t*>(&dv);
  const uint32_t* mw = reinterpret_cast<const uint32_t*>(&mv);
  const uint32_t* xw = reinterpret_cast<const uint32_t*>(&xv);
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = lo_bf(xw[j]) + (lo_bf(mw[j]) > 0.f ? lo_bf(dw[j]) : 0.f);
    const float hi = hi_bf(xw[j]) + (hi_bf(mw[j]) > 0.f ? hi_bf(dw[j]) : 0.f);
    o[j] = pack2(lo, hi);
  }
  *reinterpret_cast<uint4*>(dx + xi) = make_uint4(o[0], o[1], o[2], o[3]);
}

bool al16(const void* p) { return !(((uintptr_t)p) & 15); }

// LDS of the implicit-GEMM convolution: the filter as [produced channels rounded up to 32][9 * reduced + 8] bf16
size_t conv_mfma_lds(int produced, int reduced) { return (size_t)((produced + 31) / 32 * 32) * (18 * reduced + 16); }
constexpr size_t CONV_MFMA_LDS_MAX = 96 * 1024;
// workgroups of the forward / stride-1 kernel for P output pixels: a workgroup keeps its filter for up to 4 tiles of
// 128 pixels once there are more than 2048 of them
long conv_mfma_blocks(long P) {
  const long ntiles = (P + 127) / 128;
  const long tpw = ntiles >= 8192 ? 4 : (ntiles >= 4096 ? 2 : 1);
  return (ntiles + tpw - 1) / tpw;
}
template <int MODE, int K16, int NT, int GRP, bool LIN, bool STAT>
int conv_mfma_launch_g(hipStream_t s, const ConvArgs& p, long P, size_t lds) {
  static bool raised[64] = {};    // per device: the attribute belongs to the device's copy of the kernel
  lds += STAT ? CONV_STAT_LDS : 0;
  if (lds > 64 * 1024) {
    int dev = 0;
    PPLL_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64 || !raised[dev]) {
      PPLL_HIP(hipFuncSetAttribute((const void*)conv3x3_mfma_kernel<MODE, K16, NT, GRP, LIN, STAT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)(CONV_MFMA_LDS_MAX + CONV_STAT_LDS)));
      if (dev >= 0 && dev < 64) raised[dev] = true;
    }
  }
  hipLaunchKernelGGL((conv3x3_mfma_kernel<MODE, K16, NT, GRP, LIN, STAT>), dim3((unsigned)conv_mfma_blocks(P)), dim3(256), lds, s, p);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
template <int MODE, int K16>
int conv_mfma_launch_k(hipStream_t s, const ConvArgs& p, long P, size_t lds) {
  const int produced = MODE == 0 ? p.Co : p.Ci;
  // GRP = 1: the three taps of a filter row in flight together
  // linear tap addressing through a buffer descriptor: forward always, input gradient at stride 1; the source
  // tensor has to stay below 2^30 bytes
  const bool lin = (MODE == 0 || p.stride == 1) && (long)p.B * p.H * p.W * (16 * K16) * 2 < ((long)1 << 30);
  if (p.stat) {
    if (produced <= 32)
      return lin ? conv_mfma_launch_g<MODE, K16, 1, 1, true, true>(s, p, P, lds) : conv_mfma_launch_g<MODE, K16, 1, 1, false, true>(s, p, P, lds);
    return lin ? conv_mfma_launch_g<MODE, K16, 2, 1, true, true>(s, p, P, lds) : conv_mfma_launch_g<MODE, K16, 2, 1, false, true>(s, p, P, lds);
  }
  if (produced <= 32)
    return lin ? conv_mfma_launch_g<MODE, K16, 1, 1, true, false>(s, p, P, lds) : conv_mfma_launch_g<MODE, K16, 1, 1, false, false>(s, p, P, lds);
  return lin ? conv_mfma_launch_g<MODE, K16, 2, 1, true, false>(s, p, P, lds) : conv_mfma_launch_g<MODE, K16, 2, 1, false, false>(s, p, P, lds);
}
// k16 = reduced channels / 16: 1, 2, 3 or 4
template <int MODE>
int conv_mfma_launch(hipStream_t s, const ConvArgs& p, long P, int k16, size_t lds) {
  switch (k16) {
    case 1: return conv_mfma_launch_k<MODE, 1>(s, p, P, lds);
    case 2: return conv_mfma_launch_k<MODE, 2>(s, p, P, lds);
    case 3: return conv_mfma_launch_k<MODE, 3>(s, p, P, lds);
    case 4: return conv_mfma_launch_k<MODE, 4>(s, p, P, lds);
  }
  set_error("conv3x3: %d reduced channels have no matrix-core kernel", 16 * k16);
  return PPLL_ERR_CONFIG;
}
}  // namespace

// the convolution kernels index pixels with 32 bits
bool conv_pixels_fit(int B, int H, int W) { return (size_t)B * H * W < ((size_t)1 << 31) - 128; }
bool conv_bf16_supported(int dt, int wdt, int Ci, int Co, const void* a, const void* b, const void* c) {
  if (dt != BF16 || wdt != BF16) return false;
  if ((Ci % 16) || (Co % 16) || Ci > 128 || Co > 128) return false;
  return al16(a) && al16(b) && al16(c);
}

template <int K16, int NT>
static int conv_dgrad_s2_launch_k(hipStream_t s, const ConvArgs& p, size_t lds) {
  static bool raised[64] = {};
  if (lds > 64 * 1024) {
    int dev = 0;
    PPLL_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64 || !raised[dev]) {
      PPLL_HIP(hipFuncSetAttribute((const void*)conv3x3_dgrad_s2_kernel<K16, NT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)CONV_MFMA_LDS_MAX));
      if (dev >= 0 && dev < 64) raised[dev] = true;
    }
  }
  const long pc = (long)p.B * (p.H / 2) * (p.W / 2), tiles = 4 * ((pc + 127) / 128);
  const long tpw = tiles >= 8192 ? 4 : (tiles >= 4096 ? 2 : 1);
  hipLaunchKernelGGL((conv3x3_dgrad_s2_kernel<K16, NT>), dim3((unsigned)((tiles + tpw - 1) / tpw)), dim3(256), lds, s, p);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
static int conv_dgrad_s2_launch(hipStream_t s, const ConvArgs& p, int k16, size_t lds) {
  const bool two = p.Ci > 32;
  switch (k16) {
    case 1: return two ? conv_dgrad_s2_launch_k<1, 2>(s, p, lds) : conv_dgrad_s2_launch_k<1, 1>(s, p, lds);
    case 2: return two ? conv_dgrad_s2_launch_k<2, 2>(s, p, lds) : conv_dgrad_s2_launch_k<2, 1>(s, p, lds);
    case 3: return two ? conv_dgrad_s2_launch_k<3, 2>(s, p, lds) : conv_dgrad_s2_launch_k<3, 1>(s, p, lds);
    case 4: return two ? conv_dgrad_s2_launch_k<4, 2>(s, p, lds) : conv_dgrad_s2_launch_k<4, 1>(s, p, lds);
  }
  set_error("conv3x3: %d reduced channels have no matrix-core kernel", 16 * k16);
  return PPLL_ERR_CONFIG;
}

int launch_conv3x3_fwd_bf16(hipStream_t s, const void* x, const void* w, int B, int H, int W, int Ci, int Co,
                            int stride, void* y, float* stat, int* stat_blocks) {
  const long P = (long)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
  // The sums cost the kernel registers and ~25 % of its time at 16 channels; they pay where the BatchNorm's own pass
  // over the tensor is mostly launch and ramp, i.e. on small tensors (measured: 9 % of the step at 128 x 16 x 16 x 32,
  // 3 % at 1024 x 8 x 8 x 64, a loss at 1024 x 16 x 16 x 32 and above, where also 2048 partial rows have to be added up)
  if (conv_mfma_blocks(P) > CONV_STAT_MAX_BLOCKS) stat = nullptr;
  ConvArgs p{(const uint16_t*)x, (const uint16_t*)w, (uint16_t*)y, B, H, W, Ci, Co, stride, nullptr, nullptr, stat,
             nullptr, nullptr, nullptr, nullptr};
  if (stat_blocks) *stat_blocks = stat ? (int)conv_mfma_blocks(P) : 0;
  const size_t lds = conv_mfma_lds(Co, Ci);
  void* prof = nullptr;   // algorithmic bytes: input, output and filter once
  PPLL_TRY(profile_begin(s, 2.0 * ((double)B * H * W * Ci + (double)P * Co + 9.0 * Ci * Co), &prof, 1));
  PPLL_TRY((conv_mfma_launch<0>(s, p, P, Ci / 16, lds)));
  return profile_end(s, prof);
}

int launch_conv3x3_dgrad_bf16(hipStream_t s, const void* dy, const void* w, int B, int H, int W, int Ci, int Co,
                              int stride, const void* dres, const void* ymask, void* dx, const BnBwdSums* bn,
                              int* stat_blocks) {
  const long P = (long)B * H * W;
  // sums for the BatchNorm that dx is the output gradient of: stride 1 only, small tensors only (as in the forward)
  const bool sums = bn && bn->partials && stride == 1 && conv_mfma_blocks(P) <= CONV_BWD_STAT_MAX_BLOCKS && al16(bn->y) &&
                    al16(bn->x) && al16(bn->mean) && al16(bn->rstd);
  if (stat_blocks) *stat_blocks = sums ? (int)conv_mfma_blocks(P) : 0;
  ConvArgs p{(const uint16_t*)dy, (const uint16_t*)w, (uint16_t*)dx, B, H, W, Ci, Co, stride, (const uint16_t*)dres,
             (const uint16_t*)ymask, sums ? bn->partials : nullptr, sums ? (const uint16_t*)bn->y : nullptr,
             sums ? (const uint16_t*)bn->x : nullptr, sums ? bn->mean : nullptr, sums ? bn->rstd : nullptr};
  const size_t lds = conv_mfma_lds(Ci, Co);
  const double Po = (double)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
  void* prof = nullptr;   // algorithmic bytes: dy, dx and filter once, plus the shortcut gradient and its mask
  PPLL_TRY(profile_begin(s, 2.0 * (Po * Co + (double)P * Ci * (dres ? 3.0 : 1.0) + 9.0 * Ci * Co), &prof, 1));
  if (stride == 2 && !(H & 1) && !(W & 1) && !dres && Po * Co * 2 < (double)(1 << 30))
    PPLL_TRY(conv_dgrad_s2_launch(s, p, Co / 16, lds));
  else
    PPLL_TRY((conv_mfma_launch<1>(s, p, P, Co / 16, lds)));
  return profile_end(s, prof);
}

// forward and input gradient produce up to 64 channels (two MFMA tiles of 32; 16 and 48 leave half a tile idle)
bool conv_fwd_bf16_ok(int Ci, int Co) { return Co % 16 == 0 && Co <= 64 && Ci <= 64 && conv_mfma_lds(Co, Ci) <= CONV_MFMA_LDS_MAX; }
bool conv_dgrad_bf16_ok(int Ci, int Co) { return Ci % 16 == 0 && Ci <= 64 && Co <= 64 && conv_mfma_lds(Ci, Co) <= CONV_MFMA_LDS_MAX; }
bool conv_wgrad_bf16_ok(int Ci, int Co) {
  if (Co == 16) return Ci == 16;
  return (Co == 32 || Co == 64) && Ci % 16 == 0 && Ci >= 16 && Ci <= 64;
}

typedef __attribute__((ext_vector_type(8))) __bf16 wg_bf16x8;
// ---------------------------------------------------------------------------------------------
// Weight gradient on the matrix cores for CI -> CO channels (16, 32 or 64 each), stride 1 or 2, output
// rows of 8, 16, 24, ... pixels.  The reduction index of a 16x16x32 MFMA is the output pixel: a k-step is
// four groups of 8 consecutive pixels of one output row.  A workgroup of 8 waves takes whole images: it
// transposes x and dy of an image to [channel][pixel] in LDS.  x gets a 16-byte zero gap in front of every
// row and a zero row above and below, so that no tap needs a bounds test; with stride 2 a row of x is
// stored as its odd columns followed by its even columns, which makes the pixels that 8 consecutive
// outputs read consecutive again.  A wave owns one tile of 16 output channels for all 9 taps and all
// input-channel tiles and every (8 / tiles)-th k-step.  The fragment of the tap that starts one pixel to
// the left (and, at stride 1, to the right) is the aligned one shifted by two bytes, the neighbouring
// pixel read separately.  The k-splits of a workgroup are added in LDS in k-split order: one partial per
// workgroup, summed over workgroups by the ordered second-stage reduction.
typedef __attribute__((ext_vector_type(4))) float wg_f32x4;
constexpr int WGT_WAVES = 8;
constexpr int WGT_FOLD_BYTES = 9 * 64 * 64 * 4;      // 144 KiB: LDS the k-split sums may take
__host__ __device__ inline int wgt_pad16(int bytes) { return bytes + ((16 - bytes % 128) + 128) % 128; }   // = 16 mod 128
__host__ __device__ inline int wgt_row_stride(int W) { return 16 + 2 * W; }
__host__ __device__ inline int wgt_x_stride(int H, int W) { return wgt_pad16((H + 2) * wgt_row_stride(W) + 16); }
__host__ __device__ inline int wgt_dy_stride(int Ho, int Wo) { return wgt_pad16(Ho * Wo * 2); }

// 4 pixels x 8 channels (one uint4 per pixel) -> for channel i the 4 pixels as one uint2
__device__ __forceinline__ uint2 wgt_gather4(const uint4& p0, const uint4& p1, const uint4& p2, const uint4& p3, int i) {
  const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
  uint2 o;
  o.x = __builtin_amdgcn_perm(reinterpret_cast<const uint32_t*>(&p1)[i >> 1], reinterpret_cast<const uint32_t*>(&p0)[i >> 1], sel);
  o.y = __builtin_amdgcn_perm(reinterpret_cast<const uint32_t*>(&p3)[i >> 1], reinterpret_cast<const uint32_t*>(&p2)[i >> 1], sel);
  return o;
}

// up to 16 convolutions of one shape in a launch: blockIdx.y picks the convolution
constexpr int WGT_GROUP = 16;
struct WgtGroup { const uint16_t* x[WGT_GROUP]; const uint16_t* dy[WGT_GROUP]; float* partial[WGT_GROUP]; };

template <int CI, int CO, int S>
__global__ __launch_bounds__(64 * WGT_WAVES) void conv3x3_wgrad_tiles_kernel(WgtGroup grp, int B, int H, int W) {
  const uint16_t* __restrict__ x = grp.x[blockIdx.y];
  const uint16_t* __restrict__ dy = grp.dy[blockIdx.y];
  float* __restrict__ partial = grp.partial[blockIdx.y];
  constexpr int CT = CI / 16, WN = CO / 16, WK = WGT_WAVES / WN, NT = 64 * WGT_WAVES, NW = 9 * CI * CO;
  constexpr bool FOLD_ALL = WK * NW * 4 <= WGT_FOLD_BYTES;
  static_assert(FOLD_ALL || WK == 2, "the k-splits either fit LDS together or are two");
  extern __shared__ __align__(16) char sm[];
  const int Ho = H / S, Wo = W / S;            // S = 2: H and W are even
  const int RS = wgt_row_stride(W), CSX = wgt_x_stride(H, W), CSD = wgt_dy_stride(Ho, Wo);
  char* xt = sm;                              // x  as [CI][H + 2 rows][16-byte gap, W pixels]
  char* dt = sm + CI * CSX;                   // dy as [CO][Ho * Wo pixels]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, q = lane >> 4;
  const int wn = wave % WN, kq = wave / WN;
  for (int o = tid * 16; o < CI * CSX; o += NT * 16) *reinterpret_cast<uint4*>(xt + o) = make_uint4(0, 0, 0, 0);
  wg_f32x4 acc[9][CT];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[t][j][e] = 0.f;
  const int wo8 = Wo / 8, groups = Ho * wo8, ksteps = (groups + 3) / 4;
  const int xw = S == 1 ? W / 4 : W / 8, xitems = H * xw * (CI / 8);     // (row, 4 or 8 pixels, 8 channels)
  const int dw4 = Wo / 4, ditems = Ho * dw4 * (CO / 8);
  for (int b = blockIdx.x; b < B; b += gridDim.x) {
    const uint16_t* xb = x + (size_t)b * H * W * CI;
    const uint16_t* db = dy + (size_t)b * Ho * Wo * CO;
    __syncthreads();                          // zero fill done / the previous image's tiles are no longer read
    for (int item = tid; item < xitems; item += NT) {
      const int cg = item % (CI / 8), pg = item / (CI / 8), y = pg / xw, xg = pg % xw;
      char* row = xt + (8 * cg) * CSX + (y + 1) * RS + 16;
      if (S == 1) {
        uint4 rx[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) rx[j] = *reinterpret_cast<const uint4*>(xb + ((size_t)(y * W + 4 * xg + j)) * CI + 8 * cg);
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<uint2*>(row + i * CSX + 8 * xg) = wgt_gather4(rx[0], rx[1], rx[2], rx[3], i);
      } else {
        uint4 rx[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) rx[j] = *reinterpret_cast<const uint4*>(xb + ((size_t)(y * W + 8 * xg + j)) * CI + 8 * cg);
#pragma unroll
        for (int i = 0; i < 8; ++i) {   // odd columns first, then the even ones
          *reinterpret_cast<uint2*>(row + i * CSX + 8 * xg) = wgt_gather4(rx[1], rx[3], rx[5], rx[7], i);
          *reinterpret_cast<uint2*>(row + i * CSX + 2 * Wo + 8 * xg) = wgt_gather4(rx[0], rx[2], rx[4], rx[6], i);
        }
      }
    }
    for (int item = tid; item < ditems; item += NT) {
      const int cg = item % (CO / 8), pg = item / (CO / 8);      // pg = 4-pixel group of the image, row-major
      uint4 rd[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) rd[j] = *reinterpret_cast<const uint4*>(db + ((size_t)(4 * pg + j)) * CO + 8 * cg);
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<uint2*>(dt + (8 * cg + i) * CSD + 8 * pg) = wgt_gather4(rd[0], rd[1], rd[2], rd[3], i);
    }
    __syncthreads();
    for (int ks = kq; ks < ksteps; ks += WK) {
      // the last k-step of an image may hold fewer than four pixel groups: the others multiply by zero
      const bool live = 4 * ks + q < groups;
      const int g = live ? 4 * ks + q : 0, oy = g / wo8, x0 = 8 * (g % wo8);
      uint4 gv = make_uint4(0, 0, 0, 0);
      if (live) gv = *reinterpret_cast<const uint4*>(dt + (16 * wn + r) * CSD + g * 16);
      const wg_bf16x8 gf = __builtin_bit_cast(wg_bf16x8, gv);
#pragma unroll
      for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int t = 0; t < CT; ++t) {
          // row S*oy + ky - 1 of the image = row S*oy + ky of the padded tile
          const char* base = xt + (16 * t + r) * CSX + (S * oy + ky) * RS + 16 + 2 * x0;
          const uint4 w = *reinterpret_cast<const uint4*>(base);     // S = 1: pixels x0..x0+7; S = 2: odd columns 2 x0 + 1 ..
          const uint32_t prev = *reinterpret_cast<const uint16_t*>(base - 2);
          uint4 a0, a1, a2;
          a0.x = (w.x << 16) | prev;
          a0.y = __builtin_amdgcn_alignbyte(w.y, w.x, 2);
          a0.z = __builtin_amdgcn_alignbyte(w.z, w.y, 2);
          a0.w = __builtin_amdgcn_alignbyte(w.w, w.z, 2);
          if (S == 1) {
            const uint32_t next = *reinterpret_cast<const uint16_t*>(base + 16);
            a1 = w;
            a2.x = a0.y; a2.y = a0.z; a2.z = a0.w;
            a2.w = (next << 16) | (w.w >> 16);
          } else {
            a1 = *reinterpret_cast<const uint4*>(base + 2 * Wo);     // even columns 2 x0 ..
            a2 = w;
          }
          acc[3 * ky][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(wg_bf16x8, a0), gf, acc[3 * ky][t], 0, 0, 0);
          acc[3 * ky + 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(wg_bf16x8, a1), gf, acc[3 * ky + 1][t], 0, 0, 0);
          acc[3 * ky + 2][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(wg_bf16x8, a2), gf, acc[3 * ky + 2][t], 0, 0, 0);
        }
    }
  }
  // acc[tap][t][e] = dw[tap][ci = 16 t + 4 q + e][co = 16 wn + r] of this wave's k-steps
  float* fold = reinterpret_cast<float*>(sm);
  float* out = partial + (size_t)blockIdx.x * NW;
  __syncthreads();                            // the tiles are no longer read
  if constexpr (FOLD_ALL) {
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int t = 0; t < CT; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) fold[kq * NW + (tap * CI + 16 * t + 4 * q + e) * CO + 16 * wn + r] = acc[tap][t][e];
    __syncthreads();
    for (int i = tid; i < NW; i += NT) {
      float v = fold[i];
#pragma unroll
      for (int k = 1; k < WK; ++k) v += fold[k * NW + i];
      out[i] = v;
    }
  } else {
    // two k-splits: the second half of the waves hands its sums over through LDS
    if (kq == 1) {
#pragma unroll
      for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int t = 0; t < CT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) fold[(tap * CI + 16 * t + 4 * q + e) * CO + 16 * wn + r] = acc[tap][t][e];
    }
    __syncthreads();
    if (kq == 0) {
#pragma unroll
      for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int t = 0; t < CT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = (tap * CI + 16 * t + 4 * q + e) * CO + 16 * wn + r;
            out[i] = acc[tap][t][e] + fold[i];
          }
    }
  }
}

static size_t wgrad_tiles_lds(int H, int W, int Ci, int Co, int stride) {
  const size_t tiles = (size_t)Ci * wgt_x_stride(H, W) + (size_t)Co * wgt_dy_stride(H / stride, W / stride);
  const size_t nw = (size_t)9 * Ci * Co * 4, wk = WGT_WAVES / (Co / 16);
  const size_t fold = wk * nw <= (size_t)WGT_FOLD_BYTES ? wk * nw : nw;
  return tiles > fold ? tiles : fold;
}
static bool wgrad_tiles_ok(int H, int W, int Ci, int Co, int stride) {
  const bool chan = stride == 1 ? (Ci == Co && (Ci == 16 || Ci == 32 || Ci == 64))
                                : ((Ci == 16 && (Co == 32 || Co == 64)) || (Ci == 32 && Co == 64) || (Ci == 64 && Co == 64));
  if (!chan || stride < 1 || stride > 2 || (H % stride) || (W % stride)) return false;
  const int Wo = W / stride;
  return Wo >= 8 && (Wo % 8) == 0 && wgrad_tiles_lds(H, W, Ci, Co, stride) <= 160 * 1024;
}
// Workgroups per convolution.  A workgroup costs about 10 us before and after its images (clearing its LDS tiles,
// folding the k-splits, writing its partial filter) against 1-1.5 us per image, and its LDS footprint lets one or two
// of them run on a compute unit, so the n convolutions of a launch together get one round of those places and each
// workgroup walks over several images (measured at 10 convolutions 32 -> 32 on 128 images: 103 workgroups each 31 us
// + 9 us for adding the partial filters, 51: 26 + 6, 25: 22 + 5, 12: 32 + 5).  n = 1 gives the most there can be
// (what the partial sums are sized for).
static int wgrad_tiles_blocks(int B, int n, int places) {
  int blocks = places / (n < 1 ? 1 : n);
  blocks = blocks < 1 ? 1 : blocks;
  return B < blocks ? B : blocks;
}
// places for the workgroups of one launch on the current device: compute units x workgroups that fit one unit's LDS
static int wgrad_tiles_places(size_t lds) {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  const size_t per = lds ? ((size_t)160 * 1024) / lds : 2;
  return cus * (int)(per < 1 ? 1 : (per > 2 ? 2 : per));     // 512 threads each: two at most
}
template <int CI, int CO, int S>
static int wgrad_tiles_launch(hipStream_t s, const WgtGroup& g, int n, int B, int H, int W, int blocks) {
  const size_t lds = wgrad_tiles_lds(H, W, CI, CO, S);
  if (lds > 64 * 1024)
    PPLL_HIP(hipFuncSetAttribute((const void*)conv3x3_wgrad_tiles_kernel<CI, CO, S>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)lds));
  hipLaunchKernelGGL((conv3x3_wgrad_tiles_kernel<CI, CO, S>), dim3(blocks, n), dim3(64 * WGT_WAVES), lds, s, g, B, H, W);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
static int wgrad_tiles_dispatch(hipStream_t s, const WgtGroup& g, int n, int B, int H, int W, int Ci, int Co, int stride,
                                int blocks) {
  if (stride == 1) {
    if (Ci == 16) return wgrad_tiles_launch<16, 16, 1>(s, g, n, B, H, W, blocks);
    if (Ci == 32) return wgrad_tiles_launch<32, 32, 1>(s, g, n, B, H, W, blocks);
    return wgrad_tiles_launch<64, 64, 1>(s, g, n, B, H, W, blocks);
  }
  if (Ci == 16 && Co == 32) return wgrad_tiles_launch<16, 32, 2>(s, g, n, B, H, W, blocks);
  if (Ci == 16 && Co == 64) return wgrad_tiles_launch<16, 64, 2>(s, g, n, B, H, W, blocks);
  if (Ci == 32 && Co == 64) return wgrad_tiles_launch<32, 64, 2>(s, g, n, B, H, W, blocks);
  return wgrad_tiles_launch<64, 64, 2>(s, g, n, B, H, W, blocks);
}

size_t conv3x3_wgrad_bf16_partial_floats(int B, int H, int W, int Ci, int Co, int stride) {
  const long P = (long)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
  size_t n = (size_t)((P + WG_PIX_F - 1) / WG_PIX_F) * 9 * Ci * Co;
  if (wgrad_tiles_ok(H, W, Ci, Co, stride)) {
    const size_t m = (size_t)wgrad_tiles_blocks(B, 1, wgrad_tiles_places(wgrad_tiles_lds(H, W, Ci, Co, stride))) * 9 * Ci * Co;
    if (m > n) n = m;
  }
  return n;
}

template <int CO, int CPT>
static int wgrad_launch(hipStream_t s, const void* x, const void* dy, int B, int H, int W, int Ci, int stride,
                        float* partials, int chunks) {
  const size_t lds = ((size_t)WG_PIX_F * 9 * Ci + (size_t)WG_PIX_F * CO) * 2;
  if (lds > 64 * 1024)
    PPLL_HIP(hipFuncSetAttribute((const void*)conv3x3_wgrad_bf16_kernel<CO, CPT>,
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL((conv3x3_wgrad_bf16_kernel<CO, CPT>), dim3(chunks), dim3(256), lds, s, (const uint16_t*)x,
                     (const uint16_t*)dy, B, H, W, Ci, stride, partials);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_conv3x3_wgrad_bf16(hipStream_t s, const void* x, const void* dy, int B, int H, int W, int Ci, int Co,
                              int stride, ReduceQueue& rq, float* dw, int ci_keep) {
  const long P = (long)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
  const int chunks = (int)((P + WG_PIX_F - 1) / WG_PIX_F), nw = 9 * Ci * Co;
  const int cpt = Ci / (256 / Co);
  bool queued;
  if (wgrad_tiles_ok(H, W, Ci, Co, stride)) {
    const int blocks = wgrad_tiles_blocks(B, 1, wgrad_tiles_places(wgrad_tiles_lds(H, W, Ci, Co, stride)));
    float* part = rq.space((size_t)blocks * nw, &queued);
    WgtGroup g{};
    g.x[0] = (const uint16_t*)x; g.dy[0] = (const uint16_t*)dy; g.partial[0] = part;
    PPLL_TRY(wgrad_tiles_dispatch(s, g, 1, B, H, W, Ci, Co, stride, blocks));
    return reduce_conv_filters(s, rq, queued, part, blocks, Ci, Co, ci_keep, dw);
  }
  float* partials = rq.space((size_t)chunks * nw, &queued);
  int st = PPLL_ERR_CONFIG;
  if (Co == 16 && cpt == 1) st = wgrad_launch<16, 1>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 32 && cpt == 2) st = wgrad_launch<32, 2>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 32 && cpt == 4) st = wgrad_launch<32, 4>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 32 && cpt == 6) st = wgrad_launch<32, 6>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 32 && cpt == 8) st = wgrad_launch<32, 8>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 64 && cpt == 4) st = wgrad_launch<64, 4>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 64 && cpt == 8) st = wgrad_launch<64, 8>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 64 && cpt == 12) st = wgrad_launch<64, 12>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else if (Co == 64 && cpt == 16) st = wgrad_launch<64, 16>(s, x, dy, B, H, W, Ci, stride, partials, chunks);
  else set_error("conv3x3 weight gradient: no kernel for %d -> %d channels", Ci, Co);
  PPLL_TRY(st);
  return reduce_conv_filters(s, rq, queued, partials, chunks, Ci, Co, ci_keep, dw);
}

// Weight gradients of n convolutions of one shape in as few launches as possible (16 per launch).  Returns
// PPLL_OK with *done = false, having launched nothing, when the shape is not one the tiled kernel takes or the
// queue has no private room left for all partial sums (the caller then launches them one by one).
int launch_conv3x3_wgrad_group_bf16(hipStream_t s, const ConvWgradJob* jobs, int n, int B, int H, int W, int Ci, int Co,
                                    int stride, ReduceQueue& rq, bool* done) {
  *done = false;
  if (!wgrad_tiles_ok(H, W, Ci, Co, stride)) return PPLL_OK;
  const int blocks = wgrad_tiles_blocks(B, n < WGT_GROUP ? n : WGT_GROUP, wgrad_tiles_places(wgrad_tiles_lds(H, W, Ci, Co, stride)));
  const int nw = 9 * Ci * Co;
  const size_t need = ((size_t)blocks * nw + 63) & ~(size_t)63;
  if (!rq.arena || rq.used + need * n > rq.arena_floats) return PPLL_OK;
  for (int j0 = 0; j0 < n; j0 += WGT_GROUP) {
    const int m = n - j0 < WGT_GROUP ? n - j0 : WGT_GROUP;
    WgtGroup g{};
    for (int j = 0; j < m; ++j) {
      bool queued;
      g.x[j] = (const uint16_t*)jobs[j0 + j].x; g.dy[j] = (const uint16_t*)jobs[j0 + j].dy;
      g.partial[j] = rq.space((size_t)blocks * nw, &queued);     // queued: room was checked above
    }
    PPLL_TRY(wgrad_tiles_dispatch(s, g, m, B, H, W, Ci, Co, stride, blocks));
    for (int j = 0; j < m; ++j) PPLL_TRY(reduce_conv_filters(s, rq, true, g.partial[j], blocks, Ci, Co, Ci, jobs[j0 + j].dw));
  }
  *done = true;
  return PPLL_OK;
}

bool bn_bf16_supported(int dt, int rows, int C, const void* a, const void* b, const void* c, const void* d) {
  if (dt != BF16 || (C % 8) || C < 8 || C > 128 || (256 % (C / 8))) return false;
  if ((size_t)rows * C / 8 >= ((size_t)1 << 32)) return false;   // the kernels index 16-byte chunks with 32 bits
  return al16(a) && al16(b) && al16(c) && al16(d);
}
static int bn_blocks(int rows, int C) {
  const int lanes = 256 / (C / 8);
  int blocks = (rows + lanes * 8 - 1) / (lanes * 8);     // about eight rows per thread
  return blocks < 1 ? 1 : (blocks > 256 ? 256 : blocks);
}
template <int KIND>
static int bn_sums_launch(hipStream_t s, const BnSumArgs& p, int blocks, bool finish) {
  hipLaunchKernelGGL(bn_sums_kernel<KIND>, dim3(blocks), dim3(256), 0, s, p);
  PPLL_HIP(hipGetLastError());
  if (finish) {
    hipLaunchKernelGGL(bn_finish_kernel<KIND>, dim3(1), dim3(1024), 0, s, p, (unsigned)blocks);
    PPLL_HIP(hipGetLastError());
  }
  return PPLL_OK;
}
// the apply kernel of a small tensor (at most 1024 workgroups) finishes the sums itself
static bool bn_fused_finish(size_t chunks) { return (chunks + 255) / 256 <= 1024; }
// room for the partials of the BatchNorm's own sums kernels or of the convolution that produced its input (one row of
// pixels per BatchNorm row), whichever are more
size_t bn_bf16_partial_floats(int rows, int C) {
  const long a = bn_blocks(rows, C), b = conv_mfma_blocks(rows);
  return (size_t)(a > b ? a : b) * 2 * C;
}

// The three helpers need channel counts that are multiples of 8, 16-byte aligned tensors and fewer than 2^31 elements.
bool eltwise_bf16_ok(int dt, size_t elems, int C0, int C1, const void* a, const void* b, const void* c) {
  return dt == BF16 && (C0 % 8) == 0 && (C1 % 8) == 0 && elems < ((size_t)1 << 31) && al16(a) && al16(b) && al16(c);
}
// C a multiple of 8 that divides 256 * 8 into whole pixel lanes, at most 256 channels
bool gap_fwd_bf16_ok(int dt, int C, const void* x, const void* pooled) {
  return dt == BF16 && (C % 8) == 0 && C >= 8 && C <= 256 && (256 % (C / 8)) == 0 && al16(x) && !(((uintptr_t)pooled) & 1);
}
int launch_gap_fwd_bf16(hipStream_t s, const void* x, int B, int HW, int C, void* pooled) {
  hipLaunchKernelGGL(gap_fwd_bf16_kernel, dim3(B), dim3(256), 0, s, (const uint16_t*)x, HW, C, (uint16_t*)pooled);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
int launch_gap_bwd_bf16(hipStream_t s, const void* dpooled, int B, int HW, int C, void* dx) {
  const uint32_t chunks = (uint32_t)((size_t)B * HW * C / 8);
  hipLaunchKernelGGL(gap_bwd_bf16_kernel, dim3((chunks + 255) / 256), dim3(256), 0, s, (const uint16_t*)dpooled, (uint32_t)HW,
                     (uint32_t)C, chunks, (uint16_t*)dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
int launch_shortcut_fwd_bf16(hipStream_t s, const void* x, int B, int H, int W, int Ci, int Co, int stride, void* y) {
  const uint32_t Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  const uint32_t chunks = (uint32_t)((size_t)B * Ho * Wo * Co / 8);
  hipLaunchKernelGGL(shortcut_fwd_bf16_kernel, dim3((chunks + 255) / 256), dim3(256), 0, s, (const uint16_t*)x, (uint32_t)H,
                     (uint32_t)W, (uint32_t)Ci, (uint32_t)Co, (uint32_t)stride, Ho, Wo, chunks, (uint16_t*)y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
int launch_shortcut_bwd_bf16(hipStream_t s, const void* dy, const void* ymask, int B, int H, int W, int Ci, int Co, int stride,
                             void* dx) {
  const uint32_t Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  const uint32_t chunks = (uint32_t)((size_t)B * Ho * Wo * Ci / 8);
  hipLaunchKernelGGL(shortcut_bwd_bf16_kernel, dim3((chunks + 255) / 256), dim3(256), 0, s, (const uint16_t*)dy,
                     (const uint16_t*)ymask, (uint32_t)H, (uint32_t)W, (uint32_t)Ci, (uint32_t)Co, (uint32_t)stride, Ho, Wo, chunks,
                     (uint16_t*)dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_bn_stats_bf16(hipStream_t s, const void* x, int rows, int C, float eps, float momentum, float* partials,
                         float* mean, float* rstd, float* run_mean, float* run_var) {
  BnSumArgs p{};
  p.x = (const uint16_t*)x; p.rows = rows; p.C = C; p.partial = partials; p.eps = eps;
  p.momentum = momentum; p.out0 = mean; p.out1 = rstd; p.run_mean = run_mean; p.run_var = run_var;
  PPLL_TRY(bn_sums_launch<0>(s, p, bn_blocks(rows, C), true));
  return PPLL_OK;
}

// statistics and y = relu(bn(x) (+ res)) of a training step
// ready_blocks > 0: `partials` already holds that many rows of sums, written by the convolution that produced x
int launch_bn_train_fwd_bf16(hipStream_t s, const void* x, int rows, int C, float eps, float momentum, float* partials,
                             float* mean, float* rstd, float* run_mean, float* run_var, const float* g, const float* b,
                             const void* res, void* y, int ready_blocks) {
  BnSumArgs p{};
  p.x = (const uint16_t*)x; p.rows = rows; p.C = C; p.partial = partials; p.eps = eps;
  p.momentum = momentum; p.out0 = mean; p.out1 = rstd; p.run_mean = run_mean; p.run_var = run_var;
  const size_t chunks = (size_t)rows * C / 8;
  const int blocks = ready_blocks > 0 ? ready_blocks : bn_blocks(rows, C);
  // every workgroup of the fused kernel adds up all partial rows itself: only worth it for few of both
  if (!bn_fused_finish(chunks) || blocks > 256) {
    if (ready_blocks > 0) {
      hipLaunchKernelGGL(bn_finish_kernel<0>, dim3(1), dim3(1024), 0, s, p, (unsigned)blocks);
      PPLL_HIP(hipGetLastError());
    } else {
      PPLL_TRY(bn_sums_launch<0>(s, p, blocks, true));
    }
    return launch_bn_apply_bf16(s, x, rows, C, mean, rstd, g, b, res, y);
  }
  if (ready_blocks <= 0) PPLL_TRY(bn_sums_launch<0>(s, p, blocks, false));
  hipLaunchKernelGGL(bn_apply_fused_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, p, (unsigned)blocks, chunks,
                     g, b, (const uint16_t*)res, (uint16_t*)y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

int launch_bn_apply_bf16(hipStream_t s, const void* x, int rows, int C, const float* mean, const float* rstd,
                         const float* g, const float* b, const void* res, void* y) {
  const size_t chunks = (size_t)rows * C / 8;
  hipLaunchKernelGGL(bn_apply_bf16_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, (const uint16_t*)x,
                     chunks, C, mean, rstd, g, b, (const uint16_t*)res, (uint16_t*)y);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

// ready_blocks > 0: `partials` already holds that many rows of the two sums, written by the convolution that produced dy
int launch_bn_bwd_bf16(hipStream_t s, const void* dy, const void* y, const void* x, int rows, int C, const float* mean,
                       const float* rstd, const float* g, float* partials, float* dg, float* db, void* dx, int ready_blocks) {
  BnSumArgs p{};
  p.x = (const uint16_t*)x; p.dy = (const uint16_t*)dy; p.y = (const uint16_t*)y; p.rows = rows; p.C = C;
  p.mean = mean; p.rstd = rstd; p.partial = partials; p.out0 = db; p.out1 = dg;
  const size_t chunks = (size_t)rows * C / 8;
  const int blocks = ready_blocks > 0 ? ready_blocks : bn_blocks(rows, C);
  if (bn_fused_finish(chunks) && blocks <= 256) {
    if (ready_blocks <= 0) PPLL_TRY(bn_sums_launch<1>(s, p, blocks, false));
    hipLaunchKernelGGL(bn_bwd_apply_fused_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, p, (unsigned)blocks,
                       chunks, g, (uint16_t*)dx);
    PPLL_HIP(hipGetLastError());
    return PPLL_OK;
  }
  if (ready_blocks > 0) {
    hipLaunchKernelGGL(bn_finish_kernel<1>, dim3(1), dim3(1024), 0, s, p, (unsigned)blocks);
    PPLL_HIP(hipGetLastError());
  } else {
    PPLL_TRY(bn_sums_launch<1>(s, p, blocks, true));
  }
  hipLaunchKernelGGL(bn_bwd_apply_bf16_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s,
                     (const uint16_t*)dy, (const uint16_t*)y, (const uint16_t*)x, chunks, C, rows, mean, rstd, g, dg, db,
                     (uint16_t*)dx);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

}  // namespace ppll
