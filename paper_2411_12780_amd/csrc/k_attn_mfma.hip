// Multi-head self-attention core for head dimension 64 in bf16 on the matrix
// cores, forward and backward, one workgroup per (batch, head), one wave per
// tile of 32 tokens (T <= 256).
//
// Layout trick.  v_mfma_f32_32x32x16_bf16 gives lane l column l%32 of the
// 32 x 32 result and 16 of its rows (8*(e/4) + 4*(l/32) + e%4).  Scores are
// therefore produced transposed, S^T = K Q^T: a lane owns one query and holds
// its scores against 16 of the 32 keys of a tile, so the row softmax is a
// reduction over the lane's own registers plus one exchange with lane l^32.
// The same registers, packed to bf16, are directly the second operand of the
// next product (O^T = V^T P^T, dQ^T = K^T dS^T): the k index of an MFMA may be
// assigned to (lane half, element) in any order as long as both operands agree,
// so the first operand is fetched with the matching key order.  P and dS never
// pass through memory.
//
// Every operand passes through LDS.  K, V, Q and dO tiles are copied there with
// coalesced 16-byte loads as [token][64] rows of 128 bytes whose 16-byte granule
// index is XORed with (token/2)%8: the copy's stores, the fragment reads (32
// tokens x one granule per half wave) and the reads of the transposer below are
// then free of bank conflicts without padding.  First operands whose reduction
// index is the token (V^T, K^T, Q^T, dO^T) are transposed once per workgroup into
// [64][T padded] arrays (8 bytes of padding per row) with an in-register 4 x 8
// transpose (v_perm_b32 on four 16-byte rows).
//
// Backward: phase A (wave = query tile) forms P and dS with a lane per query
// and accumulates dQ; phase B (wave = key tile) forms them again with a lane
// per key (scores recomputed in the other orientation instead of transposing
// registers) and accumulates dK and dV.  Four LDS regions are reused between the
// phases (A: K, V, K^T, dO;  B: Q, Q^T, dO^T, dO), which keeps a 96-token
// workgroup at 51 KB, three to a compute unit.  All sums run in a fixed order.
#include "common.h"

namespace ppll {

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16x8 ld_frag(const uint16_t* p, bool ok) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (ok) v = *reinterpret_cast<const uint4*>(p);
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ uint32_t pack2(float a, float b) { return f32x2_to_bf16x2(a, b); }
__device__ __forceinline__ bf16x8 pack8(const float* v) {
  uint4 u = make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
  return __builtin_bit_cast(bf16x8, u);
}
// two 8-byte halves (tokens t..t+3 and t+8..t+11 of one row of a transposed matrix)
__device__ __forceinline__ bf16x8 ld_tfrag(const char* row, int tok) {
  uint2 a = *reinterpret_cast<const uint2*>(row + 2 * tok);
  uint2 b = *reinterpret_cast<const uint2*>(row + 2 * tok + 16);
  return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
}

// ---- [token][64] bf16 tiles in LDS, 128-byte rows, granule swizzle
__device__ __forceinline__ int rm_off(int r, int g) { return r * 128 + ((g ^ ((r >> 1) & 7)) << 4); }
__device__ __forceinline__ bf16x8 lds_frag(const char* rm, int r, int g) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(rm + rm_off(r, g)));
}
// copies T rows of 64 bf16 (`ld` elements apart) into a tile of TP rows, zero beyond T
template <int TP>
__device__ __forceinline__ void stage_rows(const uint16_t* __restrict__ src, long ld, int T, char* rm, int tid) {
  constexpr int NT = 2 * TP;   // threads of the workgroup
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + NT * i, r = c >> 3, g = c & 7;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < T) v = *reinterpret_cast<const uint4*>(src + (long)r * ld + 8 * g);
    *reinterpret_cast<uint4*>(rm + rm_off(r, g)) = v;
  }
}
__device__ __forceinline__ void write_transposed(const uint4* r, char* dst, int RS, int dc, int j0) {
  const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&r[0]);
  const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&r[1]);
  const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&r[2]);
  const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&r[3]);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
    uint2 o;
    o.x = __builtin_amdgcn_perm(w1[i >> 1], w0[i >> 1], sel);
    o.y = __builtin_amdgcn_perm(w3[i >> 1], w2[i >> 1], sel);
    *reinterpret_cast<uint2*>(dst + (8 * dc + i) * RS + 2 * j0) = o;
  }
}
// LDS tile [TP][64] -> dst[64][TP] (row stride 2*TP+8 bytes); one 4 x 8 block per thread of the 2*TP
template <int TP>
__device__ __forceinline__ void transpose_tile(const char* rm, char* dst, int tid) {
  const int jg = tid >> 3, dc = tid & 7, j0 = 4 * jg;
  uint4 r[4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) r[jj] = *reinterpret_cast<const uint4*>(rm + rm_off(j0 + jj, dc));
  write_transposed(r, dst, 2 * TP + 8, dc, j0);
}
// global rows -> dst[64][TP], zero for tokens >= T
template <int TP>
__device__ __forceinline__ void transpose_to_lds(const uint16_t* __restrict__ src, long ld, int T, char* dst, int tid) {
  const int jg = tid >> 3, dc = tid & 7, j0 = 4 * jg;
  uint4 r[4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    r[jj] = make_uint4(0, 0, 0, 0);
    if (j0 + jj < T) r[jj] = *reinterpret_cast<const uint4*>(src + (long)(j0 + jj) * ld + 8 * dc);
  }
  write_transposed(r, dst, 2 * TP + 8, dc, j0);
}

constexpr float kScale = 0.125f;   // 1/sqrt(64)

template <int NKT>
__global__ __launch_bounds__(64 * NKT) void attn_fwd_mfma_kernel(const uint16_t* __restrict__ qkv, int T, int H,
                                                                 uint16_t* __restrict__ out,
                                                                 float* __restrict__ lse_out) {
  constexpr int TP = 32 * NKT, RS = 2 * TP + 8;
  extern __shared__ __align__(16) char smem[];
  char* vt = smem;              // V^T [64][TP]
  char* krm = smem + 64 * RS;   // K   [TP][64]
  const int b = blockIdx.x / H, h = blockIdx.x % H, D = 64 * H;
  const long ld = 3L * D;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const uint16_t* base = qkv + (size_t)b * T * ld + h * 64;
  const int qi = 32 * wave + li;
  bf16x8 qf[4];   // a wave's own queries: read once, straight from global memory, in flight with the copies below
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) qf[kk] = ld_frag(base + (long)qi * ld + 16 * kk + 8 * hh, qi < T);
  transpose_to_lds<TP>(base + 2 * D, ld, T, vt, tid);
  stage_rows<TP>(base + D, ld, T, krm, tid);
  __syncthreads();
  f32x16 s[NKT];
#pragma unroll
  for (int jt = 0; jt < NKT; ++jt) {
#pragma unroll
    for (int e = 0; e < 16; ++e) s[jt][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const bf16x8 kf = lds_frag(krm, 32 * jt + li, 2 * kk + hh);
      s[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[jt], 0, 0, 0);
    }
  }
  // softmax over the keys of query qi: s[jt][e] belongs to key 32*jt + 8*(e/4) + 4*hh + e%4
  float mx = -INFINITY;
#pragma unroll
  for (int jt = 0; jt < NKT; ++jt)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int key = 32 * jt + 8 * (e >> 2) + 4 * hh + (e & 3);
      const float v = key < T ? s[jt][e] * kScale : -INFINITY;
      s[jt][e] = v;
      mx = fmaxf(mx, v);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  float sum = 0.f;
#pragma unroll
  for (int jt = 0; jt < NKT; ++jt)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float p = __expf(s[jt][e] - mx);
      s[jt][e] = p;
      sum += p;
    }
  sum += __shfl_xor(sum, 32, 64);
  const float inv = 1.0f / sum;

  f32x16 o[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
#pragma unroll
  for (int jt = 0; jt < NKT; ++jt)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      float pv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pv[e] = s[jt][8 * half + e] * inv;
      const bf16x8 pf = pack8(pv);
      const int tok = 32 * jt + 16 * half + 4 * hh;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const bf16x8 vf = ld_tfrag(vt + (32 * dt + li) * RS, tok);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[dt], 0, 0, 0);
      }
    }
  if (qi < T) {
    uint16_t* orow = out + ((size_t)b * T + qi) * D + h * 64;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 w = make_uint2(pack2(o[dt][4 * q], o[dt][4 * q + 1]), pack2(o[dt][4 * q + 2], o[dt][4 * q + 3]));
        *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * q + 4 * hh) = w;
      }
    if (hh == 0) lse_out[((size_t)b * H + h) * T + qi] = mx + __logf(sum);
  }
}

template <int NKT>
__global__ __launch_bounds__(64 * NKT, (NKT <= 4 ? 3 : 2)) void attn_bwd_mfma_kernel(const uint16_t* __restrict__ qkv,
                                                                 const uint16_t* __restrict__ out,
                                                                 const uint16_t* __restrict__ dout,
                                                                 const float* __restrict__ lse, int T, int H,
                                                                 uint16_t* __restrict__ dqkv) {
  constexpr int TP = 32 * NKT, RS = 2 * TP + 8;
  extern __shared__ __align__(16) char smem[];
  constexpr int REG = 64 * RS;     // one region: a [TP][64] tile (TP*128 bytes) or a [64][TP] transposed one
  char* r0 = smem;                 // phase A: K        phase B: Q
  char* r1 = smem + REG;           // phase A: V        phase B: Q^T
  char* r2 = smem + 2 * REG;       // phase A: K^T      phase B: dO^T
  char* r3 = smem + 3 * REG;       // both phases: dO
  float* Dsh = reinterpret_cast<float*>(smem + 4 * REG);  // [TP] <dO_i, O_i>
  float* Lsh = Dsh + TP;                                  // [TP] log-sum-exp
  const int b = blockIdx.x / H, h = blockIdx.x % H, D = 64 * H;
  const long ld = 3L * D;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, hh = lane >> 5;
  constexpr int NT = 64 * NKT;
  const uint16_t* base = qkv + (size_t)b * T * ld + h * 64;
  const uint16_t* obase = out + (size_t)b * T * D + h * 64;
  const uint16_t* dobase = dout + (size_t)b * T * D + h * 64;
  // K, V, dO -> LDS; D_i = <dO_i, O_i> from the same pass: 8 lanes per token, then a 3-step exchange
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + NT * i, r = c >> 3, g = c & 7;
    uint4 kv = make_uint4(0, 0, 0, 0), vv = kv, dov = kv, ov = kv;
    if (r < T) {
      kv = *reinterpret_cast<const uint4*>(base + (long)r * ld + D + 8 * g);
      vv = *reinterpret_cast<const uint4*>(base + (long)r * ld + 2 * D + 8 * g);
      dov = *reinterpret_cast<const uint4*>(dobase + (long)r * D + 8 * g);
      ov = *reinterpret_cast<const uint4*>(obase + (long)r * D + 8 * g);
    }
    const int off = rm_off(r, g);
    *reinterpret_cast<uint4*>(r0 + off) = kv;
    *reinterpret_cast<uint4*>(r1 + off) = vv;
    *reinterpret_cast<uint4*>(r3 + off) = dov;
    const uint32_t* aw = reinterpret_cast<const uint32_t*>(&dov);
    const uint32_t* ow = reinterpret_cast<const uint32_t*>(&ov);
    float dd = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      dd += __uint_as_float(aw[w] << 16) * __uint_as_float(ow[w] << 16) +
            __uint_as_float(aw[w] & 0xffff0000u) * __uint_as_float(ow[w] & 0xffff0000u);
    dd += __shfl_xor(dd, 1, 64);
    dd += __shfl_xor(dd, 2, 64);
    dd += __shfl_xor(dd, 4, 64);
    if (g == 0) {
      Dsh[r] = dd;
      Lsh[r] = r < T ? lse[((size_t)b * H + h) * T + r] : 0.f;
    }
  }
  __syncthreads();
  transpose_tile<TP>(r0, r2, tid);   // K^T
  __syncthreads();

  // ---------------- phase A: wave = query tile, lane = query; dQ
  {
    const int qi = 32 * wave + li;
    bf16x8 qf[4], dof[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      qf[kk] = ld_frag(base + (long)qi * ld + 16 * kk + 8 * hh, qi < T);
      dof[kk] = lds_frag(r3, qi, 2 * kk + hh);
    }
    const float lse_i = Lsh[qi], d_i = Dsh[qi];
    f32x16 dq[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[dt][e] = 0.f;
#pragma unroll 1
    for (int jt = 0; jt < NKT; ++jt) {
      const int kj = 32 * jt + li;
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 kf = lds_frag(r0, kj, 2 * kk + hh);
        const bf16x8 vf = lds_frag(r1, kj, 2 * kk + hh);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[kk], dp, 0, 0, 0);
      }
      float ds[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = 32 * jt + 8 * (e >> 2) + 4 * hh + (e & 3);
        const float p = key < T ? __expf(s[e] * kScale - lse_i) : 0.f;
        ds[e] = p * (dp[e] - d_i);
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const bf16x8 dsf = pack8(ds + 8 * half);
        const int tok = 32 * jt + 16 * half + 4 * hh;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          const bf16x8 ktf = ld_tfrag(r2 + (32 * dt + li) * RS, tok);
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf, dq[dt], 0, 0, 0);
        }
      }
    }
    if (qi < T) {
      uint16_t* row = dqkv + ((size_t)b * T + qi) * ld + h * 64;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 w = make_uint2(pack2(dq[dt][4 * q] * kScale, dq[dt][4 * q + 1] * kScale),
                               pack2(dq[dt][4 * q + 2] * kScale, dq[dt][4 * q + 3] * kScale));
          *reinterpret_cast<uint2*>(row + 32 * dt + 8 * q + 4 * hh) = w;
        }
    }
  }

  // ---------------- phase B: wave = key tile, lane = key; dK, dV
  {
    const int kj = 32 * wave + li;
    bf16x8 kf[4], vf[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      kf[kk] = lds_frag(r0, kj, 2 * kk + hh);
      vf[kk] = lds_frag(r1, kj, 2 * kk + hh);
    }
    __syncthreads();                               // every wave is done with K, V and K^T
    stage_rows<TP>(base, ld, T, r0, tid);          // Q
    transpose_tile<TP>(r3, r2, tid);               // dO^T
    __syncthreads();
    transpose_tile<TP>(r0, r1, tid);               // Q^T
    __syncthreads();
    f32x16 dk[2], dv[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) { dk[dt][e] = 0.f; dv[dt][e] = 0.f; }
#pragma unroll 1
    for (int it = 0; it < NKT; ++it) {
      const int qrow = 32 * it + li;
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 qf = lds_frag(r0, qrow, 2 * kk + hh);
        const bf16x8 dof = lds_frag(r3, qrow, 2 * kk + hh);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[kk], s, 0, 0, 0);     // rows = queries, lane = key
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dof, vf[kk], dp, 0, 0, 0);
      }
      float p[16], ds[16];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int q0 = 32 * it + 8 * q4 + 4 * hh;
        const float4 l4 = *reinterpret_cast<const float4*>(Lsh + q0);
        const float4 d4 = *reinterpret_cast<const float4*>(Dsh + q0);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float pe = (q0 + e) < T ? __expf(s[4 * q4 + e] * kScale - lv[e]) : 0.f;
          p[4 * q4 + e] = pe;
          ds[4 * q4 + e] = pe * (dp[4 * q4 + e] - dvv[e]);
        }
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const bf16x8 pf = pack8(p + 8 * half), dsf = pack8(ds + 8 * half);
        const int tok = 32 * it + 16 * half + 4 * hh;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          const bf16x8 dotf = ld_tfrag(r2 + (32 * dt + li) * RS, tok);
          const bf16x8 qtf = ld_tfrag(r1 + (32 * dt + li) * RS, tok);
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dotf, pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtf, dsf, dk[dt], 0, 0, 0);
        }
      }
    }
    if (kj < T) {
      uint16_t* row = dqkv + ((size_t)b * T + kj) * ld + h * 64;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 wk = make_uint2(pack2(dk[dt][4 * q] * kScale, dk[dt][4 * q + 1] * kScale),
                                pack2(dk[dt][4 * q + 2] * kScale, dk[dt][4 * q + 3] * kScale));
          uint2 wv = make_uint2(pack2(dv[dt][4 * q], dv[dt][4 * q + 1]), pack2(dv[dt][4 * q + 2], dv[dt][4 * q + 3]));
          *reinterpret_cast<uint2*>(row + D + 32 * dt + 8 * q + 4 * hh) = wk;
          *reinterpret_cast<uint2*>(row + 2 * D + 32 * dt + 8 * q + 4 * hh) = wv;
        }
    }
  }
}

#define ATTN_DISPATCH(NKT_VALUE, CALL)                \
  switch (NKT_VALUE) {                                \
    case 1: { constexpr int NKT = 1; CALL; break; }   \
    case 2: { constexpr int NKT = 2; CALL; break; }   \
    case 3: { constexpr int NKT = 3; CALL; break; }   \
    case 4: { constexpr int NKT = 4; CALL; break; }   \
    case 5: { constexpr int NKT = 5; CALL; break; }   \
    case 6: { constexpr int NKT = 6; CALL; break; }   \
    case 7: { constexpr int NKT = 7; CALL; break; }   \
    default: { constexpr int NKT = 8; CALL; break; }  \
  }

template <int NKT>
int launch_fwd(hipStream_t s, const uint16_t* qkv, int B, int T, int H, uint16_t* out, float* lse) {
  constexpr int TP = 32 * NKT, RS = 2 * TP + 8;
  const size_t lds = (size_t)64 * RS + (size_t)TP * 128;
  if (lds > 64 * 1024)
    PPLL_HIP(hipFuncSetAttribute((const void*)attn_fwd_mfma_kernel<NKT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)lds));
  hipLaunchKernelGGL((attn_fwd_mfma_kernel<NKT>), dim3(B * H), dim3(64 * NKT), lds, s, qkv, T, H, out, lse);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}

template <int NKT>
int launch_bwd(hipStream_t s, const uint16_t* qkv, const uint16_t* out, const uint16_t* dout, const float* lse, int B,
               int T, int H, uint16_t* dqkv) {
  constexpr int TP = 32 * NKT, RS = 2 * TP + 8;
  const size_t lds = (size_t)4 * 64 * RS + 2 * TP * sizeof(float);   // 135 KB at T = 256
  if (lds > 64 * 1024)
    PPLL_HIP(hipFuncSetAttribute((const void*)attn_bwd_mfma_kernel<NKT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)lds));
  hipLaunchKernelGGL((attn_bwd_mfma_kernel<NKT>), dim3(B * H), dim3(64 * NKT), lds, s, qkv, out, dout, lse, T, H, dqkv);
  PPLL_HIP(hipGetLastError());
  return PPLL_OK;
}
}  // namespace

bool attention_mfma_supported(int dt, int T, int H, int dh, const void* a, const void* b, const void* c, const void* d) {
  if (dt != BF16 || dh != 64 || T < 1 || T > 256 || H < 1) return false;
  return !((((uintptr_t)a) | ((uintptr_t)b) | ((uintptr_t)c) | ((uintptr_t)d)) & 15);
}

int launch_attention_fwd_mfma(hipStream_t s, const void* qkv, int B, int T, int H, void* out, float* lse) {
  int st = PPLL_OK;
  ATTN_DISPATCH((T + 31) / 32, st = launch_fwd<NKT>(s, (const uint16_t*)qkv, B, T, H, (uint16_t*)out, lse));
  return st;
}

int launch_attention_bwd_mfma(hipStream_t s, const void* qkv, const void* out, const void* dout, const float* lse,
                              int B, int T, int H, void* dqkv) {
  int st = PPLL_OK;
  ATTN_DISPATCH((T + 31) / 32, st = launch_bwd<NKT>(s, (const uint16_t*)qkv, (const uint16_t*)out,
                                                     (const uint16_t*)dout, lse, B, T, H, (uint16_t*)dqkv));
  return st;
}

}  // namespace ppll
