// bf16 GEMM on the CDNA4 matrix cores: C[M,N] = A(M,K) . B(K,N), fp32
// accumulation in v_mfma_f32_32x32x16_bf16, operands staged through LDS.
//
// One 256-thread workgroup (4 waves, 2 x 2) owns a 128 x 128 output tile and
// walks K in steps of 64; each wave owns 64 x 64 = 2 x 2 MFMA tiles.  Both
// operands live in LDS as [row][k] with k contiguous, which is what an MFMA
// operand fragment wants (a lane holds 8 consecutive k of one row).  An operand
// whose k is contiguous in memory (activations in Y = X W^T-style products, the
// [in,out] weight in dX = dY W^T) is copied with 16-byte loads; an operand whose
// other index is contiguous (the [in,out] weight in Y = X W, both operands of
// dW = X^T dY) is transposed in registers on the way in, so no transposed copies
// of weights or activations exist in HBM.
//
// LDS rows are 144 bytes apart (128 of data + 16 of padding) and the 16-byte
// k-granule index is XORed with (row / 16) % 8: with that layout the fragment
// reads (ds_read_b128, 32 rows x 2 granules per wave) and the 8-byte writes of
// the transposing loader are both free of bank conflicts.
//
// The MFMA is issued with the B tile as its first operand, i.e. it produces C
// transposed: a lane then holds 4 consecutive columns of one C row, so bias,
// residual, saved pre-activation and the output move as 8/16-byte vectors.
//
// Split-K (weight gradients: tiny outputs, reduction over all tokens): every
// split writes its fp32 partial tile, a second kernel adds the splits in a
// fixed order, so results are reproducible (no float atomics).
#include "common.h"

namespace ppll {

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int ROW_BYTES = 144;

struct MfmaArgs {
  const uint16_t* A; long lda;      // AT ? A[k*lda + m] : A[m*lda + k]
  const uint16_t* B; long ldb;      // BT ? B[k*ldb + n] : B[n*ldb + k]
  void* C; int c_f32; long ldc;
  int M, N, K;
  int tiles_m, tiles_n;
  int kt_per_split;                 // k-tiles per split
  float* partial;                   // [splits][M][N] when split-K
  float* colsum;                    // optional: [splits][N] sums over k of B(k, n) (bias gradient), else null
  const float* bias;
  const uint16_t* residual; long ldr;
  int epilogue;
  uint16_t* C2;
  const uint16_t* aux; long ldaux;
};

__device__ __forceinline__ float gelu_f(float h) { return 0.5f * h * (1.0f + erff(h * 0.70710678118654752f)); }
__device__ __forceinline__ float dgelu_f(float h) {
  float cdf = 0.5f * (1.0f + erff(h * 0.70710678118654752f));
  float pdf = 0.39894228040143268f * __expf(-0.5f * h * h);
  return cdf + h * pdf;
}

__device__ __forceinline__ int lds_off(int row, int granule16) {
  return row * ROW_BYTES + ((granule16 ^ ((row >> 4) & 7)) << 4);
}

// k contiguous in memory: 4 chunks of 8 bf16 per thread
template <int ROWS>
__device__ __forceinline__ void load_direct(const uint16_t* __restrict__ base, long ld, int row0, int nrows, int k0,
                                            int kend, int tid, uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = tid + 256 * i, row = c >> 3, g = c & 7;
    int k = k0 + g * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row0 + row < nrows && k < kend) v = *reinterpret_cast<const uint4*>(base + (long)(row0 + row) * ld + k);
    r[i] = v;
  }
}
__device__ __forceinline__ void store_direct(char* lds, int tid, const uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = tid + 256 * i, row = c >> 3, g = c & 7;
    *reinterpret_cast<uint4*>(lds + lds_off(row, g)) = r[i];
  }
}

// the row index contiguous in memory: thread (mg, kg) takes rows mg*8..+7 and k = kg*4..+3
__device__ __forceinline__ void load_transposed(const uint16_t* __restrict__ base, long ld, int row0, int nrows, int k0,
                                                int kend, int tid, uint4 (&r)[4]) {
  int mg = tid & 15, kg = tid >> 4;
  int row = row0 + mg * 8;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int k = k0 + kg * 4 + j;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < nrows && k < kend) v = *reinterpret_cast<const uint4*>(base + (long)k * ld + row);
    r[j] = v;
  }
}
__device__ __forceinline__ void store_transposed(char* lds, int tid, const uint4 (&r)[4]) {
  int mg = tid & 15, kg = tid >> 4;
  const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&r[0]);
  const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&r[1]);
  const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&r[2]);
  const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&r[3]);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
    uint2 o;
    o.x = __builtin_amdgcn_perm(w1[i >> 1], w0[i >> 1], sel);   // k, k+1
    o.y = __builtin_amdgcn_perm(w3[i >> 1], w2[i >> 1], sel);   // k+2, k+3
    int row = mg * 8 + i;
    *reinterpret_cast<uint2*>(lds + lds_off(row, kg >> 1) + (kg & 1) * 8) = o;
  }
}

template <bool AT, bool BT>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(MfmaArgs p) {
  __shared__ __align__(16) char lds_a[BM * ROW_BYTES];
  __shared__ __align__(16) char lds_b[BN * ROW_BYTES];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int tile = blockIdx.x;
  const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
  const int split = blockIdx.y;
  const int nkt = (p.K + BK - 1) / BK;
  const int kt0 = split * p.kt_per_split;
  const int kt1 = min(nkt, kt0 + p.kt_per_split);

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  uint4 ra[4], rb[4];
  auto load_tiles = [&](int kt) {
    int k0 = kt * BK;
    if (AT) load_transposed(p.A, p.lda, m0, p.M, k0, p.K, tid, ra);
    else load_direct<BM>(p.A, p.lda, m0, p.M, k0, p.K, tid, ra);
    if (BT) load_transposed(p.B, p.ldb, n0, p.N, k0, p.K, tid, rb);
    else load_direct<BN>(p.B, p.ldb, n0, p.N, k0, p.K, tid, rb);
  };
  if (kt0 < kt1) load_tiles(kt0);
  const int frag_row = lane & 31, frag_g = lane >> 5;
  // bias gradient riding along: the workgroups of the first tile row also add up their B tile over k
  const bool do_colsum = p.colsum != nullptr && m0 == 0;
  float csum = 0.f;
  for (int kt = kt0; kt < kt1; ++kt) {
    __syncthreads();
    if (AT) store_transposed(lds_a, tid, ra); else store_direct(lds_a, tid, ra);
    if (BT) store_transposed(lds_b, tid, rb); else store_direct(lds_b, tid, rb);
    __syncthreads();
    if (kt + 1 < kt1) load_tiles(kt + 1);
    if (do_colsum) {   // thread (row = tid/2, half = tid%2) sums 4 of the row's 8 granules; their order is irrelevant
      const char* rowp = lds_b + (tid >> 1) * ROW_BYTES + (tid & 1) * 64;
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        uint4 w = *reinterpret_cast<const uint4*>(rowp + gq * 16);
        csum += bf16_to_f32((uint16_t)(w.x & 0xffff)) + bf16_to_f32((uint16_t)(w.x >> 16)) +
                bf16_to_f32((uint16_t)(w.y & 0xffff)) + bf16_to_f32((uint16_t)(w.y >> 16)) +
                bf16_to_f32((uint16_t)(w.z & 0xffff)) + bf16_to_f32((uint16_t)(w.z >> 16)) +
                bf16_to_f32((uint16_t)(w.w & 0xffff)) + bf16_to_f32((uint16_t)(w.w >> 16));
      }
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int im = 0; im < 2; ++im)
        fa[im] = *reinterpret_cast<const bf16x8*>(lds_a + lds_off(wm * 64 + im * 32 + frag_row, kk * 2 + frag_g));
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
        fb[jn] = *reinterpret_cast<const bf16x8*>(lds_b + lds_off(wn * 64 + jn * 32 + frag_row, kk * 2 + frag_g));
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int im = 0; im < 2; ++im)
          acc[jn][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[jn], fa[im], acc[jn][im], 0, 0, 0);
    }
  }

  if (do_colsum) {
    csum += __shfl_xor(csum, 1, 64);
    const int n = n0 + (tid >> 1);
    if (!(tid & 1) && n < p.N) p.colsum[(size_t)split * p.N + n] = csum;
  }
  // acc[jn][im][4q + e] = C[m][n] with m = m0 + wm*64 + im*32 + lane%32, n = n0 + wn*64 + jn*32 + 8q + 4*(lane/32) + e
#pragma unroll
  for (int im = 0; im < 2; ++im) {
    const int m = m0 + wm * 64 + im * 32 + (lane & 31);
    if (m >= p.M) continue;
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * 64 + jn * 32 + 8 * q + 4 * (lane >> 5);
        if (n >= p.N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[jn][im][4 * q + e];
        if (p.partial) {
          *reinterpret_cast<float4*>(p.partial + ((size_t)split * p.M + m) * p.N + n) = make_float4(v[0], v[1], v[2], v[3]);
          continue;
        }
        if (p.bias) {
          float4 b = *reinterpret_cast<const float4*>(p.bias + n);
          v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
        }
        if (p.residual) {
          uint2 r = *reinterpret_cast<const uint2*>(p.residual + (size_t)m * p.ldr + n);
          v[0] += bf16_to_f32((uint16_t)(r.x & 0xffff)); v[1] += bf16_to_f32((uint16_t)(r.x >> 16));
          v[2] += bf16_to_f32((uint16_t)(r.y & 0xffff)); v[3] += bf16_to_f32((uint16_t)(r.y >> 16));
        }
        if (p.epilogue == EPI_DGELU) {
          uint2 h = *reinterpret_cast<const uint2*>(p.aux + (size_t)m * p.ldaux + n);
          v[0] *= dgelu_f(bf16_to_f32((uint16_t)(h.x & 0xffff))); v[1] *= dgelu_f(bf16_to_f32((uint16_t)(h.x >> 16)));
          v[2] *= dgelu_f(bf16_to_f32((uint16_t)(h.y & 0xffff))); v[3] *= dgelu_f(bf16_to_f32((uint16_t)(h.y >> 16)));
        }
        if (p.c_f32) {
          *reinterpret_cast<float4*>((float*)p.C + (size_t)m * p.ldc + n) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
          uint2 o;
          o.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
          o.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
          *reinterpret_cast<uint2*>((uint16_t*)p.C + (size_t)m * p.ldc + n) = o;
          if (p.epilogue == EPI_GELU) {
            uint2 g;
            g.x = (uint32_t)f32_to_bf16(gelu_f(v[0])) | ((uint32_t)f32_to_bf16(gelu_f(v[1])) << 16);
            g.y = (uint32_t)f32_to_bf16(gelu_f(v[2])) | ((uint32_t)f32_to_bf16(gelu_f(v[3])) << 16);
            *reinterpret_cast<uint2*>(p.C2 + (size_t)m * p.ldc + n) = g;
          }
        }
      }
    }
  }
}

// C[i] = sum over splits of partial[s][i], fixed order
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* partial, int splits, size_t mn, float* C) {
  size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= mn) return;
  float4 acc = *reinterpret_cast<const float4*>(partial + i);
  for (int s = 1; s < splits; ++s) {
    float4 v = *reinterpret_cast<const float4*>(partial + (size_t)s * mn + i);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  *reinterpret_cast<float4*>(C + i) = acc;
}

bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }
}  // namespace

// True when the MFMA kernel can take this product as it stands.
bool gemm_mfma_supported(const GemmArgs& g) {
  if (g.a_dt != BF16 || g.b_dt != BF16) return false;
  if (g.M < 1 || g.N < 1 || g.K < 1 || (g.N & 7) || (g.K & 7)) return false;
  const bool at = g.a_sm == 1 && g.a_sk != 1, bt = g.b_sn == 1 && g.b_sk != 1;
  if (!at && g.a_sk != 1) return false;
  if (!bt && g.b_sk != 1) return false;
  const long lda = at ? g.a_sk : g.a_sm, ldb = bt ? g.b_sk : g.b_sn;
  if ((lda & 7) || (ldb & 7) || (g.ldc & 3)) return false;
  if (at && (g.M & 7)) return false;
  if (!aligned16(g.A) || !aligned16(g.B) || !aligned16(g.C)) return false;
  if (g.bias && !aligned16(g.bias)) return false;
  if (g.residual && (g.r_dt != BF16 || (g.ldr & 3) || !aligned16(g.residual))) return false;
  if (g.epilogue == EPI_GELU && (g.c_dt != BF16 || !g.C2 || !aligned16(g.C2))) return false;
  if (g.epilogue == EPI_DGELU && (g.aux_dt != BF16 || (g.ldaux & 3) || !aligned16(g.aux))) return false;
  if (g.c_dt == BF16 && (g.ldc & 3)) return false;
  return true;
}

// Number of K splits for a product (1 = none) and the partial floats it needs.
int gemm_mfma_splits(int M, int N, int K) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int nkt = (K + BK - 1) / BK;
  if (tiles >= 128 || nkt < 8) return 1;
  int splits = (256 + tiles - 1) / tiles;          // about one workgroup per compute unit
  if (splits > nkt / 2) splits = nkt / 2;
  int per = (nkt + splits - 1) / splits;
  return (nkt + per - 1) / per;
}
size_t gemm_mfma_partial_floats(int M, int N, int K) {
  int s = gemm_mfma_splits(M, N, K);
  return s > 1 ? (size_t)s * M * N + (size_t)s * N : 0;   // tile partials, then bias-gradient partials
}

int launch_gemm_mfma(hipStream_t s, const GemmArgs& g, float* partial, size_t partial_floats) {
  const bool at = g.a_sm == 1 && g.a_sk != 1, bt = g.b_sn == 1 && g.b_sk != 1;
  MfmaArgs p{};
  p.A = (const uint16_t*)g.A; p.lda = at ? g.a_sk : g.a_sm;
  p.B = (const uint16_t*)g.B; p.ldb = bt ? g.b_sk : g.b_sn;
  p.C = g.C; p.c_f32 = g.c_dt == F32; p.ldc = g.ldc;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.tiles_m = (g.M + BM - 1) / BM; p.tiles_n = (g.N + BN - 1) / BN;
  p.bias = g.bias; p.residual = (const uint16_t*)g.residual; p.ldr = g.ldr;
  p.epilogue = g.epilogue; p.C2 = (uint16_t*)g.C2; p.aux = (const uint16_t*)g.aux; p.ldaux = g.ldaux;
  const int nkt = (g.K + BK - 1) / BK;
  int splits = 1;
  const bool plain = !g.bias && !g.residual && g.epilogue == EPI_NONE && g.c_dt == F32 && g.ldc == g.N;
  if (plain && partial) {
    splits = gemm_mfma_splits(g.M, g.N, g.K);
    if ((size_t)splits * g.M * g.N + (size_t)splits * g.N > partial_floats) splits = 1;
  }
  float* colsum_partial = splits > 1 ? partial + (size_t)splits * g.M * g.N : nullptr;
  p.colsum = g.colsum ? (splits > 1 ? colsum_partial : g.colsum) : nullptr;
  p.kt_per_split = (nkt + splits - 1) / splits;
  p.partial = splits > 1 ? partial : nullptr;
  dim3 grid(p.tiles_m * p.tiles_n, splits);
  if (at && bt) hipLaunchKernelGGL((gemm_mfma_kernel<true, true>), grid, dim3(256), 0, s, p);
  else if (at) hipLaunchKernelGGL((gemm_mfma_kernel<true, false>), grid, dim3(256), 0, s, p);
  else if (bt) hipLaunchKernelGGL((gemm_mfma_kernel<false, true>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((gemm_mfma_kernel<false, false>), grid, dim3(256), 0, s, p);
  PPLL_HIP(hipGetLastError());
  if (splits > 1) {
    size_t mn = (size_t)g.M * g.N;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((mn / 4 + 255) / 256), dim3(256), 0, s, partial, splits, mn, (float*)g.C);
    PPLL_HIP(hipGetLastError());
    if (g.colsum) PPLL_TRY(reduce_partials(s, colsum_partial, splits, g.N, g.N, 1.0f, g.colsum));
  }
  return PPLL_OK;
}

}  // namespace ppll
