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
#ifdef PPLL_GEMM_TRACE
  long long* trace;                 // [workgroup][8] wall-clock stamps (development builds only)
#endif
  int xcd_map;                      // 1: ids 8 apart share a tile row (many tile rows), 2: ids 8 apart share a
                                    // split (split-K), 0: row-major ids
  int splits;
};

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
__device__ __forceinline__ float gelu_fast(float h) { float c, d; cdf_pdf(h, c, d); return h * c; }
__device__ __forceinline__ float dgelu_fast(float h) { float c, d; cdf_pdf(h, c, d); return c + h * d; }
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

__device__ __forceinline__ int lds_off(int row, int granule16) {
  return row * ROW_BYTES + ((granule16 ^ ((row >> 4) & 7)) << 4);
}

// k contiguous in memory: ROWS/32 chunks of 8 bf16 per thread
template <int ROWS>
__device__ __forceinline__ void load_direct(const uint16_t* __restrict__ base, long ld, int row0, int nrows, int k0,
                                            int kend, int tid, uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    int c = tid + 256 * i, row = c >> 3, g = c & 7;
    int k = k0 + g * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row0 + row < nrows && k < kend) v = *reinterpret_cast<const uint4*>(base + (long)(row0 + row) * ld + k);
    r[i] = v;
  }
}
template <int ROWS>
__device__ __forceinline__ void store_direct(char* lds, int tid, const uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
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

constexpr int STAGE_LD = BN + 4;                      // fp32 staging tile of the epilogue, padded row
constexpr int oper_bytes(int tm) { return (tm + BN) * ROW_BYTES; }   // one stage of both operand tiles
constexpr int lds_bytes(int tm) { return 2 * oper_bytes(tm); }        // two stages; the epilogue tile reuses them
static_assert(BM * STAGE_LD * 4 <= lds_bytes(BM) && 64 * STAGE_LD * 4 <= lds_bytes(64),
              "epilogue staging tile must fit in the operand stages");

struct TileRegs { uint4 a[4], b[4]; };

// TM = rows of the output tile: 128 (wave tile 64 x 64) or, for outputs with too few 128-row
// tiles to fill the chip, 64 (wave tile 32 x 64; direct A loader only).
// PF = k-tiles in flight in registers ahead of the one being multiplied (4 measured slower than 2).
template <bool AT, bool BT, int TM, int PF = 2>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(MfmaArgs p) {
  static_assert(TM == 128 || (TM == 64 && !AT), "64-row tiles are for the direct A loader");
  constexpr int IM = TM / 64;                  // 32-row MFMA tiles per wave along m
  constexpr int OPER_BYTES = oper_bytes(TM);
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  // Workgroup id -> tile.  Consecutive ids go to the 8 XCDs round-robin and each XCD has its own
  // L2, so the tiles of one row (they share the A panel) are given ids that are 8 apart: they
  // land on one XCD, next to each other in its dispatch order, and the panel is fetched once.
  // With split-K (xcd_map 2) it is the splits that are dealt to the XCDs: all tiles of one k-range
  // run on one XCD, so the two token panels of that range are fetched from HBM once.
  int tm, tn, split = blockIdx.y;
  if (p.xcd_map == 1) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    tm = (slot / p.tiles_n) * 8 + xcd; tn = slot % p.tiles_n;
    if (tm >= p.tiles_m) return;
  } else if (p.xcd_map == 2) {
    const int tiles = p.tiles_m * p.tiles_n;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    split = (slot / tiles) * 8 + xcd;
    const int tile = slot % tiles;
    tm = tile / p.tiles_n; tn = tile % p.tiles_n;
    if (split >= p.splits) return;
  } else {
    tm = blockIdx.x / p.tiles_n; tn = blockIdx.x % p.tiles_n;
  }
  const int m0 = tm * TM, n0 = tn * BN;
  const int nkt = (p.K + BK - 1) / BK;
  const int kt0 = split * p.kt_per_split;
  const int nk = min(nkt, kt0 + p.kt_per_split) - kt0;

  f32x16 acc[2][IM];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < IM; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // Software pipeline: two LDS stages and PF register sets, so that the global loads of k-tiles
  // i+2 .. i+1+PF are in flight while tile i is multiplied and tile i+1 is written to LDS.
  const int frag_row = lane & 31, frag_g = lane >> 5;
  auto gload = [&](int i, TileRegs& r) {
    const int k0 = (kt0 + i) * BK;
    if (AT) load_transposed(p.A, p.lda, m0, p.M, k0, p.K, tid, r.a);
    else load_direct<TM>(p.A, p.lda, m0, p.M, k0, p.K, tid, r.a);
    if (BT) load_transposed(p.B, p.ldb, n0, p.N, k0, p.K, tid, r.b);
    else load_direct<BN>(p.B, p.ldb, n0, p.N, k0, p.K, tid, r.b);
  };
  auto lstore = [&](int stage, const TileRegs& r) {
    char* la = smem + stage * OPER_BYTES;
    char* lb = la + TM * ROW_BYTES;
    if (AT) store_transposed(la, tid, r.a); else store_direct<TM>(la, tid, r.a);
    if (BT) store_transposed(lb, tid, r.b); else store_direct<BN>(lb, tid, r.b);
  };
  // bias gradient riding along: the workgroups of the first tile row also add up their B tile over k
  const bool do_colsum = p.colsum != nullptr && m0 == 0;
  float csum = 0.f;
  auto compute = [&](int stage) {
    const char* la = smem + stage * OPER_BYTES;
    const char* lb = la + TM * ROW_BYTES;
    if (do_colsum) {   // thread (row = tid/2, half = tid%2) sums 4 of the row's 8 granules; their order is irrelevant
      const char* rowp = lb + (tid >> 1) * ROW_BYTES + (tid & 1) * 64;
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
      bf16x8 fa[IM], fb[2];
#pragma unroll
      for (int im = 0; im < IM; ++im)
        fa[im] = *reinterpret_cast<const bf16x8*>(la + lds_off(wm * (TM / 2) + im * 32 + frag_row, kk * 2 + frag_g));
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
        fb[jn] = *reinterpret_cast<const bf16x8*>(lb + lds_off(wn * 64 + jn * 32 + frag_row, kk * 2 + frag_g));
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int im = 0; im < IM; ++im)
          acc[jn][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[jn], fa[im], acc[jn][im], 0, 0, 0);
    }
  };

#ifdef PPLL_GEMM_TRACE
  long long* tr = p.trace + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 8;
  if (tid == 0) tr[0] = wall_clock64();
#define TRACE(i) if (tid == 0) tr[i] = wall_clock64();
  long long tacc[3] = {0, 0, 0}, tlast = 0;   // compute, LDS store (incl. wait for the loads), barrier
#define TRACE_T(k) { long long now = __builtin_readcyclecounter(); if (k > 0) tacc[k - 1] += now - tlast; tlast = now; }
#else
#define TRACE(i)
#define TRACE_T(k)
#endif
  // tile t travels in register set t % 2 and LDS stage t % 2.  (Reading the A fragments of a
  // k-contiguous A straight from global memory instead, to halve the LDS traffic, was measured
  // 18 % slower: 32-byte pieces of 32 different rows per load instruction.)
  static_assert(PF == 2, "the loop below is written for two register sets");
  TileRegs r[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (j < nk) gload(j, r[j]);
  if (nk > 0) lstore(0, r[0]);
  __syncthreads();
  TRACE(1)
  if (2 < nk) gload(2, r[0]);
  for (int i0 = 0; i0 < nk; i0 += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int i = i0 + u;
      if (i >= nk) break;
      TRACE_T(0)
      compute(u);
      TRACE_T(1)
      if (i + 1 < nk) lstore(u ^ 1, r[u ^ 1]);
      TRACE_T(2)
      __syncthreads();
      TRACE_T(3)
      if (i + 3 < nk) gload(i + 3, r[u ^ 1]);
    }
  }

  TRACE(2)
#ifdef PPLL_GEMM_TRACE
  if (tid == 0) { tr[5] = tacc[0]; tr[6] = tacc[1]; tr[7] = tacc[2]; }
#endif
  if (do_colsum) {
    csum += __shfl_xor(csum, 1, 64);
    const int n = n0 + (tid >> 1);
    if (!(tid & 1) && n < p.N) p.colsum[(size_t)split * p.N + n] = csum;
  }

  // Epilogue through LDS: the accumulators (lane = one C row, 4 consecutive columns per group)
  // are laid down as an fp32 tile, then every thread takes 8 consecutive columns of a row, so
  // bias / residual / saved pre-activation are read and C is written in full 128-column rows.
  __syncthreads();   // every wave is done with the operand stages
  float* stage = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int im = 0; im < IM; ++im)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = wm * (TM / 2) + im * 32 + (lane & 31), col = wn * 64 + jn * 32 + 8 * q + 4 * (lane >> 5);
        *reinterpret_cast<float4*>(stage + row * STAGE_LD + col) =
            make_float4(acc[jn][im][4 * q], acc[jn][im][4 * q + 1], acc[jn][im][4 * q + 2], acc[jn][im][4 * q + 3]);
      }
  __syncthreads();
  TRACE(3)
#pragma unroll 2
  for (int pass = 0; pass < TM / 16; ++pass) {
    const int row = pass * 16 + (tid >> 4), c8 = (tid & 15) * 8;
    const int m = m0 + row, n = n0 + c8;
    if (m >= p.M || n >= p.N) continue;
    float v[8];
    {
      const float4 lo = *reinterpret_cast<const float4*>(stage + row * STAGE_LD + c8);
      const float4 hi = *reinterpret_cast<const float4*>(stage + row * STAGE_LD + c8 + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    }
    if (p.partial) {
      float* dst = p.partial + ((size_t)split * p.M + m) * p.N + n;
      *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
      continue;
    }
    if (p.bias) {
      const float4 b0 = *reinterpret_cast<const float4*>(p.bias + n), b1 = *reinterpret_cast<const float4*>(p.bias + n + 4);
      v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w; v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
    }
    if (p.residual) {
      const uint4 r = *reinterpret_cast<const uint4*>(p.residual + (size_t)m * p.ldr + n);
      const uint32_t* w = reinterpret_cast<const uint32_t*>(&r);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(w[e] << 16); v[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
    }
    if (p.epilogue == EPI_DGELU) {
      const uint4 hq = *reinterpret_cast<const uint4*>(p.aux + (size_t)m * p.ldaux + n);
      const uint32_t* w = reinterpret_cast<const uint32_t*>(&hq);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[2 * e] *= dgelu_fast(__uint_as_float(w[e] << 16));
        v[2 * e + 1] *= dgelu_fast(__uint_as_float(w[e] & 0xffff0000u));
      }
    }
    if (p.c_f32) {
      float* dst = (float*)p.C + (size_t)m * p.ldc + n;
      *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      uint4 o;
      o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]); o.z = pack_bf16x2(v[4], v[5]); o.w = pack_bf16x2(v[6], v[7]);
      *reinterpret_cast<uint4*>((uint16_t*)p.C + (size_t)m * p.ldc + n) = o;
      if (p.epilogue == EPI_GELU) {
        uint4 g;
        g.x = pack_bf16x2(gelu_fast(v[0]), gelu_fast(v[1])); g.y = pack_bf16x2(gelu_fast(v[2]), gelu_fast(v[3]));
        g.z = pack_bf16x2(gelu_fast(v[4]), gelu_fast(v[5])); g.w = pack_bf16x2(gelu_fast(v[6]), gelu_fast(v[7]));
        *reinterpret_cast<uint4*>(p.C2 + (size_t)m * p.ldc + n) = g;
      }
    }
  }
  TRACE(4)
}

// C[i] = sum over splits of partial[s][i], fixed order; the trailing workgroups do the same for
// the bias-gradient partials [splits][N] when there are any.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* partial, int splits, size_t mn, float* C,
                                                            int main_blocks, const float* cs_partial, int N,
                                                            float* cs_out) {
  if ((int)blockIdx.x >= main_blocks) {
    const int n = ((int)blockIdx.x - main_blocks) * 256 + threadIdx.x;
    if (n >= N) return;
    float acc = 0.f;
    for (int s = 0; s < splits; ++s) acc += cs_partial[(size_t)s * N + n];
    cs_out[n] = acc;
    return;
  }
  size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= mn) return;
  float4 acc = *reinterpret_cast<const float4*>(partial + i);
  for (int s = 1; s < splits; ++s) {
    float4 v = *reinterpret_cast<const float4*>(partial + (size_t)s * mn + i);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  *reinterpret_cast<float4*>(C + i) = acc;
}

#ifdef PPLL_GEMM_TRACE
long long* g_gemm_trace = nullptr;
#endif
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
  if ((lda & 7) || (ldb & 7) || (g.ldc & (g.c_dt == BF16 ? 7 : 3))) return false;
  if (at && (g.M & 7)) return false;
  if (!aligned16(g.A) || !aligned16(g.B) || !aligned16(g.C)) return false;
  if (g.bias && !aligned16(g.bias)) return false;
  if (g.residual && (g.r_dt != BF16 || (g.ldr & 7) || !aligned16(g.residual))) return false;
  if (g.epilogue == EPI_GELU && (g.c_dt != BF16 || !g.C2 || !aligned16(g.C2))) return false;
  if (g.epilogue == EPI_DGELU && (g.aux_dt != BF16 || (g.ldaux & 7) || !aligned16(g.aux))) return false;
  return true;
}

// Number of K splits for a product (1 = none) and the partial floats it needs.
int gemm_mfma_splits(int M, int N, int K) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int nkt = (K + BK - 1) / BK;
  if (tiles >= 128 || nkt < 8) return 1;
  int splits = (256 + tiles - 1) / tiles;          // about one workgroup per compute unit
  if (nkt >= 32) {                                  // a multiple of 8, so that splits can be dealt to the 8 XCDs evenly
    splits = ((splits + 7) / 8) * 8;
    while (splits > 8 && splits > nkt / 4) splits -= 8;
  } else if (splits > nkt / 2) {
    splits = nkt / 2;
  }
  int per = (nkt + splits - 1) / splits;
  int real = (nkt + per - 1) / per;
  return (nkt >= 32 && real != splits) ? splits : real;   // keep the multiple of 8 (a trailing split may be short or empty)
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
  p.tiles_n = (g.N + BN - 1) / BN;
  // 64-row tiles when 128-row tiles would leave compute units without a workgroup
  const bool small_m = !at && ((g.M + BM - 1) / BM) * p.tiles_n < 256;
  const int tm_rows = small_m ? 64 : BM;
  p.tiles_m = (g.M + tm_rows - 1) / tm_rows;
  p.bias = g.bias; p.residual = (const uint16_t*)g.residual; p.ldr = g.ldr;
  p.epilogue = g.epilogue; p.C2 = (uint16_t*)g.C2; p.aux = (const uint16_t*)g.aux; p.ldaux = g.ldaux;
#ifdef PPLL_GEMM_TRACE
  p.trace = g_gemm_trace;
#endif
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
  p.splits = splits;
  p.xcd_map = (splits > 1 && splits % 8 == 0) ? 2 : (p.tiles_m >= 16 ? 1 : 0);
  dim3 grid(p.tiles_m * p.tiles_n, splits);
  if (p.xcd_map == 1) grid = dim3(((p.tiles_m + 7) / 8) * 8 * p.tiles_n, splits);
  if (p.xcd_map == 2) grid = dim3(p.tiles_m * p.tiles_n * splits, 1);
  static bool lds_opted_in = false;   // > 64 KB of dynamic LDS needs a one-time opt-in per kernel
  if (!lds_opted_in) {
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<true, true, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<true, false, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<false, true, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<false, false, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
    lds_opted_in = true;
  }
  void* prof = nullptr;
  PPLL_TRY(profile_begin(s, 2.0 * g.M * g.N * g.K, &prof));
  if (small_m) {
    if (bt) hipLaunchKernelGGL((gemm_mfma_kernel<false, true, 64>), grid, dim3(256), lds_bytes(64), s, p);
    else hipLaunchKernelGGL((gemm_mfma_kernel<false, false, 64>), grid, dim3(256), lds_bytes(64), s, p);
  } else if (at && bt) hipLaunchKernelGGL((gemm_mfma_kernel<true, true, 128>), grid, dim3(256), lds_bytes(128), s, p);
  else if (at) hipLaunchKernelGGL((gemm_mfma_kernel<true, false, 128>), grid, dim3(256), lds_bytes(128), s, p);
  else if (bt) hipLaunchKernelGGL((gemm_mfma_kernel<false, true, 128>), grid, dim3(256), lds_bytes(128), s, p);
  else hipLaunchKernelGGL((gemm_mfma_kernel<false, false, 128>), grid, dim3(256), lds_bytes(128), s, p);
  PPLL_HIP(hipGetLastError());
  PPLL_TRY(profile_end(s, prof));
  if (splits > 1) {
    size_t mn = (size_t)g.M * g.N;
    const int main_blocks = (int)((mn / 4 + 255) / 256), extra = g.colsum ? (g.N + 255) / 256 : 0;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(main_blocks + extra), dim3(256), 0, s, partial, splits, mn, (float*)g.C,
                       main_blocks, colsum_partial, g.N, g.colsum);
    PPLL_HIP(hipGetLastError());
  }
  return PPLL_OK;
}

}  // namespace ppll
