// Linear-layer products with few output rows: C[M,N] = A[M,K] B[K,N] with M up to 256, bf16
// operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16), the epilogues of the tiled kernel.
//
// These are the products of the last auxiliary encoder layer when only its class-token rows are
// computed (one row per image: M = batch): forward Q / projection / fc1 / fc2 and their input
// gradients.  They have almost no arithmetic (0.04-0.15 GFLOP) and a reduction index of 384 to
// 1536, so what they cost is latency: 128-row tiles give 3 to 12 workgroups that walk K one
// 64-wide step after the other.  Here a workgroup owns a 32 x 32 output tile and its four waves
// split K between them (each wave a contiguous quarter), every wave reading its operand fragments
// straight from memory in the MFMA's register layout, several k-steps in flight at once; the four
// partial tiles meet in LDS, are added in wave order (results do not depend on timing) and pass
// through the epilogue.  N/32 x M/32 workgroups: 48 to 192 for the shapes above.
//
// Operand layouts: A is [M][K] with k contiguous (row stride lda: the class-token rows of a token
// matrix are T*D apart).  B is either [N][K] with k contiguous (input gradients: W stored
// [in,out] read as B(k = out, n = in)), one 16-byte load per fragment, or [K][N] with n contiguous
// (forward: W [in,out]): a lane then needs 8 consecutive k of one column.  Each wave copies its
// 64 x 32 piece of B to a private LDS tile as it lies in memory (16-byte loads and stores) and
// takes the fragments out with the transposing LDS read; eight two-byte loads per fragment
// instead were measured at 12.9 us per product against 5.7 us for the k-contiguous case.
#include "common.h"

namespace ppll {

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int OOB = 0x7fffffff;        // no buffer here reaches 2^30 bytes (checked on the host)
constexpr int OOB_BASE = 0x40000000;   // stays out of range after a k offset (< 2^30) is added
constexpr int U = 4;                   // k-steps (of 16) per group of loads
constexpr int PART_LD = 36;            // row pitch of a partial tile in LDS (floats)

struct RowsArgs {
  const uint16_t* A; long lda;
  const uint16_t* B; long ldb;
  void* C; int c_f32; long ldc;
  int M, N, K;
  const float* bias;
  const uint16_t* residual; long ldr;
  int epilogue;
  uint16_t* C2;
  const uint16_t* aux; long ldaux;
  uint32_t a_bytes, b_bytes;
  int steps_per_wave;                  // 16-wide k-steps of each of the four waves
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_rsrc(const void* ptr, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(ptr), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ bf16x8 load8(__amdgpu_buffer_rsrc_t r, int off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
  return __builtin_bit_cast(bf16x8, v);
}
typedef __attribute__((ext_vector_type(4))) short s16x4;
constexpr int TR_PITCH = 80;           // bytes between the k rows of a wave's [64 k][32 n] tile of B in LDS
// 4 consecutive k of one column out of a [k][n] tile: lane r of a 16-lane group hands in the address of 4 columns
// (4 (r % 4) ..) at k row r / 4 and receives column r of the group's 16 at those four k rows
__device__ __forceinline__ uint2 lds_read_tr(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  return __builtin_bit_cast(uint2, v);
}

struct Frags { bf16x8 a[U], b[U]; uint4 raw[4]; };   // raw: a [K][N] operand on its way to LDS

template <bool BT>
__global__ __launch_bounds__(256) void gemm_rows_kernel(RowsArgs p) {
  __shared__ __align__(16) float part[4][32][PART_LD];
  __shared__ __align__(16) char btile[BT ? 4 : 1][BT ? U * 16 * TR_PITCH : 16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 31, g = lane >> 5;
  const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const __amdgpu_buffer_rsrc_t rsA = rows_rsrc(p.A, p.a_bytes), rsB = rows_rsrc(p.B, p.b_bytes);
  // this lane's fragment row of A (output row m0 + r) and of B (output column n0 + r), 8 k from k = .. + 8 g on
  const int a_base = m0 + r < p.M ? (int)((long)(m0 + r) * p.lda * 2) : OOB_BASE;
  const int b_base = n0 + r < p.N ? (int)((long)(n0 + r) * p.ldb * 2) : OOB_BASE;   // [N][K]
  const int k_wave = wave * p.steps_per_wave * 16, k_first = k_wave + 8 * g;
  // [K][N]: piece j of the lane's copy of a 64 x 32 group: k row lane/4 + 16 j, columns n0 + 8 (lane % 4) .. + 7
  const int t_row = lane >> 2, t_col = (lane & 3) * 8;
  const int t_base = n0 + t_col < p.N ? (n0 + t_col) * 2 : OOB_BASE;
  const int b_step = (int)(p.ldb * 2);   // [K][N]: bytes between consecutive k
  // lane part of a fragment address in the LDS tile: k row 8 (lane / 32) + (lane % 16) / 4, columns 16 ((lane / 16) % 2) + 4 (lane % 4)
  const int tr_lane = (8 * g + ((lane & 15) >> 2)) * TR_PITCH + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

  auto load_group = [&](int gi, Frags& f) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = gi * U + u, k = k_first + 16 * s;
      const bool in = s < p.steps_per_wave && k < p.K;
      f.a[u] = load8(rsA, in ? a_base + 2 * k : OOB);
      if (BT) {     // k rows 16 u .. 16 u + 15 of the group hold step s
        const int kr = k_wave + 16 * s + t_row;
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsB, (s < p.steps_per_wave && kr < p.K) ? t_base + kr * b_step : OOB, 0, 0);
        f.raw[u] = make_uint4(v.x, v.y, v.z, v.w);
      } else {
        f.b[u] = load8(rsB, in ? b_base + 2 * k : OOB);
      }
    }
  };
  // [K][N] operand: through the wave's LDS tile into fragments
  auto transpose_group = [&](Frags& f) {
    if (!BT) return;
    char* tile = btile[BT ? wave : 0];
#pragma unroll
    for (int u = 0; u < U; ++u) *reinterpret_cast<uint4*>(tile + (16 * u + t_row) * TR_PITCH + t_col * 2) = f.raw[u];
    wave_sync();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const char* q = tile + tr_lane + u * 16 * TR_PITCH;
      const uint2 lo = lds_read_tr(q), hi = lds_read_tr(q + 4 * TR_PITCH);
      f.b[u] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
    }
    wave_sync();   // every lane has its fragments before the tile is written again
  };
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  // the MFMA takes the B fragment first: a lane then holds 4 consecutive columns (n) of one output row (m)
  auto multiply = [&](const Frags& f) {
#pragma unroll
    for (int u = 0; u < U; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[u], f.a[u], acc, 0, 0, 0);
  };
  Frags f0, f1;
  const int groups = (p.steps_per_wave + U - 1) / U;
  load_group(0, f0);
  for (int gi = 0; gi < groups; gi += 2) {   // groups past the wave's range read as zeros
    load_group(gi + 1, f1);
    transpose_group(f0);
    multiply(f0);
    load_group(gi + 2, f0);
    transpose_group(f1);
    multiply(f1);
  }
  // acc[4 q + e] = C[m0 + r][n0 + 8 q + 4 g + e] summed over this wave's k
#pragma unroll
  for (int q = 0; q < 4; ++q)
    *reinterpret_cast<float4*>(&part[wave][r][8 * q + 4 * g]) = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
  __syncthreads();
  const int mm = tid >> 3, nn = (tid & 7) * 4, m = m0 + mm, n = n0 + nn;
  if (m >= p.M || n >= p.N) return;     // N is a multiple of 8: four columns from a multiple of 4 below N are all inside
  float v[4];
  {
    float4 t = *reinterpret_cast<const float4*>(&part[0][mm][nn]);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float4 x = *reinterpret_cast<const float4*>(&part[w][mm][nn]);
      t.x += x.x; t.y += x.y; t.z += x.z; t.w += x.w;
    }
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  if (p.bias) {
    const float4 b = *reinterpret_cast<const float4*>(p.bias + n);
    v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
  }
  if (p.residual) {
    const uint2 w = *reinterpret_cast<const uint2*>(p.residual + (size_t)m * p.ldr + n);
    v[0] += __uint_as_float(w.x << 16); v[1] += __uint_as_float(w.x & 0xffff0000u);
    v[2] += __uint_as_float(w.y << 16); v[3] += __uint_as_float(w.y & 0xffff0000u);
  }
  if (p.epilogue == EPI_DGELU) {
    const uint2 w = *reinterpret_cast<const uint2*>(p.aux + (size_t)m * p.ldaux + n);
    v[0] *= __uint_as_float(w.x << 16); v[1] *= __uint_as_float(w.x & 0xffff0000u);
    v[2] *= __uint_as_float(w.y << 16); v[3] *= __uint_as_float(w.y & 0xffff0000u);
  }
  if (p.c_f32) {
    *reinterpret_cast<float4*>((float*)p.C + (size_t)m * p.ldc + n) = make_float4(v[0], v[1], v[2], v[3]);
    return;
  }
  uint16_t* c = (uint16_t*)p.C + (size_t)m * p.ldc + n;
  if (p.epilogue == EPI_GELU) {   // C2 = gelu(h), C = gelu'(h): one evaluation of the normal CDF and density
    float gl[4], dg[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float cdf, pdf;
      cdf_pdf(v[e], cdf, pdf);
      gl[e] = v[e] * cdf; dg[e] = cdf + v[e] * pdf;
    }
    *reinterpret_cast<uint2*>(c) = make_uint2(f32x2_to_bf16x2(dg[0], dg[1]), f32x2_to_bf16x2(dg[2], dg[3]));
    *reinterpret_cast<uint2*>(p.C2 + (size_t)m * p.ldc + n) = make_uint2(f32x2_to_bf16x2(gl[0], gl[1]), f32x2_to_bf16x2(gl[2], gl[3]));
  } else {
    *reinterpret_cast<uint2*>(c) = make_uint2(f32x2_to_bf16x2(v[0], v[1]), f32x2_to_bf16x2(v[2], v[3]));
  }
}

bool aligned_to(const void* p, uintptr_t a) { return (((uintptr_t)p) & (a - 1)) == 0; }
}  // namespace

constexpr int ROWS_MAX_M = 256;

bool gemm_rows_supported(const GemmArgs& g) {
  if (g.a_dt != BF16 || g.b_dt != BF16 || g.colsum) return false;
  if (g.M < 1 || g.M > ROWS_MAX_M || g.N < 1 || g.K < 1 || (g.N & 7) || (g.K & 7)) return false;
  if (g.a_sk != 1 || (g.a_sm & 7) || !aligned_to(g.A, 16)) return false;
  const bool bt = g.b_sn == 1 && g.b_sk != 1;
  if (bt) {
    if ((g.b_sk & 7) || !aligned_to(g.B, 16)) return false;
  } else {
    if (g.b_sk != 1 || (g.b_sn & 7) || !aligned_to(g.B, 16)) return false;
  }
  if (g.c_dt == BF16 ? ((g.ldc & 3) || !aligned_to(g.C, 8)) : ((g.ldc & 3) || !aligned_to(g.C, 16))) return false;
  if (g.bias && !aligned_to(g.bias, 16)) return false;
  if (g.residual && (g.r_dt != BF16 || (g.ldr & 3) || !aligned_to(g.residual, 8))) return false;
  if (g.epilogue == EPI_GELU && (g.c_dt != BF16 || !g.C2 || !aligned_to(g.C2, 8))) return false;
  if (g.epilogue == EPI_DGELU && (g.aux_dt != BF16 || (g.ldaux & 3) || !aligned_to(g.aux, 8))) return false;
  // operands are addressed with 32-bit byte offsets
  const long lim = (1L << 30) - 64;
  const long a_bytes = ((long)(g.M - 1) * g.a_sm + g.K) * 2;
  const long b_bytes = bt ? ((long)(g.K - 1) * g.b_sk + g.N) * 2 : ((long)(g.N - 1) * g.b_sn + g.K) * 2;
  return a_bytes <= lim && b_bytes <= lim;
}

int launch_gemm_rows(hipStream_t s, const GemmArgs& g) {
  if (!gemm_rows_supported(g)) { set_error("launch_gemm_rows: unsupported product"); return PPLL_ERR_CONFIG; }
  const bool bt = g.b_sn == 1 && g.b_sk != 1;
  RowsArgs p{};
  p.A = (const uint16_t*)g.A; p.lda = g.a_sm;
  p.B = (const uint16_t*)g.B; p.ldb = bt ? g.b_sk : g.b_sn;
  p.C = g.C; p.c_f32 = g.c_dt == F32; p.ldc = g.ldc;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.bias = g.bias; p.residual = (const uint16_t*)g.residual; p.ldr = g.ldr;
  p.epilogue = g.epilogue; p.C2 = (uint16_t*)g.C2; p.aux = (const uint16_t*)g.aux; p.ldaux = g.ldaux;
  p.a_bytes = (uint32_t)(((long)(g.M - 1) * g.a_sm + g.K) * 2);
  p.b_bytes = (uint32_t)(bt ? ((long)(g.K - 1) * g.b_sk + g.N) * 2 : ((long)(g.N - 1) * g.b_sn + g.K) * 2);
  const int steps = (g.K + 15) / 16;
  p.steps_per_wave = (steps + 3) / 4;
  const dim3 grid((g.N + 31) / 32, (g.M + 31) / 32);
  void* prof = nullptr;
  PPLL_TRY(profile_begin(s, 2.0 * g.M * g.N * g.K, &prof, 2));
  if (bt) hipLaunchKernelGGL(gemm_rows_kernel<true>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(gemm_rows_kernel<false>, grid, dim3(256), 0, s, p);
  PPLL_HIP(hipGetLastError());
  return profile_end(s, prof);
}

}  // namespace ppll
