// bf16 GEMM on the CDNA4 matrix cores: C[M,N] = A(M,K) . B(K,N), fp32
// accumulation in v_mfma_f32_32x32x16_bf16, operands staged through LDS.
//
// One 256-thread workgroup (4 waves, 2 x 2) owns a 128 x 128 output tile and
// walks K in steps of 64; each wave owns 64 x 64 = 2 x 2 MFMA tiles.  An MFMA
// operand fragment is 8 consecutive k of one row per lane.  An operand whose k is
// contiguous in memory (activations in Y = X W^T-style products, the [in,out]
// weight in dX = dY W^T) lies in LDS as [row][k] and a fragment is one 16-byte
// read.  An operand whose other index is contiguous (the [in,out] weight in
// Y = X W, both operands of dW = X^T dY) lies in LDS as it lies in memory, [k][row],
// and the fragment comes out of two transposing LDS reads (ds_read_b64_tr_b16: 16
// lanes hand in the addresses of a 16 x 4 block of 16-bit elements and get it back
// transposed), so no transposed copies of weights or activations exist in HBM and
// no lane shuffles happen on the way in: every tile is copied with 16-byte loads
// and 16-byte LDS stores.
//
// The 16-byte k-granules of a [row][k] tile are permuted by an XOR with row bits;
// a [k][row] tile has its k rows 320 bytes apart: with these the fragment reads
// and the stores run at the rate of linear ones (timed with a micro-benchmark of
// the access patterns).
//
// The MFMA is issued with the B tile as its first operand, i.e. it produces C
// transposed: a lane then holds 4 consecutive columns of one C row, so bias,
// residual, saved GELU derivative and the output move as 8/16-byte vectors.
//
// Split-K (weight gradients: tiny outputs, reduction over all tokens): every
// split writes its fp32 partial tile, a second kernel adds the splits in a
// fixed order, so results are reproducible (no float atomics).
#include "common.h"
#include <atomic>
#include <algorithm>

namespace ppll {

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 128, BN = 128, BK = 64;


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
  uint32_t a_bytes, b_bytes, c_bytes, r_bytes, aux_bytes, partial_bytes;   // extents of the buffers above
  int xcd_map;                      // 1: ids 8 apart share a tile row (many tile rows), 2: ids 8 apart share a
                                    // split (split-K), 0: row-major ids
  int splits;
  // k_range set: the k-range is given outright (balanced grouped launch), kt_count k-tiles from k-tile kt_first on.
  // tile_partial, when set, receives the whole fp32 tile ([128][128], then 128 column sums) in place of C and colsum.
  int k_range, kt_first, kt_count;
  float* tile_partial;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) { return f32x2_to_bf16x2(a, b); }

// LDS layout of an operand tile.  Measured on the chip (16 waves of one compute unit issuing one access pattern;
// units per wave instruction: a linear ds_read_b128 takes 4.1, a linear ds_read_b64 2.4, a linear ds_write_b128 13):
//  - [row][64 k] (k contiguous in memory): rows 128 bytes apart, the 16-byte granule index XORed with (row/2)%8:
//    fragment reads 4.1, stores as fast as linear ones;
//  - [64 k][128 rows] (row index contiguous in memory): k rows TR_PITCH = 320 bytes apart: the two transposing
//    8-byte reads of a fragment take 2.4 each (4.0 at 288 or 384 bytes, 8.0 at 256), the stores are 256-byte
//    rows.  (The earlier layout, transposed in registers on the way in, [row][k] with rows 160 bytes apart, paid
//    8.0 per 8-byte store, eight of them and sixteen byte permutes per thread and k-step.)
constexpr int TR_PITCH = 320;
struct RowMajorTile {   // [row][64 k]
  static __device__ __forceinline__ int off(int row, int granule16) { return row * 128 + ((granule16 ^ ((row >> 1) & 7)) << 4); }
};
constexpr int tile_bytes(bool tr, int rows) { return tr ? BK * TR_PITCH : rows * 128; }

typedef __attribute__((ext_vector_type(4))) short s16x4;
// 4 consecutive k of one row out of a [k][row] tile: lane r of a 16-lane group hands in the address of 4 rows
// (4 (r % 4) ..) at k row r / 4 and receives row r of the group's 16 at those four k rows
__device__ __forceinline__ uint2 lds_read_tr(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  return __builtin_bit_cast(uint2, v);
}

// ---- Buffer addressing.  Operands, outputs and epilogue inputs are reached through raw buffer
// descriptors: a load whose byte offset lies beyond the buffer returns 0 and a store there is
// dropped, so the tile edges (rows beyond M or N, k beyond K or beyond a split's range) need no
// branches: an out-of-range lane simply gets the offset OOB.  Straight-line code also lets the
// compiler count outstanding loads exactly, so the loads of the k-tile two steps ahead stay in
// flight while the previous one is written to LDS.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int OOB = 0x7fffffff;   // no buffer here reaches 2^30 bytes (checked on the host)
constexpr int OOB_BASE = 0x40000000;   // a base offset that stays out of range after a k-step (< 2^30) is added
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* ptr, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(ptr), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, int off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void buf_store16(__amdgpu_buffer_rsrc_t r, int off, uint4 v) {
  const u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_amdgcn_raw_buffer_store_b128(w, r, off, 0, 0);
}

// One operand tile (ROWS x 64) on its way from memory to LDS, as seen by one thread.
//  [row][k] (k contiguous in memory): ROWS/32 pieces of 8 bf16; piece i is row (tid + 256 i)/8, k-granule tid%8.
//  [k][row] (row index contiguous; ROWS = 128): 4 pieces; piece j is k row tid/16 + 16 j, rows 8 (tid%16) .. +7.
template <bool TR, int ROWS>
struct OperandLoader {
  static_assert(!TR || ROWS == 128, "a [k][row] tile is 128 rows wide");
  static constexpr int NP = TR ? 4 : ROWS / 32;
  int off[NP];      // byte offset of each piece at k = 0 of the thread's k-range; OOB_BASE if its row does not exist
  int kl;           // first k (within a tile) of the thread's pieces
  int ld2;          // [k][row]: bytes between consecutive k
  __device__ __forceinline__ void init(long ld, int row0, int nrows, int tid) {
    if (TR) {
      const int row = row0 + (tid & 15) * 8;
      kl = tid >> 4; ld2 = (int)(ld * 2);
#pragma unroll
      for (int j = 0; j < 4; ++j) off[j] = row < nrows ? (int)(((long)(kl + 16 * j) * ld + row) * 2) : OOB_BASE;
    } else {
      kl = (tid & 7) * 8; ld2 = 0;
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const int row = row0 + ((tid + 256 * i) >> 3);
        off[i] = row < nrows ? (int)(((long)row * ld + kl) * 2) : OOB_BASE;
      }
    }
  }
  // pieces of the k-tile starting at k0; k >= kend reads as zero
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, int k0, int kend, uint4 (&r)[4]) const {
    if (TR) {
      const int step = k0 * ld2;
#pragma unroll
      for (int j = 0; j < 4; ++j) r[j] = buf_load16(rsrc, (k0 + kl + 16 * j < kend) ? off[j] + step : OOB);
    } else {
      const bool kin = k0 + kl < kend;
#pragma unroll
      for (int i = 0; i < NP; ++i) r[i] = buf_load16(rsrc, kin ? off[i] + 2 * k0 : OOB);
    }
  }
  // piece q (0..3) of the thread's LDS writes of one tile
  __device__ __forceinline__ void store_part(char* lds, int tid, const uint4 (&r)[4], int q) const {
    if (TR) {
      *reinterpret_cast<uint4*>(lds + (kl + 16 * q) * TR_PITCH + (tid & 15) * 16) = r[q];
    } else if (q < NP) {
      const int c = tid + 256 * q;
      *reinterpret_cast<uint4*>(lds + RowMajorTile::off(c >> 3, c & 7)) = r[q];
    }
  }
};

constexpr int STAGE_LD = BN + 4;                      // fp32 staging tile of the epilogue, padded row
// one stage of both operand tiles; two stages, or the epilogue's staging tile if that is larger
constexpr int oper_bytes(bool at, bool bt, int tm) { return tile_bytes(at, tm) + tile_bytes(bt, BN); }
constexpr int lds_bytes(bool at, bool bt, int tm) {
  return 2 * oper_bytes(at, bt, tm) > tm * STAGE_LD * 4 ? 2 * oper_bytes(at, bt, tm) : tm * STAGE_LD * 4;
}

struct TileRegs { uint4 a[4], b[4]; };

// AT: A is stored [K][M] (transposing loader), else [M][K].  BT likewise for B ([K][N] / [N][K]).
// TM = rows of the output tile: 128 (wave tile 64 x 64) or, for outputs with too few 128-row
// tiles to fill the chip, 64 (wave tile 32 x 64; direct A loader only).
// One output tile; bid_x, bid_y are the workgroup's place in the (virtual) grid of this product.
template <bool AT, bool BT, int TM>
__device__ __forceinline__ void gemm_mfma_tile(const MfmaArgs& p, const int bid_x, const int bid_y) {
  static_assert(TM == 128 || (TM == 64 && !AT), "64-row tiles are for the direct A loader");
  constexpr int IM = TM / 64;                  // 32-row MFMA tiles per wave along m
  constexpr int OPER_BYTES = oper_bytes(AT, BT, TM);
  constexpr int A_BYTES = tile_bytes(AT, TM);   // the B tile of a stage follows the A tile
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  // Workgroup id -> tile.  Consecutive ids go to the 8 XCDs round-robin and each XCD has its own
  // L2, so the tiles of one row (they share the A panel) are given ids that are 8 apart: they
  // land on one XCD, next to each other in its dispatch order, and the panel is fetched once.
  // With split-K (xcd_map 2) it is the splits that are dealt to the XCDs: all tiles of one k-range
  // run on one XCD, so the two token panels of that range are fetched from HBM once.
  int tm, tn, split = bid_y;
  if (p.xcd_map == 1) {
    const int xcd = bid_x & 7, slot = bid_x >> 3;
    tm = (slot / p.tiles_n) * 8 + xcd; tn = slot % p.tiles_n;
    if (tm >= p.tiles_m) return;
  } else if (p.xcd_map == 2) {
    const int tiles = p.tiles_m * p.tiles_n;
    const int xcd = bid_x & 7, slot = bid_x >> 3;
    split = (slot / tiles) * 8 + xcd;
    const int tile = slot % tiles;
    tm = tile / p.tiles_n; tn = tile % p.tiles_n;
    if (split >= p.splits) return;
  } else {
    tm = bid_x / p.tiles_n; tn = bid_x % p.tiles_n;
  }
  const int m0 = tm * TM, n0 = tn * BN;
  const int nkt = (p.K + BK - 1) / BK;
  const int kt0 = p.k_range ? p.kt_first : split * p.kt_per_split;
  const int nk = p.k_range ? p.kt_count : min(nkt, kt0 + p.kt_per_split) - kt0;   // k-tiles of this workgroup (a trailing split may have none)
  const int kbeg = kt0 * BK, kend = min(p.K, (kt0 + nk) * BK);

  f32x16 acc[2][IM];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < IM; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  const __amdgpu_buffer_rsrc_t rsA = make_rsrc(p.A, p.a_bytes), rsB = make_rsrc(p.B, p.b_bytes);
  OperandLoader<AT, TM> ldA;
  OperandLoader<BT, BN> ldB;
  ldA.init(p.lda, m0, p.M, tid);
  ldB.init(p.ldb, n0, p.N, tid);
  // k-tile i of this workgroup -> registers; tiles past the end read as zeros without touching memory
  auto gload = [&](int i, TileRegs& r) {
    const int k0 = kbeg + i * BK;
    ldA.load(rsA, k0, kend, r.a);
    ldB.load(rsB, k0, kend, r.b);
  };
  auto lstore_part = [&](int stage, const TileRegs& r, int q) {
    char* la = smem + stage * OPER_BYTES;
    ldA.store_part(la, tid, r.a, q);
    ldB.store_part(la + A_BYTES, tid, r.b, q);
  };
  const int frag_row = lane & 31, frag_g = lane >> 5;
  // lane part of a fragment address in a [k][row] tile: k row 8 (lane/32) + (lane%16)/4, rows 16 ((lane/16)%2) + 4 (lane%4)
  const int tr_lane = (8 * (lane >> 5) + ((lane & 15) >> 2)) * TR_PITCH + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
  // fragment of rows row0 .. row0+31 at k = 16 kk .. +15 of an operand tile
  auto frag = [&](const char* tile, bool tr, int row0, int kk) -> bf16x8 {
    if (tr) {
      const char* p = tile + tr_lane + kk * 16 * TR_PITCH + row0 * 2;
      const uint2 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * TR_PITCH);
      return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
    }
    return *reinterpret_cast<const bf16x8*>(tile + RowMajorTile::off(row0 + frag_row, kk * 2 + frag_g));
  };
  auto load_frags = [&](int stage, int kk, bf16x8 (&fa)[IM], bf16x8 (&fb)[2]) {
    const char* la = smem + stage * OPER_BYTES;
    const char* lb = la + A_BYTES;
#pragma unroll
    for (int im = 0; im < IM; ++im) fa[im] = frag(la, AT, wm * (TM / 2) + im * 32, kk);
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) fb[jn] = frag(lb, BT, wn * 64 + jn * 32, kk);
  };
  // bias gradient riding along: the workgroups of the first tile row also add up their B tile over k, each thread
  // the pieces it copies itself (8 columns at its k rows), out of the registers they travel in
  const bool do_colsum = BT && p.colsum != nullptr && m0 == 0;
  float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto colsum_add = [&](const uint4& w) {
    csum[0] += bf16_to_f32((uint16_t)(w.x & 0xffff)); csum[1] += bf16_to_f32((uint16_t)(w.x >> 16));
    csum[2] += bf16_to_f32((uint16_t)(w.y & 0xffff)); csum[3] += bf16_to_f32((uint16_t)(w.y >> 16));
    csum[4] += bf16_to_f32((uint16_t)(w.z & 0xffff)); csum[5] += bf16_to_f32((uint16_t)(w.z >> 16));
    csum[6] += bf16_to_f32((uint16_t)(w.w & 0xffff)); csum[7] += bf16_to_f32((uint16_t)(w.w >> 16));
  };
  bf16x8 fa[2][IM], fb[2][2];   // operand fragments of two consecutive 16-wide k-steps
  // Multiplies the k-tile in LDS stage `stage` (its first fragments are already in fa[0], fb[0])
  // and, between the groups of MFMAs, writes the next tile (registers rn) to the other stage, so
  // that the LDS writes and the fragment reads of the following k-step run under the matrix pipe.
  auto multiply = [&](int stage, const TileRegs& rn, bool stage_next) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) load_frags(stage, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int im = 0; im < IM; ++im)
          acc[jn][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][jn], fa[kk & 1][im], acc[jn][im], 0, 0, 0);
      if (stage_next) {
        lstore_part(stage ^ 1, rn, kk);
        if (do_colsum) colsum_add(rn.b[kk]);
      }
    }
  };
  // One full step: multiply tile i (stage u), stage tile i+1, then refill the freed register
  // set with tile i+3 and fetch the first fragments of tile i+1.
  auto step = [&](int u, TileRegs& rn, int i) {
    multiply(u, rn, true);
    __syncthreads();
    load_frags(u ^ 1, 0, fa[0], fb[0]);
    gload(i + 3, rn);
  };

  // Software pipeline: two LDS stages and two register sets.  Tile t travels in register set
  // t % 2 and LDS stage t % 2; while tile i is multiplied, tile i+1 moves from registers to LDS
  // and tiles i+2, i+3 are in flight from memory.  (Reading the A fragments of a k-contiguous A
  // straight from global memory instead, to halve the LDS traffic, was measured 18 % slower:
  // 32-byte pieces of 32 different rows per load instruction.)
  TileRegs r[2];
  gload(0, r[0]);
  gload(1, r[1]);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    lstore_part(0, r[0], q);
    if (do_colsum) colsum_add(r[0].b[q]);
  }
  __syncthreads();
  gload(2, r[0]);
  if (nk > 0) {
    load_frags(0, 0, fa[0], fb[0]);
    int i = 0;
    for (; i + 2 < nk; i += 2) {
      step(0, r[1], i);
      step(1, r[0], i + 1);
    }
    if (nk - i == 2) {
      step(0, r[1], i);
      multiply(1, r[0], false);
    } else {
      multiply(0, r[1], false);
    }
  }


  // Epilogue through LDS: the accumulators (lane = one C row, 4 consecutive columns per group)
  // are laid down as an fp32 tile, then every thread takes 8 consecutive columns of a row, so
  // bias / residual / saved GELU derivative are read and C is written in full 128-column rows.
  // What the write-out needs from memory is requested first, so it arrives during the staging.
  constexpr int NPASS = TM / 16;
  const int prow = tid >> 4, c8 = (tid & 15) * 8, n = n0 + c8;
  const bool nok = n < p.N;
  const int ncol2 = nok ? 2 * n : OOB_BASE, ncol4 = nok ? 4 * n : OOB_BASE;   // column part of a byte offset; out of range beyond N
  float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  uint4 resv[NPASS], auxv[NPASS];
  const bool has_bias = p.bias != nullptr && !p.partial, has_res = p.residual != nullptr && !p.partial;
  const bool has_aux = p.epilogue == EPI_DGELU && !p.partial;
  if (has_bias) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.bias, (uint32_t)p.N * 4u);
    const uint4 b0 = buf_load16(rs, nok ? n * 4 : OOB), b1 = buf_load16(rs, nok ? n * 4 + 16 : OOB);
    bias8[0] = __uint_as_float(b0.x); bias8[1] = __uint_as_float(b0.y); bias8[2] = __uint_as_float(b0.z);
    bias8[3] = __uint_as_float(b0.w); bias8[4] = __uint_as_float(b1.x); bias8[5] = __uint_as_float(b1.y);
    bias8[6] = __uint_as_float(b1.z); bias8[7] = __uint_as_float(b1.w);
  }
  if (has_res) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.residual, p.r_bytes);
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int m = m0 + pass * 16 + prow;
      resv[pass] = buf_load16(rs, m < p.M ? (int)(((long)m * p.ldr) * 2) + ncol2 : OOB);
    }
  }
  if (has_aux) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.aux, p.aux_bytes);
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int m = m0 + pass * 16 + prow;
      auxv[pass] = buf_load16(rs, m < p.M ? (int)(((long)m * p.ldaux) * 2) + ncol2 : OOB);
    }
  }
  __syncthreads();   // every wave is done with the operand stages
  float* stage = reinterpret_cast<float*>(smem);
  if (do_colsum) {   // 16 threads (k rows tid/16 + 16 j) hold partial sums of the same 8 columns: added in order of tid/16
    float* cs = stage;                                  // [16][128]
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[(tid >> 4) * BN + (tid & 15) * 8 + e] = csum[e];
    __syncthreads();
    if (tid < BN) {
      float t = 0.f;
#pragma unroll
      for (int g = 0; g < 16; ++g) t += cs[g * BN + tid];
      if (p.tile_partial) p.tile_partial[BM * BN + tid] = t;
      else if (n0 + tid < p.N) p.colsum[(size_t)split * p.N + n0 + tid] = t;
    }
    __syncthreads();
  }
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
  const __amdgpu_buffer_rsrc_t rsC = p.tile_partial ? make_rsrc(p.tile_partial, BM * BN * 4)
                                     : p.partial    ? make_rsrc(p.partial, p.partial_bytes) : make_rsrc(p.C, p.c_bytes);
  const __amdgpu_buffer_rsrc_t rsC2 = make_rsrc(p.C2 ? (const void*)p.C2 : p.C, p.C2 ? p.c_bytes : 0u);
  const bool out_f32 = p.partial != nullptr || p.tile_partial != nullptr || p.c_f32;
#pragma unroll
  for (int pass = 0; pass < NPASS; ++pass) {
    const int row = pass * 16 + prow, m = m0 + row;
    const bool ok = m < p.M;
    float v[8];
    {
      const float4 lo = *reinterpret_cast<const float4*>(stage + row * STAGE_LD + c8);
      const float4 hi = *reinterpret_cast<const float4*>(stage + row * STAGE_LD + c8 + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += bias8[e];
    if (has_res) {
      const uint32_t* w = reinterpret_cast<const uint32_t*>(&resv[pass]);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(w[e] << 16); v[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
    }
    if (has_aux) {
      const uint32_t* w = reinterpret_cast<const uint32_t*>(&auxv[pass]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {   // the saved GELU derivative
        v[2 * e] *= __uint_as_float(w[e] << 16);
        v[2 * e + 1] *= __uint_as_float(w[e] & 0xffff0000u);
      }
    }
    if (out_f32) {
      const long e0 = p.partial ? ((long)split * p.M + m) * p.N : (long)m * p.ldc;
      const int off = p.tile_partial ? (row * BN + c8) * 4 : ok ? (int)(e0 * 4) + ncol4 : OOB;
      buf_store16(rsC, off, make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
      buf_store16(rsC, (ok || p.tile_partial) ? off + 16 : OOB, make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])));
    } else {
      const int off = ok ? (int)(((long)m * p.ldc) * 2) + ncol2 : OOB;
      if (p.epilogue == EPI_GELU) {   // C2 = gelu(h), C = gelu'(h) from one evaluation of the normal CDF and density
        float gl[8], dg[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float cdf, pdf;
          cdf_pdf(v[e], cdf, pdf);
          gl[e] = v[e] * cdf; dg[e] = cdf + v[e] * pdf;
        }
        uint4 o, g;
        o.x = pack_bf16x2(dg[0], dg[1]); o.y = pack_bf16x2(dg[2], dg[3]); o.z = pack_bf16x2(dg[4], dg[5]); o.w = pack_bf16x2(dg[6], dg[7]);
        g.x = pack_bf16x2(gl[0], gl[1]); g.y = pack_bf16x2(gl[2], gl[3]); g.z = pack_bf16x2(gl[4], gl[5]); g.w = pack_bf16x2(gl[6], gl[7]);
        buf_store16(rsC, off, o);
        buf_store16(rsC2, off, g);
      } else {
        uint4 o;
        o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]); o.z = pack_bf16x2(v[4], v[5]); o.w = pack_bf16x2(v[6], v[7]);
        buf_store16(rsC, off, o);
      }
    }
  }
}

template <bool AT, bool BT, int TM>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(MfmaArgs p) {
  gemm_mfma_tile<AT, BT, TM>(p, (int)blockIdx.x, (int)blockIdx.y);
}

// Several products C_j = A_j^T B_j (both operands stored [K][.], fp32 output, optional column sums
// of B_j: the weight and bias gradients of a set of Linear layers) in one launch, no split-K: the
// tiles of all products together fill the chip, so every tile walks its whole K and nothing
// passes through partial buffers.  Tiles are numbered product by product; XCD x (workgroup id % 8)
// takes a contiguous range of them, so the tiles that share operand panels share an L2.
struct GroupedProblem {
  const uint16_t* A; const uint16_t* B; float* C; float* colsum;
  int lda, ldb, ldc, M, N, K, tiles_m, tiles_n, first_tile;
  uint32_t a_bytes, b_bytes, c_bytes;
};
constexpr int GROUP_MAX = 24;
struct GroupedArgs {
  int n, total_tiles, per_xcd;
  GroupedProblem prob[GROUP_MAX];
};
// Tile t of the set -> its product and its place there (tm * tiles_n + tn).  Within a product the tiles are numbered
// across its shorter side first: a stretch of consecutive tiles then needs all panels of the short side and only its
// own panels of the long side, so where a stretch ends inside a product the next XCD fetches the few short-side panels
// again and nothing else twice.
template <class Args>
__device__ __forceinline__ int grouped_locate(const Args& a, int t, int& bid) {
  int j = 0;
  while (j + 1 < a.n && t >= a.prob[j + 1].first_tile) ++j;
  const int local = t - a.prob[j].first_tile, tiles_m = a.prob[j].tiles_m, tiles_n = a.prob[j].tiles_n;
  bid = tiles_m >= tiles_n ? local : (local % tiles_m) * tiles_n + local / tiles_m;
  return j;
}
template <class Args>
__device__ __forceinline__ MfmaArgs grouped_problem(const Args& a, int j) {
  MfmaArgs p{};
  p.A = a.prob[j].A; p.lda = a.prob[j].lda; p.B = a.prob[j].B; p.ldb = a.prob[j].ldb;
  p.C = a.prob[j].C; p.c_f32 = 1; p.ldc = a.prob[j].ldc;
  p.M = a.prob[j].M; p.N = a.prob[j].N; p.K = a.prob[j].K;
  p.tiles_m = a.prob[j].tiles_m; p.tiles_n = a.prob[j].tiles_n;
  p.kt_per_split = (p.K + BK - 1) / BK;
  p.colsum = a.prob[j].colsum;
  p.a_bytes = a.prob[j].a_bytes; p.b_bytes = a.prob[j].b_bytes; p.c_bytes = a.prob[j].c_bytes;
  p.splits = 1; p.xcd_map = 0;
  return p;
}
__global__ __launch_bounds__(256, 2) void gemm_mfma_grouped_kernel(GroupedArgs a) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int t = xcd * a.per_xcd + slot;
  if (slot >= a.per_xcd || t >= a.total_tiles) return;
  int bid;
  const int j = grouped_locate(a, t, bid);
  const MfmaArgs p = grouped_problem(a, j);
  gemm_mfma_tile<true, true, 128>(p, bid, 0);
}

// The same set of products with the work dealt out more evenly.  One whole tile per workgroup leaves the chip unevenly
// loaded when the tiles number a little more than the compute units (345 tiles of 130 k-steps on 256 units with two
// workgroups each: 89 units work on two tiles from start to end while 167 finish their one tile early and idle, and
// the launch lasts as long as the pairs).  Here the tiles beyond the last full round of one-per-unit are cut along k
// into `cuts` parts, each a workgroup of its own: a unit then holds a whole tile and a part of one.  A part leaves its
// fp32 sums in a slot of a workspace and a second kernel adds the parts of each divided tile in ascending k: results
// do not depend on timing.
constexpr int SLOT_FLOATS = BM * BN + BN;           // a tile's partial sums, then its 128 column sums
struct BalancedArgs {
  // products with a long reduction come first: their tiles [0, whole_tiles) run whole, [whole_tiles, long_tiles) are
  // divided into `cuts` parts; the tiles of products with a short reduction, [long_tiles, total_tiles), run whole at the end
  int n, total_tiles, long_tiles, whole_tiles, cuts;
  float* ws;                                        // [divided tile][part] slots
  GroupedProblem prob[GROUP_MAX];
};
__global__ __launch_bounds__(256, 2) void gemm_mfma_balanced_kernel(BalancedArgs a) {
  // workgroup id -> item.  Ids are handed out in order, round-robin over the 8 XCDs: the whole tiles come first (they
  // start first and take longest), then the parts, then the short tiles; within each kind XCD x takes a contiguous
  // stretch, so neighbouring tiles (they share operand panels) share an L2.
  const int xcd = blockIdx.x & 7;
  int slot = blockIdx.x >> 3;
  const int parts = (a.long_tiles - a.whole_tiles) * a.cuts;
  const int per1 = (a.whole_tiles + 7) >> 3, per2 = (parts + 7) >> 3, per3 = (a.total_tiles - a.long_tiles + 7) >> 3;
  int t, c = -1;
  if (slot < per1) {
    t = xcd * per1 + slot;
    if (t >= a.whole_tiles) return;
  } else if ((slot -= per1) < per2) {
    const int i = xcd * per2 + slot;
    if (i >= parts) return;
    t = a.whole_tiles + i / a.cuts; c = i % a.cuts;
  } else {
    slot -= per2;
    t = a.long_tiles + xcd * per3 + slot;
    if (slot >= per3 || t >= a.total_tiles) return;
  }
  int bid;
  const int j = grouped_locate(a, t, bid);
  MfmaArgs p = grouped_problem(a, j);
  if (c >= 0) {
    const int nkt = p.kt_per_split, per = (nkt + a.cuts - 1) / a.cuts;
    p.k_range = 1; p.kt_first = min(c * per, nkt); p.kt_count = min(per, nkt - p.kt_first);
    p.tile_partial = a.ws + ((size_t)(t - a.whole_tiles) * a.cuts + c) * SLOT_FLOATS;
  }
  gemm_mfma_tile<true, true, 128>(p, bid, 0);
}
// One workgroup per divided tile: the sum of its parts, added in ascending k.
__global__ __launch_bounds__(256) void gemm_mfma_balanced_sum_kernel(BalancedArgs a) {
  const int d = blockIdx.x >> 2, quarter = blockIdx.x & 3, t = a.whole_tiles + d;   // 4 workgroups per tile, 32 rows each
  int bid;
  const int j = grouped_locate(a, t, bid);
  const GroupedProblem& q = a.prob[j];
  const int m0 = (bid / q.tiles_n) * BM, n0 = (bid % q.tiles_n) * BN;
  const int tid = threadIdx.x, c4 = (tid & 31) * 4;
  const float* slot0 = a.ws + (size_t)d * a.cuts * SLOT_FLOATS;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = quarter * 32 + r * 8 + (tid >> 5);
    float4 acc = *reinterpret_cast<const float4*>(slot0 + row * BN + c4);
    for (int c = 1; c < a.cuts; ++c) {
      const float4 v = *reinterpret_cast<const float4*>(slot0 + (size_t)c * SLOT_FLOATS + row * BN + c4);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const int m = m0 + row, n = n0 + c4;
    if (m < q.M && n < q.N) *reinterpret_cast<float4*>(q.C + (size_t)m * q.ldc + n) = acc;   // N is a multiple of 8
  }
  if (quarter == 0 && q.colsum && m0 == 0 && tid < BN) {
    float acc = slot0[BM * BN + tid];
    for (int c = 1; c < a.cuts; ++c) acc += slot0[(size_t)c * SLOT_FLOATS + BM * BN + tid];
    if (n0 + tid < q.N) q.colsum[n0 + tid] = acc;
  }
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

bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }
// bytes from the first to one past the last element of an operand (transposed: [K][rows], else [rows][K])
long operand_bytes(bool transposed, int rows, int K, long ld) {
  return 2 * (transposed ? (long)(K - 1) * ld + rows : (long)(rows - 1) * ld + K);
}
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
  // the kernel addresses every buffer with 32-bit byte offsets
  const long lim = (1L << 30) - 64;
  if (operand_bytes(at, g.M, g.K, lda) > lim || operand_bytes(bt, g.N, g.K, ldb) > lim) return false;
  if (((long)(g.M - 1) * g.ldc + g.N) * 4 > lim) return false;
  if (g.residual && ((long)(g.M - 1) * g.ldr + g.N) * 2 > lim) return false;
  if (g.epilogue == EPI_DGELU && ((long)(g.M - 1) * g.ldaux + g.N) * 2 > lim) return false;
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

// True when a set of products can go into one grouped launch: each a transposed-transposed product
// with a plain fp32 output (what a weight gradient is).
bool gemm_mfma_groupable(const GemmArgs& g) {
  if (!gemm_mfma_supported(g)) return false;
  const bool at = g.a_sm == 1 && g.a_sk != 1, bt = g.b_sn == 1 && g.b_sk != 1;
  return at && bt && !g.bias && !g.residual && g.epilogue == EPI_NONE && g.c_dt == F32;
}

// Workgroups of a balanced grouped launch on the current device: one per compute unit, a multiple of 8.
static int balanced_workgroups() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return (cus / 8) * 8;
}
// More than 64 KB of dynamic LDS needs an opt-in per kernel, and the attribute belongs to a device's copy of the
// kernel: true (once per device and flag set) when the caller still has to raise it on the current device.
static bool lds_opt_in_due(std::atomic<bool> (&done)[64]) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return true;
  return !done[dev].exchange(true);
}
constexpr int BALANCED_MAX_CUTS = 4;
// room for the parts of the divided tiles: at most two per workgroup
size_t gemm_mfma_balanced_floats() { return (size_t)balanced_workgroups() * 2 * SLOT_FLOATS; }

static void fill_problem(GroupedProblem& q, const GemmArgs& g, int first_tile) {
  q.A = (const uint16_t*)g.A; q.lda = (int)g.a_sk; q.B = (const uint16_t*)g.B; q.ldb = (int)g.b_sk;
  q.C = (float*)g.C; q.ldc = (int)g.ldc; q.colsum = g.colsum;
  q.M = g.M; q.N = g.N; q.K = g.K;
  q.tiles_m = (g.M + BM - 1) / BM; q.tiles_n = (g.N + BN - 1) / BN;
  q.first_tile = first_tile;
  q.a_bytes = (uint32_t)operand_bytes(true, g.M, g.K, g.a_sk);
  q.b_bytes = (uint32_t)operand_bytes(true, g.N, g.K, g.b_sk);
  q.c_bytes = (uint32_t)(((long)(g.M - 1) * g.ldc + g.N) * 4);
}

int launch_gemm_mfma_grouped(hipStream_t s, const GemmArgs* gs, int n, float* ws, size_t ws_floats) {
  static std::atomic<bool> opted_in[64];
  if (lds_opt_in_due(opted_in)) {
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_grouped_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(true, true, 128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_balanced_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(true, true, 128)));
  }
  // Balanced launch: the whole set in one launch, a workspace for the divided tiles, tiles that leave a last round
  // partly filled, and a reduction long enough to cut
  const int wgs = balanced_workgroups();
  if (ws && wgs >= 8 && n <= GROUP_MAX && ws_floats >= (size_t)wgs * 2 * SLOT_FLOATS) {
    BalancedArgs a{};
    a.n = n; a.ws = ws;
    constexpr int LONG_NKT = 32;                    // k-steps from which a reduction counts as long
    int tiles = 0, min_nkt = 1 << 30, filled = 0;
    double flops = 0.0;
    for (int pass = 0; pass < 2; ++pass) {          // long reductions first, then the short ones
      for (int j = 0; j < n; ++j) {
        const int nkt = (gs[j].K + BK - 1) / BK;
        if ((nkt >= LONG_NKT) != (pass == 0)) continue;
        fill_problem(a.prob[filled], gs[j], tiles);
        tiles += a.prob[filled].tiles_m * a.prob[filled].tiles_n;
        ++filled;
        if (pass == 0) min_nkt = std::min(min_nkt, nkt);
        flops += 2.0 * gs[j].M * gs[j].N * gs[j].K;
      }
      if (pass == 0) a.long_tiles = tiles;
    }
    const int rest = a.long_tiles % wgs;
    // parts per left-over tile: 2, more when the left-over tiles are few (measured at 89 left-over tiles on 256 units:
    // 2 parts 124 + 10 us for the two kernels, 3 parts 123 + 13, 4 parts 121 + 16; undivided 160), each of 8 k-steps or
    // more, within the workspace
    int cuts = rest > 0 ? std::max(2, wgs / (2 * rest)) : 1;
    cuts = std::min(cuts, BALANCED_MAX_CUTS);
    while (cuts > 1 && (min_nkt / cuts < 8 || (long)rest * cuts > 2L * wgs)) --cuts;
    if (rest > 0 && cuts > 1) {
      a.total_tiles = tiles; a.whole_tiles = a.long_tiles - rest; a.cuts = cuts;
      void* prof = nullptr;
      PPLL_TRY(profile_begin(s, flops, &prof));
      const int parts = rest * cuts;
      const int grid = 8 * ((a.whole_tiles + 7) / 8 + (parts + 7) / 8 + (tiles - a.long_tiles + 7) / 8);
      hipLaunchKernelGGL(gemm_mfma_balanced_kernel, dim3(grid), dim3(256), lds_bytes(true, true, 128), s, a);
      PPLL_HIP(hipGetLastError());
      hipLaunchKernelGGL(gemm_mfma_balanced_sum_kernel, dim3(4 * rest), dim3(256), 0, s, a);
      PPLL_HIP(hipGetLastError());
      PPLL_TRY(profile_end(s, prof));
      return PPLL_OK;
    }
  }

  for (int j0 = 0; j0 < n; j0 += GROUP_MAX) {
    GroupedArgs a{};
    a.n = n - j0 < GROUP_MAX ? n - j0 : GROUP_MAX;
    int tiles = 0;
    double flops = 0.0;
    for (int j = 0; j < a.n; ++j) {
      const GemmArgs& g = gs[j0 + j];
      fill_problem(a.prob[j], g, tiles);
      tiles += a.prob[j].tiles_m * a.prob[j].tiles_n;
      flops += 2.0 * g.M * g.N * g.K;
    }
    a.total_tiles = tiles;
    a.per_xcd = (tiles + 7) / 8;
    void* prof = nullptr;
    PPLL_TRY(profile_begin(s, flops, &prof));
    hipLaunchKernelGGL(gemm_mfma_grouped_kernel, dim3(8 * a.per_xcd), dim3(256), lds_bytes(true, true, 128), s, a);
    PPLL_HIP(hipGetLastError());
    PPLL_TRY(profile_end(s, prof));
  }
  return PPLL_OK;
}

int launch_gemm_mfma(hipStream_t s, const GemmArgs& g, float* partial, size_t partial_floats) {
  const bool at = g.a_sm == 1 && g.a_sk != 1, bt = g.b_sn == 1 && g.b_sk != 1;
  MfmaArgs p{};
  p.A = (const uint16_t*)g.A; p.lda = at ? g.a_sk : g.a_sm;
  p.B = (const uint16_t*)g.B; p.ldb = bt ? g.b_sk : g.b_sn;
  p.C = g.C; p.c_f32 = g.c_dt == F32; p.ldc = g.ldc;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.tiles_n = (g.N + BN - 1) / BN;
  // 64-row tiles when 128-row tiles would leave more than half of the compute units without a workgroup
  // (between 128 and 256 tiles the 128-row kernel was measured faster: 18.2 against 20.3 us at 8320 x 384 x 1536)
  const bool small_m = !at && ((g.M + BM - 1) / BM) * p.tiles_n < 128;
  const int tm_rows = small_m ? 64 : BM;
  p.tiles_m = (g.M + tm_rows - 1) / tm_rows;
  p.bias = g.bias; p.residual = (const uint16_t*)g.residual; p.ldr = g.ldr;
  p.epilogue = g.epilogue; p.C2 = (uint16_t*)g.C2; p.aux = (const uint16_t*)g.aux; p.ldaux = g.ldaux;
  const int nkt = (g.K + BK - 1) / BK;
  int splits = 1;
  const bool plain = !g.bias && !g.residual && g.epilogue == EPI_NONE && g.c_dt == F32 && g.ldc == g.N;
  if (plain && partial) {
    splits = gemm_mfma_splits(g.M, g.N, g.K);
    if ((size_t)splits * g.M * g.N + (size_t)splits * g.N > partial_floats) splits = 1;
    if ((size_t)splits * g.M * g.N * 4 > ((size_t)1 << 30) - 64) splits = 1;
  }
  float* colsum_partial = splits > 1 ? partial + (size_t)splits * g.M * g.N : nullptr;
  p.colsum = g.colsum ? (splits > 1 ? colsum_partial : g.colsum) : nullptr;
  p.kt_per_split = (nkt + splits - 1) / splits;
  p.partial = splits > 1 ? partial : nullptr;
  p.splits = splits;
  p.a_bytes = (uint32_t)operand_bytes(at, g.M, g.K, p.lda);
  p.b_bytes = (uint32_t)operand_bytes(bt, g.N, g.K, p.ldb);
  p.c_bytes = (uint32_t)(((long)(g.M - 1) * g.ldc + g.N) * (p.c_f32 ? 4 : 2));
  p.r_bytes = g.residual ? (uint32_t)(((long)(g.M - 1) * g.ldr + g.N) * 2) : 0u;
  p.aux_bytes = g.epilogue == EPI_DGELU ? (uint32_t)(((long)(g.M - 1) * g.ldaux + g.N) * 2) : 0u;
  p.partial_bytes = splits > 1 ? (uint32_t)((size_t)splits * g.M * g.N * 4) : 0u;
  p.xcd_map = (splits > 1 && splits % 8 == 0) ? 2 : (p.tiles_m >= 16 ? 1 : 0);
  dim3 grid(p.tiles_m * p.tiles_n, splits);
  if (p.xcd_map == 1) grid = dim3(((p.tiles_m + 7) / 8) * 8 * p.tiles_n, splits);
  if (p.xcd_map == 2) grid = dim3(p.tiles_m * p.tiles_n * splits, 1);
  static std::atomic<bool> opted_in[64];
  if (lds_opt_in_due(opted_in)) {
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<true, true, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(true, true, 128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<true, false, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(true, false, 128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<false, true, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(false, true, 128)));
    PPLL_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<false, false, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(false, false, 128)));
  }
  void* prof = nullptr;
  PPLL_TRY(profile_begin(s, 2.0 * g.M * g.N * g.K, &prof, g.M < 256 && !at ? 2 : 0));   // few output rows: a class of its own
  if (small_m) {
    if (bt) hipLaunchKernelGGL((gemm_mfma_kernel<false, true, 64>), grid, dim3(256), lds_bytes(false, true, 64), s, p);
    else hipLaunchKernelGGL((gemm_mfma_kernel<false, false, 64>), grid, dim3(256), lds_bytes(false, false, 64), s, p);
  } else if (at && bt) hipLaunchKernelGGL((gemm_mfma_kernel<true, true, 128>), grid, dim3(256), lds_bytes(true, true, 128), s, p);
  else if (at) hipLaunchKernelGGL((gemm_mfma_kernel<true, false, 128>), grid, dim3(256), lds_bytes(true, false, 128), s, p);
  else if (bt) hipLaunchKernelGGL((gemm_mfma_kernel<false, true, 128>), grid, dim3(256), lds_bytes(false, true, 128), s, p);
  else hipLaunchKernelGGL((gemm_mfma_kernel<false, false, 128>), grid, dim3(256), lds_bytes(false, false, 128), s, p);
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
