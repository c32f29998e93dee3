// bf16 GEMM for gfx950: C = epilogue(A B^T), A [M,K] and B [N,K] K-contiguous, fp32 accumulate
// on the MFMA units (v_mfma_f32_16x16x32_bf16: per flop it moves half the accumulator registers of the
// 32x32x16 form, and measured 2 % faster here at a 12 % higher sustained clock).
//
// Tiling.  One workgroup of 512 threads (8 wavefronts, 2 along M x 4 along N) owns a
// 256 x 256 tile of the accumulator and walks K in steps of 64.  Each wavefront owns a
// 128 x 64 sub-tile = 8 x 4 MFMA tiles of 16 x 16 (128 accumulator registers per lane).
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers, no LDS store instructions), two stages of 64 KB.  A direct load writes the 64 lanes'
// 16-byte chunks to consecutive LDS addresses, so a stage is unpadded (128-byte rows) and bank
// conflicts are avoided by permuting the chunks of each row: chunk c of tile row r is stored at
// chunk position c ^ ((r ^ (r >> 3)) & 7), applied on the global side of the load (which chunk a
// lane fetches) and undone in the fragment-read addresses.  Fragment registers are double-buffered;
// the loads of tile kt+2 are issued right after the barrier that ends step kt.
//
// SwiGLU mode (the gate/up projection of one expert, Sec. 3.1): the 256 B-rows of a tile are
// 128 rows of W1 followed by the SAME 128 rows of W3, and each wavefront's four N sub-tiles are
// two (gate, up) pairs for the same 32 output columns, so silu(gate) * up is formed in registers and
// only the product is written, rounded once to bf16.
//
// Grouped mode (dynamic skipping, Sec. 3.3): M tiles are looked up in a device-side tile map
// (expert, first row); rows of A may be gathered through an index list.
//
// Workgroup order: consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with a
// private L2.  Ids are remapped so that every XCD works on a contiguous run of tiles, ordered
// 8 (gate/up) or 4 (down) M-tiles deep before moving along N, so that the 32 tiles in flight on one
// XCD share operand panels.
#include "common.h"

namespace moep {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // one 16-byte chunk

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int THREADS = 512;
constexpr int ROW_BYTES = 128;                 // 64 bf16, unpadded (chunks are permuted instead)
constexpr int TILE_BYTES = BM * ROW_BYTES;     // one operand tile (BM == BN)
constexpr int STAGE_BYTES = 2 * TILE_BYTES;    // A tile then B tile
constexpr int LDS_BYTES = 2 * STAGE_BYTES;     // 131072
static_assert(BM == GEMM_BM, "grouped tile maps are built for 256-row tiles");

struct KArgs {
  const u32x4* A; const u32x4* B0; const u32x4* B1;
  const int32_t* a_rows;
  void* C;
  const float* row_scale;
  const int32_t* tile_expert; const int32_t* tile_row0; const int32_t* seg_end;
  const int32_t* tiles_in_use;
  int64_t M, ldc;
  uint32_t lda_chunks, ldb_chunks;   // leading dimensions in 16-byte chunks
  int64_t b_expert_chunks;           // expert stride of B in 16-byte chunks
  int N, K;
  int m_tiles, n_tiles;
};

template <int EPI>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_bf16_kernel(KArgs p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- which tile -------------------------------------------------------------
  // Grouped launches are sized for the largest possible tile map; only its leading entries hold work.
  // Spreading just those over the XCDs keeps every XCD busy (the launch's surplus workgroups leave here).
  const uint32_t m_tiles = p.tiles_in_use ? (uint32_t)*p.tiles_in_use : (uint32_t)p.m_tiles;
  const uint32_t nblk = p.tiles_in_use ? m_tiles * (uint32_t)p.n_tiles : gridDim.x;
  uint32_t bid = blockIdx.x;
  if (bid >= nblk) return;
  {  // XCD-aware remap: ids i, i+8, i+16, ... run on XCD i % 8; give each XCD a contiguous run.
    const uint32_t per = nblk >> 3, rem = nblk & 7;
    const uint32_t xcd = bid & 7, j = bid >> 3;
    bid = xcd * per + (xcd < rem ? xcd : rem) + j;
  }
  constexpr uint32_t GROUP_M = EPI == EPI_SWIGLU ? 8 : 4;   // measured: the long-K down projection prefers 4 x 8 tiles per XCD
  const uint32_t group_sz = GROUP_M * p.n_tiles;
  const uint32_t group = bid / group_sz;
  const uint32_t first_m = group * GROUP_M;
  const uint32_t gm = min(m_tiles - first_m, GROUP_M);
  const uint32_t in_group = bid - group * group_sz;
  const int tm = first_m + in_group % gm;
  const int tn = in_group / gm;

  int64_t row0, row_end;
  const u32x4* B0 = p.B0;
  const u32x4* B1 = p.B1;
  if (p.tile_expert) {
    const int e = p.tile_expert[tm];
    if (e < 0) return;                               // uniform over the workgroup
    row0 = p.tile_row0[tm];
    row_end = p.seg_end[e];
    B0 += (int64_t)e * p.b_expert_chunks;
    if (EPI == EPI_SWIGLU) B1 += (int64_t)e * p.b_expert_chunks;
  } else {
    row0 = (int64_t)tm * BM;
    row_end = p.M;
  }

  // ---- global -> LDS direct loads ---------------------------------------------------
  // Wavefront w fills tile rows 32 w .. 32 w + 31 of both operands: 4 loads per operand, each
  // 8 rows x 8 chunks = 1 KB of LDS written contiguously in lane order.  Lane l lands on row
  // (l >> 3), chunk position (l & 7) of its 8-row group and therefore fetches chunk
  // (l & 7) ^ swz(row) of that row from global memory.
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  uint32_t a_off[4], b_off[4];
  const u32x4* b_base;
  {
    const int rr0 = wave_u * 32;                       // uniform: first tile row of this wavefront
    if (EPI == EPI_SWIGLU) b_base = rr0 < 128 ? B0 : B1;   // rows 0..127 gate, 128..255 up
    else b_base = B0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tr = rr0 + 8 * i + (lane >> 3);        // tile row
      const int cch = (lane & 7) ^ ((tr ^ (tr >> 3)) & 7);
      int64_t r = row0 + tr;
      if (r >= row_end) r = row_end - 1;               // tail rows re-read the last valid row
      const int64_t src = p.a_rows ? (int64_t)p.a_rows[r] : r;
      a_off[i] = (uint32_t)src * p.lda_chunks + cch;
      // LDS row 32 P + 16 b + f of the B tile holds weight row 32 P + 8 (f >> 2) + 4 b + (f & 3) (see epilogue).
      const int trp = (tr & ~31) | ((tr & 12) << 1) | ((tr & 16) >> 2) | (tr & 3);
      int n = EPI == EPI_SWIGLU ? tn * 128 + (trp & 127) : tn * BN + trp;
      if (n >= p.N) n = p.N - 1;
      b_off[i] = (uint32_t)n * p.ldb_chunks + cch;
    }
  }
  typedef __attribute__((address_space(3))) char lds_char;
  typedef const __attribute__((address_space(1))) void* gptr_t;
  lds_char* const lds3 = (lds_char*)lds;
#define MOEP_LOAD_TILE(kt, stage)                                                             \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                             \
    __builtin_amdgcn_global_load_lds((gptr_t)(p.A + a_off[i] + (uint32_t)(kt) * 8u),          \
        (__attribute__((address_space(3))) void*)(lds3 + (stage) * STAGE_BYTES +              \
                                                  (wave_u * 32 + 8 * i) * ROW_BYTES), 16, 0, 0); \
    __builtin_amdgcn_global_load_lds((gptr_t)(b_base + b_off[i] + (uint32_t)(kt) * 8u),       \
        (__attribute__((address_space(3))) void*)(lds3 + (stage) * STAGE_BYTES + TILE_BYTES + \
                                                  (wave_u * 32 + 8 * i) * ROW_BYTES), 16, 0, 0); \
  }

  // ---- fragment addresses ---------------------------------------------------------
  // MFMA 16x16x32: lane l supplies row (l & 15) and the 8 k-values 8 (l >> 4) .. + 7 of A, and the
  // same for B (as [N,K]); a K step of 64 is two slices: chunk 4 s + (l >> 4) of the row, found at
  // position chunk ^ swz(row); swz only touches the low chunk bits, so slice s is at
  // (address of slice 0) ^ (s << 6).
  const int frow = lane & 15, fk = lane >> 4;
  int a_frag[8], b_frag[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int tr = wm * 128 + i * 16 + frow;
    a_frag[i] = tr * ROW_BYTES + ((fk ^ ((tr ^ (tr >> 3)) & 7)) << 4);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tr = EPI == EPI_SWIGLU ? (j >> 1) * 128 + wn * 32 + (j & 1) * 16 + frow : wn * 64 + j * 16 + frow;
    b_frag[j] = TILE_BYTES + tr * ROW_BYTES + ((fk ^ ((tr ^ (tr >> 3)) & 7)) << 4);
  }

  f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  // Step kt of the K loop works on stage cur = kt & 1, two slices of 32 k-values:
  //   slice 0: read slice 1, MFMAs of slice 0 (reads issued in the MFMAs' shadow, one per two MFMAs)
  //   wait until this wavefront's loads of tile kt+1 have landed and its own reads are done,
  //   barrier (now every wavefront has read all of stage cur and stage cur^1 is complete),
  //   issue the loads of tile kt+2 into stage cur, read slice 0 of the other stage,
  //   MFMAs of slice 1.
  bf16x8 fa[2][8], fb[2][4];
#define MOEP_READ_FRAGS(stage, kk, slot)                                                      \
  {                                                                                           \
    const char* st_ = lds + (stage) * STAGE_BYTES;                                            \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                             \
      fb[slot][j] = *(const bf16x8*)(st_ + (b_frag[j] ^ ((kk) << 6)));                        \
    _Pragma("unroll") for (int i = 0; i < 8; ++i)                                             \
      fa[slot][i] = *(const bf16x8*)(st_ + (a_frag[i] ^ ((kk) << 6)));                        \
  }
#define MOEP_MFMA(slot)                                                                       \
  _Pragma("unroll") for (int i = 0; i < 8; ++i)                                               \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                             \
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
#define MOEP_INTERLEAVE_READS()                                                               \
  _Pragma("unroll") for (int q_ = 0; q_ < 12; ++q_) {                                         \
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                        \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                        \
  }                                                                                           \
  __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
#define MOEP_WAIT_ALL() __builtin_amdgcn_s_waitcnt(0x0070)
#define MOEP_STEP(kt, HAS_NEXT, HAS_NEXT2)                                                    \
  {                                                                                           \
    const int cur_ = (kt) & 1;                                                                \
    MOEP_READ_FRAGS(cur_, 1, 1)                                                               \
    MOEP_MFMA(0)                                                                              \
    MOEP_INTERLEAVE_READS()                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                        \
    MOEP_WAIT_ALL();                                                                          \
    __builtin_amdgcn_s_barrier();                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                        \
    if (HAS_NEXT2) { MOEP_LOAD_TILE((kt) + 2, cur_) }                                         \
    if (HAS_NEXT) MOEP_READ_FRAGS(cur_ ^ 1, 0, 0)                                             \
    MOEP_MFMA(1)                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                        \
  }

  const int nk = p.K / BK;
  MOEP_LOAD_TILE(0, 0)
  MOEP_WAIT_ALL();
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  if (nk > 1) { MOEP_LOAD_TILE(1, 1) }
  MOEP_READ_FRAGS(0, 0, 0)
  __builtin_amdgcn_sched_barrier(0);
  int kt = 0;
  for (; kt + 2 < nk; ++kt) MOEP_STEP(kt, true, true)
  if (kt + 1 < nk) {
    MOEP_STEP(kt, true, false)
    ++kt;
  }
  MOEP_STEP(kt, false, false)
#undef MOEP_LOAD_TILE
#undef MOEP_READ_FRAGS
#undef MOEP_MFMA
#undef MOEP_STEP
#undef MOEP_INTERLEAVE_READS
#undef MOEP_WAIT_ALL

  // ---- epilogue ---------------------------------------------------------------------
  // The MFMAs were issued with the weight fragment as the first operand, so a 16x16 accumulator tile is
  // the TRANSPOSE of the output tile: register v of lane l holds output row (l % 16) of row group i and
  // fragment row f = 4 (l / 16) + v of weight tile j.  The B tile was loaded with its rows permuted inside
  // every block of 32 (LDS row 32 P + 16 b + f = weight row 32 P + 8 (f / 4) + 4 b + f % 4), hence tiles
  // 2 P and 2 P + 1 together give each lane 8 CONSECUTIVE output columns 32 P + 8 (l / 16) .. + 7:
  // one 16-byte store of bf16 (two of fp32) per lane, 64 contiguous bytes per row and store.
  const int q8 = 8 * (lane >> 4);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t r = row0 + wm * 128 + i * 16 + (lane & 15);
    if (r >= row_end) continue;
    if (EPI == EPI_SWIGLU) {
      const int n = tn * 128 + wn * 32 + q8;
      if (n < p.N) {
        bf16x2 o[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          f32x2 h;
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const int b = c >> 1, v = 2 * (c & 1) + d;
            const float g = acc[i][b][v], u = acc[i][2 + b][v];
            h[d] = g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
          }
          o[c] = __builtin_convertvector(h, bf16x2);
        }
        *(u32x4*)((uint16_t*)p.C + r * p.ldc + n) = __builtin_bit_cast(u32x4, o);
      }
    } else {
#pragma unroll
      for (int P = 0; P < 2; ++P) {
        const int n = tn * BN + wn * 64 + 32 * P + q8;
        if (n >= p.N) continue;
        if (EPI == EPI_STORE) {
          bf16x2 o[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const f32x2 h = {acc[i][2 * P + (c >> 1)][2 * (c & 1)], acc[i][2 * P + (c >> 1)][2 * (c & 1) + 1]};
            o[c] = __builtin_convertvector(h, bf16x2);
          }
          *(u32x4*)((uint16_t*)p.C + r * p.ldc + n) = __builtin_bit_cast(u32x4, o);
        } else {
          const float sc = p.row_scale[r];
          float* dst = (float*)p.C + r * p.ldc + n;
          *(f32x4*)dst = sc * acc[i][2 * P];
          *(f32x4*)(dst + 4) = sc * acc[i][2 * P + 1];
        }
      }
    }
  }
}

template <int EPI>
int launch(const KArgs& k, uint32_t blocks, hipStream_t s) {
  static bool attr_set = false;   // raising the dynamic LDS limit is per function, once
  if (!attr_set) {
    MOEP_HIP(hipFuncSetAttribute((const void*)gemm_bf16_kernel<EPI>,
                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
    attr_set = true;
  }
  hipLaunchKernelGGL(gemm_bf16_kernel<EPI>, dim3(blocks), dim3(THREADS), LDS_BYTES, s, k);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace

int launch_gemm_bf16(const GemmArgs& g, hipStream_t s, const char* name) {
  if (g.K % BK || g.K <= 0) return fail(MOEP_EUNSUPPORTED, "%s: K=%d must be a positive multiple of %d", name, g.K, BK);
  if (g.lda % 8 || g.ldc <= 0) return fail(MOEP_EINVAL, "%s: bad leading dimension", name);
  if (g.M <= 0 || g.N <= 0) return MOEP_OK;
  // 16-byte loads and stores: operand bases and row pitches must keep every 8-element group aligned
  if (((uintptr_t)g.A | (uintptr_t)g.B0 | (uintptr_t)g.B1 | (uintptr_t)g.C) & 15)
    return fail(MOEP_EUNSUPPORTED, "%s: operands must be 16-byte aligned", name);
  if (g.N % 8 || g.ldc % 8) return fail(MOEP_EUNSUPPORTED, "%s: N=%d and ldc must be multiples of 8", name, g.N);
  KArgs k;
  k.A = (const u32x4*)g.A; k.B0 = (const u32x4*)g.B0; k.B1 = (const u32x4*)g.B1;
  k.a_rows = g.a_rows; k.C = g.C; k.row_scale = g.row_scale;
  k.tile_expert = g.tile_expert; k.tile_row0 = g.tile_row0; k.seg_end = g.seg_end;
  k.tiles_in_use = g.tile_expert ? g.tiles_in_use : nullptr;
  k.M = g.M; k.ldc = g.ldc;
  k.lda_chunks = (uint32_t)(g.lda / 8); k.ldb_chunks = (uint32_t)(g.K / 8);
  k.b_expert_chunks = g.b_expert_stride / 8;
  k.N = g.N; k.K = g.K;
  const int64_t m_tiles = g.tile_expert ? g.max_m_tiles : ceil_div(g.M, BM);
  const int64_t n_tiles = g.epilogue == EPI_SWIGLU ? ceil_div(g.N, 128) : ceil_div(g.N, BN);
  // Row offsets are kept as 32-bit counts of 16-byte chunks.
  const int64_t a_rows_max = g.a_rows ? g.M : m_tiles * BM;   // gathered rows index x, checked by the caller
  if (a_rows_max * (g.lda / 8) >= ((int64_t)1 << 32) || (int64_t)g.N * (g.K / 8) >= ((int64_t)1 << 32))
    return fail(MOEP_EUNSUPPORTED, "%s: operand larger than 64 GiB", name);
  if (m_tiles * n_tiles >= ((int64_t)1 << 31)) return fail(MOEP_EUNSUPPORTED, "%s: too many tiles", name);
  k.m_tiles = (int)m_tiles; k.n_tiles = (int)n_tiles;
  const uint32_t blocks = (uint32_t)(m_tiles * n_tiles);
  Timed t(name, s);
  switch (g.epilogue) {
    case EPI_STORE: return launch<EPI_STORE>(k, blocks, s);
    case EPI_SWIGLU: return launch<EPI_SWIGLU>(k, blocks, s);
    case EPI_ROWSCALE_F32: return launch<EPI_ROWSCALE_F32>(k, blocks, s);
  }
  return fail(MOEP_EINVAL, "%s: unknown epilogue %d", name, g.epilogue);
}

}  // namespace moep
