// bf16 GEMM for gfx950 on PACKED operands: C = epilogue(A B^T), fp32 accumulate on the MFMA units
// (v_mfma_f32_16x16x32_bf16).  Every bf16 expert GEMM runs here: the dense pass (every expert on every
// token, Sec. 3.1 / Sec. 3.2) and, in grouped mode, the routed rows of the skipping forward (Sec. 3.3)
// and of the rank-limited pass.  The operands are re-read many times; re-laying them out once is
// almost free.
//
// Packed layout.  A matrix X [R, K] is cut into blocks of 256 rows x 32 k-values ("slices").  Block
// (row tile t, slice s) is 16 KB, stored contiguously at ((t * K/32) + s) * 16 KB; inside it row p
// takes 64 bytes and its four 16-byte chunks are permuted, chunk c at position c ^ ((p >> 2) & 3).
// That is exactly the image the kernel wants in LDS (fragment reads of 16 consecutive rows are then
// free of bank conflicts), so a wavefront's direct global->LDS load moves 1 KB of CONSECUTIVE bytes:
// eight full cache lines per instruction whatever K is, where the row-major layout offers 128-byte
// pieces one row pitch apart (or half lines, with 32-wide slices).
// Weight blocks carry two more permutations (see pack_kernel): the rows of every group of 32 are
// reordered so that the transposed accumulator tiles give each lane 8 consecutive output columns, and
// for the gate/up projection a block holds 128 rows of W1 followed by the same 128 rows of W3.
//
// Kernel.  One workgroup of 256 threads (4 wavefronts, 2 along M x 2 along N, one per SIMD) owns a
// 256 x 256 tile of the accumulator (256 x 128 outputs in SwiGLU mode); a wavefront owns 128 x 128 =
// 8 x 8 MFMA tiles, whose 256 accumulator registers sit in the AGPR half of the wavefront's 512 registers.
// K is walked one slice (one MFMA depth) at a time through a ring of NS = 5 LDS stages of 32 KB.  In
// the step that multiplies slice g a wavefront also issues its 8 direct loads of slice g + NS - 1 (one
// per 6 MFMAs, into the stage whose fragments were read two steps ago) and reads the fragments of slice
// g + 1 into the other half of a double-buffered fragment register set: 64 MFMAs, 16 LDS reads and 8
// loads per step.  Loads are spread evenly over the step, never issued in bursts.  The wavefronts
// meet at a barrier every SECOND step only: before it each waits until all but its 8 newest loads have
// landed, which covers the two slices read in the two steps that follow; the stage a step's loads
// overwrite was last read two steps earlier, i.e. before the previous barrier.
// Workgroups are persistent (one per compute unit) and the ring runs across tile boundaries: while the
// last slices of a tile are multiplied and its epilogue runs, the first slices of the workgroup's next
// tile are already being fetched.  The loader changes tile only BETWEEN runs of steps (a tile's steps
// are cut where the loader, NS - 1 slices ahead, reaches the end of its tile), so the hot loop is a
// single basic block of two steps with no tile bookkeeping in it; with a branch in the loop the
// register allocator moved accumulators between AGPRs and VGPRs on every step.
//
// The 32 workgroups of an XCD are kept in step, round of tiles by round of tiles, through a counter in
// device memory (bounded wait, see round_sync).
//
// Epilogues.  The MFMAs take the weight fragment as first operand, so an accumulator tile is the
// transpose of the output tile and (with the row permutation above) a lane holds 8 consecutive output
// columns of one row: one 16-byte store.  SwiGLU mode (Sec. 3.1) forms silu(gate) * up in registers,
// rounds once to bf16 and writes the result in the PACKED layout of an A operand with K = N, ready
// for the down projection: 16 rows x 64 bytes = 1 KB contiguous per wavefront store.
//
// Workgroup order: logical tile ids are dealt round-robin to the 8 XCDs (as the hardware deals
// workgroups) and remapped so that every XCD works on a contiguous run of tiles, GROUP_M M-tiles deep
// before moving along N, so that the 32 tiles in flight on one XCD share operand panels in its L2.
// Grouped launches read that order from a table the dispatch kernels lay out, with the groups of M tiles
// aligned to the experts' segments (a group that straddled two experts would share no weight panel).
#include <mutex>

#include "common.h"

namespace moep {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // one 16-byte chunk

constexpr int THREADS = 256;
constexpr int SYNC_POLLS = 64;                // bound of a workgroup's wait for the others of its XCD
constexpr uint32_t SYNC_EVERY = 4;            // tiles between two line-ups (1: 0.9 % slower; the L2 hit rate is the same)
constexpr int NS = 5;                       // ring stages
constexpr int SLICE = 256 * 64;             // one operand block: 256 rows x 32 bf16
constexpr int STAGE = 2 * SLICE;            // A block then B block
constexpr int LDS_BYTES = NS * STAGE;       // 160 KB
static_assert(GEMM_BM == 256, "tiles are 256 rows");
static_assert((NS - 1) % 2 == 0, "the loader must be an even number of slices ahead (steps come in pairs)");

// LDS row p of a weight block holds weight row perm32(p) of the tile: inside every group of 32 rows,
// LDS row 16 b + f is weight row 8 (f >> 2) + 4 b + (f & 3).
__host__ __device__ constexpr int perm32(int p) {
  return (p & ~31) | ((p & 12) << 1) | ((p & 16) >> 2) | (p & 3);
}

// ---- packing ---------------------------------------------------------------------------------
// mode 0: A operand, block row p of tile t = source row 256 t + p.
// mode 1: weight, 256 output columns per tile: block row p = row 256 t + perm32(p) of W0.
// mode 2: gate/up weight pair, 128 output columns per tile: block row p < 128 = row 128 t + perm32(p) of
//         W0, block row p >= 128 = row 128 t + perm32(p - 128) of W1.
// mode 3: gathered A operand of a grouped GEMM: block row p of tile t = source row rows_of[tile_row0[t] + p]
//         (the rows routed to the tile's expert, Sec. 3.3); tiles beyond the number in use are left alone.
// Rows beyond the last one re-read the last row (their products are never stored).
// One workgroup moves a pair of slices (64 k-values) of one tile, so that whole 128-byte lines are read;
// blockIdx.z selects the expert of a weight stack.
struct PackArgs {
  const u32x4* W0; const u32x4* W1;
  u32x4* dst;
  int64_t ld_chunks;      // source leading dimension in 16-byte chunks
  int64_t rows;           // valid source rows (modes 0..2)
  int64_t src_expert_chunks, dst_expert_chunks;   // per-expert strides (blockIdx.z)
  const int32_t* rows_of; const int32_t* tile_expert; const int32_t* tile_row0; const int32_t* seg_end;
  const int32_t* tiles_in_use;
  int nsl;                // K / 32
  int mode;
};

__global__ __launch_bounds__(256) void pack_kernel(PackArgs p) {
  const int t = blockIdx.x;
  const int sp = blockIdx.y;                 // slice pair
  const u32x4* W0 = p.W0 + (int64_t)blockIdx.z * p.src_expert_chunks;
  const u32x4* W1 = p.W1 + (int64_t)blockIdx.z * p.src_expert_chunks;
  u32x4* dst = p.dst + (int64_t)blockIdx.z * p.dst_expert_chunks;
  int64_t g_row0 = 0, g_end = 0;
  if (p.mode == 3) {
    if (t >= *p.tiles_in_use) return;
    g_row0 = p.tile_row0[t];
    g_end = p.seg_end[p.tile_expert[t]];
  }
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int q = it * 256 + threadIdx.x;    // 2048 chunks: 256 rows x 8 chunks of a 128-byte line
    const int row = q >> 3, c8 = q & 7;
    const u32x4* src = W0;
    int64_t r;
    if (p.mode == 3) {
      int64_t slot = g_row0 + row;
      if (slot >= g_end) slot = g_end - 1;
      r = p.rows_of[slot];
    } else {
      if (p.mode == 0) r = (int64_t)t * 256 + row;
      else if (p.mode == 1) r = (int64_t)t * 256 + perm32(row);
      else {
        r = (int64_t)t * 128 + perm32(row & 127);
        if (row >= 128) src = W1;
      }
      if (r >= p.rows) r = p.rows - 1;
    }
    const u32x4 v = src[r * p.ld_chunks + (int64_t)sp * 8 + c8];
    const int s = 2 * sp + (c8 >> 2);
    const int pos = (c8 & 3) ^ ((row >> 2) & 3);
    dst[((int64_t)t * p.nsl + s) * 1024 + row * 4 + pos] = v;
  }
}

// ---- GEMM --------------------------------------------------------------------------------------
struct KArgs {
  const char* A;          // packed, tile-major
  const char* B;          // packed weight blocks
  void* C;                // EPI_STORE: row-major bf16 [M, ldc]; EPI_SWIGLU: packed A operand with K = N
  int64_t M, ldc;
  int N;                  // output columns
  int nsl;                // K / 32
  int m_tiles, n_tiles;
  // grouped mode (rows partitioned into per-expert segments, tile t = rows tile_row0[t] .. of expert
  // tile_expert[t]; A and a packed C are indexed by TILE, a row-major C by row)
  const int32_t* tile_expert; const int32_t* tile_row0; const int32_t* seg_end; const int32_t* tiles_in_use;
  int64_t b_expert_bytes;
  const float* row_scale;
  // dense batched mode: `experts` independent GEMMs of the same shape in one launch, tile ids expert-major;
  // expert e reads A + e a_expert_bytes (0: A shared), B + e b_expert_bytes, writes C + e c_expert_bytes
  int experts;
  int64_t a_expert_bytes, c_expert_bytes;
  // EPI_ROWSCALE_F32: rows with row_dest[r] >= 0 go, as bf16 and unscaled, to row row_dest[r] of direct_out
  const int32_t* row_dest;
  uint16_t* direct_out;
  const uint32_t* tile_order;   // grouped mode, optional: entry bid = (M tile << 12) | N tile
};

// Round counters of the persistent workgroups, one per XCD (64 bytes apart); see round_sync in the kernel.
// They only ever grow, by a multiple of the XCD's workgroup count per launch; 64 bits wide, so they never wrap.
// Launches that overlap on one GPU share them: their workgroups may then wait for each other up to the
// bound, nothing else.  Workgroup b is taken to run on XCD b % 8 (how this part deals workgroups out); were
// that ever not so, the line-ups would group the wrong workgroups and cost time, never a result.
__device__ unsigned long long g_round_count[8 * 8];

template <int EPI, bool GROUPED>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_packed_kernel(KArgs p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave_u >> 1, wn = wave_u & 1;
  const int nsl = p.nsl;
  // Grouped launches are sized for the largest possible tile map; only its leading entries hold work.
  const uint32_t m_tiles = GROUPED ? (uint32_t)*p.tiles_in_use : (uint32_t)p.m_tiles;
  const uint32_t per_expert = m_tiles * (uint32_t)p.n_tiles;
  const uint32_t nblk = GROUPED ? per_expert : per_expert * (uint32_t)p.experts;
  const uint32_t G = gridDim.x;

  // Logical tile id -> (tm, tn).  Ids i, i + 8, ... belong to XCD i % 8 (the grid is a multiple of 8 or
  // a single round); every XCD gets a contiguous run of tiles, GROUP_M M-tiles deep.
  constexpr uint32_t GROUP_M = EPI == EPI_SWIGLU ? GEMM_GROUP_M_SWIGLU : GEMM_GROUP_M_STORE;
  // weight blocks of the tile's expert
  auto b_tile = [&](int tm_, int tn_, int e_) {
    const char* b = p.B + ((size_t)tn_ * nsl) * SLICE + wave_u * 4096;
    b += (int64_t)(GROUPED ? p.tile_expert[tm_] : e_) * p.b_expert_bytes;
    return b;
  };
  // Dense: e = the GEMM of a batched launch the tile belongs to; each of them is dealt to the XCDs exactly as a
  // launch of its own would be when its tile count is a multiple of 8, else the batch is one flat run of tiles.
  auto decode = [&](uint32_t L, int& tm, int& tn, int& e) {
    const uint32_t xcd = L & 7, j = L >> 3;
    if (GROUPED) {
      // the order of the tiles was laid out by the caller (groups of M tiles aligned to experts, see order_kernel);
      // XCD x walks entries x per + min(x, rem) ... of it
      const uint32_t per = nblk >> 3, rem = nblk & 7;
      const uint32_t v = p.tile_order[xcd * per + (xcd < rem ? xcd : rem) + j];
      e = 0;
      tm = (int)(v >> 12);
      tn = (int)(v & 4095u);
    } else {
      uint32_t bid;
      if ((per_expert & 7) == 0) {
        const uint32_t per8 = per_expert >> 3;
        const uint32_t eu = j / per8;
        e = (int)eu;
        bid = xcd * per8 + (j - eu * per8);
      } else {
        const uint32_t per = nblk >> 3, rem = nblk & 7;
        bid = xcd * per + (xcd < rem ? xcd : rem) + j;
        const uint32_t eu = bid / per_expert;
        e = (int)eu;
        bid -= eu * per_expert;
      }
      const uint32_t group_sz = GROUP_M * (uint32_t)p.n_tiles;
      const uint32_t group = bid / group_sz;
      const uint32_t first_m = group * GROUP_M;
      const uint32_t gm = min(m_tiles - first_m, GROUP_M);
      const uint32_t in_group = bid - group * group_sz;
      tm = (int)(first_m + in_group % gm);
      tn = (int)(in_group / gm);
    }
  };

  // ---- loader state (all wave-uniform) ----------------------------------------------------------
  // A wavefront moves 4 KB of each operand block per slice: KB 4 w .. 4 w + 3.
  uint32_t L_ld = blockIdx.x;
  if (L_ld >= nblk) return;
  int tm_ld, tn_ld, e_ld;
  decode(L_ld, tm_ld, tn_ld, e_ld);
  const char* a_ld = p.A + (int64_t)e_ld * p.a_expert_bytes + ((size_t)tm_ld * nsl) * SLICE + wave_u * 4096;
  const char* b_ld = b_tile(tm_ld, tn_ld, e_ld);
  int s_ld = 0;
  int st_ld = 0;                      // byte offset of the stage the next slice goes to
  bool ld_ok = true;
  const uint32_t lane_off = lane * 16;
  typedef __attribute__((address_space(3))) char lds_char;
  typedef const __attribute__((address_space(1))) void* gptr_t;
  lds_char* const lds3 = (lds_char*)lds;
  // per-lane global addresses of this wavefront's part of the next slice (kept in registers so that the
  // step that issues the loads has no address arithmetic to do first)
  const char* ga = a_ld + lane_off;
  const char* gb = b_ld + lane_off;
#define MOEP_LOAD1(q)                                                                           \
  __builtin_amdgcn_global_load_lds((gptr_t)((q) < 4 ? ga : gb),                                   \
      (__attribute__((address_space(3))) void*)(lds3 + st_ld + ((q) < 4 ? 0 : SLICE) + wave_u * 4096), 16, ((q) & 3) * 1024, 0);
  // After a slice has been issued: next slice, next stage (branch-free, so that it can be scheduled into
  // the shadow of the MFMAs).  Past the end of the workgroup's stream the loader stays on its last slice:
  // the re-reads are in bounds and land in stages nobody reads again, every step issues the same loads and
  // the wait counts below hold to the end.
#define MOEP_ADVANCE_LOADER()                                                                   \
  {                                                                                             \
    const int adv_ = ld_ok ? SLICE : 0;                                                         \
    a_ld += adv_; b_ld += adv_;                                                                 \
    s_ld += ld_ok ? 1 : 0;                                                                      \
    st_ld = st_ld + STAGE == LDS_BYTES ? 0 : st_ld + STAGE;                                     \
    ga = a_ld + lane_off; gb = b_ld + lane_off;                                                 \
  }
  // The workgroups of an XCD start every SYNC_EVERY-th round of tiles together: they share operand panels through the
  // XCD's L2 only while they walk K within a few steps of each other, and left alone they settle, from
  // one build of this file to the next, either there or in a state where every panel is fetched about three
  // times over (L2 hit rate 0.45 instead of 0.80, 7 % slower).  Arrivals are counted in a counter that only
  // grows; every workgroup arrives `arrivals_due` times per launch (its last arrival makes up for the line-ups
  // it did not take part in), so the count stays a multiple of the XCD's workgroup count from launch to launch.  The wait is bounded (SYNC_POLLS polls about a thousand cycles
  // apart); a workgroup that ran into the bound goes on alone and polls no more in this launch.  Only the
  // timing depends on any of this, never a result.
  const uint32_t rounds = (nblk + G - 1) / G;
  const bool sync_on = nblk > G && (G & 7) == 0 && (G >> 3) < 65536u;
  bool poll_ok = true;
  uint32_t switches = 0, arrivals = 0;
  const uint32_t arrivals_due = (rounds + SYNC_EVERY - 1) / SYNC_EVERY;
  auto round_sync = [&](bool last) {
    int w_ = wave_u;                          // (opaque: the comparison is then made here, from a scalar register,
    asm volatile("" : "+s"(w_));              // instead of being kept as a 0/1 value in a vector register across the K loop)
    if (w_ != 0) return;
    unsigned long long* c = &g_round_count[(blockIdx.x & 7) * 8];
    unsigned long long old_v = 0;
    if (lane == 0)
      old_v = __hip_atomic_fetch_add(c, (unsigned long long)(last ? arrivals_due - arrivals : 1u), __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
    ++arrivals;
    if (last || !poll_ok) return;
    // Everyone has arrived when the count reaches the next multiple of n above the value this arrival saw.
    // (wave-uniform 32-bit arithmetic: old mod n from the two halves of the 64-bit count, n < 2^16)
    const uint32_t n = G >> 3;
    const uint32_t old_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)old_v);
    const uint32_t old_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(old_v >> 32));
    const uint32_t two32_mod_n = (0xffffffffu % n + 1u) % n;
    const uint32_t old_mod_n = ((old_hi % n) * two32_mod_n + old_lo % n) % n;
    const uint32_t target_lo = old_lo - old_mod_n + n;          // low word of the target; the count moves by far
    int polls = 0;                                              // less than 2^31 while this workgroup waits
    for (;;) {
      uint32_t now_v = 0;
      if (lane == 0) now_v = (uint32_t)__hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t now = (uint32_t)__builtin_amdgcn_readfirstlane((int)now_v);
      if ((int32_t)(now - target_lo) >= 0) break;
      if (++polls >= SYNC_POLLS) { poll_ok = false; break; }
      __builtin_amdgcn_s_sleep(16);
    }
  };
  // ... and, between runs of steps, the next tile of this workgroup
#define MOEP_NEXT_LOAD_TILE()                                                                   \
  if (s_ld == nsl) {                                                                            \
    s_ld = 0;                                                                                   \
    L_ld += G;                                                                                  \
    ++switches;                                                                                 \
    if (sync_on && (L_ld >= nblk || switches % SYNC_EVERY == 0)) {                               \
      round_sync(L_ld >= nblk);                                                                 \
      __builtin_amdgcn_s_barrier();                                                             \
    }                                                                                           \
    if (L_ld < nblk) {                                                                          \
      decode(L_ld, tm_ld, tn_ld, e_ld);                                                         \
      a_ld = p.A + (int64_t)e_ld * p.a_expert_bytes + ((size_t)tm_ld * nsl) * SLICE + wave_u * 4096; \
      b_ld = b_tile(tm_ld, tn_ld, e_ld);                                                        \
    } else {                                                                                    \
      ld_ok = false;                                                                            \
      a_ld -= SLICE; b_ld -= SLICE;                                                             \
    }                                                                                           \
    ga = a_ld + lane_off; gb = b_ld + lane_off;                                                 \
  }

  // ---- fragment addresses -------------------------------------------------------------------------
  // MFMA 16x16x32: lane l supplies row (l & 15) and k-values 8 (l >> 4) .. + 7 of both operands, i.e.
  // chunk (l >> 4) of the row, found at position chunk ^ ((row >> 2) & 3); tile rows are multiples of 16
  // apart, so the permutation depends on the lane only and every fragment is base + constant.
  const int frow = lane & 15, fk = lane >> 4;
  const int fpos = (fk ^ ((frow >> 2) & 3)) << 4;
  const int a_fb = (wm * 128 + frow) * 64 + fpos;
  const int b_fb = SLICE + ((EPI == EPI_SWIGLU ? wn * 64 : wn * 128) + frow) * 64 + fpos;
  int st_rd = 0;                      // byte offset of the stage the next fragment read takes
  int ra = a_fb, rb = b_fb;           // the same, added to the lane's fragment offsets

  f32x4 acc[8][8];
#define MOEP_ZERO_ACC()                                                                         \
  _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                 \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                               \
      _Pragma("unroll") for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
  bf16x8 fa[2][8], fb[2][8];
  // B tile j of a wavefront: SwiGLU: gate tiles 0 .. 3 and up tiles 4 .. 7 (128 rows further) of the same
  // 64 columns; otherwise eight consecutive 16-row tiles.
#define MOEP_RB(slot, j)                                                                        \
  fb[slot][j] = *(const bf16x8*)(lds + rb + (EPI == EPI_SWIGLU ? ((j) >> 2) * 8192 + ((j) & 3) * 1024 : (j) * 1024));
#define MOEP_RA(slot, i) fa[slot][i] = *(const bf16x8*)(lds + ra + (i) * 1024);
  // (B fragments visited back and forth, so that only one operand changes from one MFMA to the next: 0.6 % faster)
#define MOEP_MFMA(slot)                                                                         \
  _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                 \
    _Pragma("unroll") for (int jj = 0; jj < 8; ++jj) {                                          \
      const int j = (i & 1) ? 7 - jj : jj;                                                      \
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0); }
  // Source order = wanted issue order (a direct load writes LDS, so the compiler keeps it ordered with
  // the fragment reads around it): two fragment reads, one direct load, eight times over, spread over
  // the first 48 of the step's 64 MFMAs by the scheduling groups below.
#define MOEP_READS_LOADS(slot)                                                                  \
  MOEP_RB(slot, 0) MOEP_RB(slot, 1) MOEP_LOAD1(0) MOEP_RB(slot, 2) MOEP_RB(slot, 3) MOEP_LOAD1(1) \
  MOEP_RB(slot, 4) MOEP_RB(slot, 5) MOEP_LOAD1(2) MOEP_RB(slot, 6) MOEP_RB(slot, 7) MOEP_LOAD1(3) \
  MOEP_RA(slot, 0) MOEP_RA(slot, 1) MOEP_LOAD1(4) MOEP_RA(slot, 2) MOEP_RA(slot, 3) MOEP_LOAD1(5) \
  MOEP_RA(slot, 4) MOEP_RA(slot, 5) MOEP_LOAD1(6) MOEP_RA(slot, 6) MOEP_RA(slot, 7) MOEP_LOAD1(7)
#define MOEP_READS(slot)                                                                        \
  MOEP_RB(slot, 0) MOEP_RB(slot, 1) MOEP_RB(slot, 2) MOEP_RB(slot, 3)                           \
  MOEP_RB(slot, 4) MOEP_RB(slot, 5) MOEP_RB(slot, 6) MOEP_RB(slot, 7)                           \
  MOEP_RA(slot, 0) MOEP_RA(slot, 1) MOEP_RA(slot, 2) MOEP_RA(slot, 3)                           \
  MOEP_RA(slot, 4) MOEP_RA(slot, 5) MOEP_RA(slot, 6) MOEP_RA(slot, 7)
  // Two MFMAs, a fragment read, two MFMAs, a fragment read, two MFMAs, a direct load: never more than one
  // memory instruction between two MFMAs (1 % faster than 3 + read + 3 + read + load).
#define MOEP_SCHED(LOADS)                                                                       \
  _Pragma("unroll") for (int q_ = 0; q_ < 8; ++q_) {                                            \
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                          \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                          \
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                          \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                          \
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                          \
    if (LOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                               \
  }
  // s_waitcnt immediates: vmcnt in bits 3:0 and 15:14, lgkmcnt in bits 11:8 (0 here), expcnt 6:4 left at 7.
  // Loads complete in issue order, so "at most 8 outstanding" means that everything but the slice issued in
  // this step has landed, in particular the two slices whose fragments are read before the next barrier
  // (stores of an epilogue only add to the count).
  constexpr int VM_MAIN = 8;
  constexpr int W_MAIN = 0x0070 | (VM_MAIN & 15) | ((VM_MAIN >> 4) << 14);
  // One step: multiply the slice whose fragments are in `slot`; meanwhile fetch the slice NS - 1 ahead and
  // read the next slice's fragments into the other slot.  The barrier at the end of every second step tells
  // every wavefront that the next two slices have landed for all of them and that all of them have read
  // the fragments of the two stages that the next two steps' loads overwrite.
#define MOEP_STEP(slot, BAR)                                                                    \
  {                                                                                             \
    MOEP_READS_LOADS((slot) ^ 1)                                                                \
    MOEP_MFMA(slot)                                                                             \
    MOEP_SCHED(true)                                                                            \
    MOEP_ADVANCE_LOADER()                                                                       \
    st_rd = st_rd + STAGE == LDS_BYTES ? 0 : st_rd + STAGE;                                     \
    ra = a_fb + st_rd; rb = b_fb + st_rd;                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                          \
    if (BAR) {                                                                                  \
      __builtin_amdgcn_s_waitcnt(W_MAIN);                                                       \
      __builtin_amdgcn_s_barrier();                                                             \
    }                                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                          \
  }

  // ---- prologue: the first NS - 1 slices of this workgroup's stream -----------------------------------
#pragma unroll 1
  for (int n = 0; n < NS - 1; ++n) {
    MOEP_LOAD1(0) MOEP_LOAD1(1) MOEP_LOAD1(2) MOEP_LOAD1(3) MOEP_LOAD1(4) MOEP_LOAD1(5) MOEP_LOAD1(6) MOEP_LOAD1(7)
    MOEP_ADVANCE_LOADER()
    MOEP_NEXT_LOAD_TILE()
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  MOEP_READS(0)
  st_rd = STAGE;
  ra = a_fb + st_rd; rb = b_fb + st_rd;
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): stage 0 is overwritten by the second step's loads, and
  __builtin_amdgcn_s_barrier();         // no barrier separates it from these reads otherwise
  __builtin_amdgcn_sched_barrier(0);

  uint32_t L_mm = blockIdx.x;
  int tm, tn, e_mm;
  decode(L_mm, tm, tn, e_mm);
  for (;;) {
    MOEP_ZERO_ACC()
    // The loader is NS - 1 slices ahead and changes tile between two runs of steps, never inside one.  K / 32
    // and NS - 1 are even, so every run is a whole number of step pairs.
    for (int left = nsl; left > 0;) {
      const int run = min(left, nsl - s_ld);
#pragma unroll 1
      for (int s_mm = 0; s_mm < run; s_mm += 2) {
        MOEP_STEP(0, false)
        MOEP_STEP(1, true)
      }
      left -= run;
      MOEP_NEXT_LOAD_TILE()
    }

    // ---- epilogue of tile (tm, tn) ------------------------------------------------------------------
    // Register v of lane l of accumulator tile (i, j) holds output row 16 i + (l % 16) of the wavefront's
    // 128 rows and fragment row f = 4 (l / 16) + v of weight tile j; with the row permutation of the weight
    // blocks, tiles 2 P and 2 P + 1 together give the lane the 8 consecutive columns 32 P + 8 (l / 16) .. + 7.
    // The lane id is recomputed here, in a form the compiler cannot move: anything derived from a value that
    // lives across the K loop is hoisted above it and held (or spilled) there, and the loop has no register to spare.
    int lane_e;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_e));
    const int q8 = 8 * (lane_e >> 4);
    int64_t row0 = (int64_t)tm * 256, row_end = p.M;
    if (GROUPED) {
      row0 = p.tile_row0[tm];
      row_end = p.seg_end[p.tile_expert[tm]];
    }
    char* const c_base = (char*)p.C + (GROUPED ? (int64_t)0 : (int64_t)e_mm * p.c_expert_bytes);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int prow = wm * 128 + i * 16 + (lane_e & 15);          // row inside the tile
      const int64_t r = row0 + prow;
      if (r >= row_end) continue;
      if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int P = 0; P < 2; ++P) {
        const int n = tn * 128 + wn * 64 + 32 * P + q8;
        if (n < p.N) {
          bf16x2 o[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            f32x2 h;
#pragma unroll
            for (int d = 0; d < 2; ++d) {
              const int b = 2 * P + (c >> 1), v = 2 * (c & 1) + d;
              const float g = acc[i][b][v], u = acc[i][4 + b][v];
              h[d] = g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
            }
            o[c] = __builtin_convertvector(h, bf16x2);
          }
          // packed A operand with K = N: slice n / 32, chunk (l / 16) of row prow
          char* dst = c_base + ((size_t)tm * (p.N >> 5) + (n >> 5)) * SLICE + prow * 64 +
                      (((lane_e >> 4) ^ ((prow >> 2) & 3)) << 4);
          *(u32x4*)dst = __builtin_bit_cast(u32x4, o);
        }
        }
      } else {
        int64_t dest = -1;                                       // EPI_ROWSCALE_F32: >= 0: this row is a token's only slot
        if (EPI == EPI_ROWSCALE_F32 && p.row_dest) dest = p.row_dest[r];
#pragma unroll
        for (int P = 0; P < 4; ++P) {
          const int n = tn * 256 + wn * 128 + 32 * P + q8;
          if (n >= p.N) continue;
          if (EPI == EPI_STORE || (EPI == EPI_ROWSCALE_F32 && dest >= 0)) {
            bf16x2 o[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const f32x2 h = {acc[i][2 * P + (c >> 1)][2 * (c & 1)], acc[i][2 * P + (c >> 1)][2 * (c & 1) + 1]};
              o[c] = __builtin_convertvector(h, bf16x2);
            }
            uint16_t* const row = EPI == EPI_STORE ? (uint16_t*)c_base + r * p.ldc : p.direct_out + dest * p.ldc;
            *(u32x4*)(row + n) = __builtin_bit_cast(u32x4, o);
          } else {                                               // EPI_ROWSCALE_F32
            const float sc = p.row_scale[r];
            float* dst = (float*)c_base + r * p.ldc + n;
            *(f32x4*)dst = sc * acc[i][2 * P];
            *(f32x4*)(dst + 4) = sc * acc[i][2 * P + 1];
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    L_mm += G;
    if (L_mm >= nblk) break;   // (the loads still in flight are re-reads; the wavefront ends when they are back)
    decode(L_mm, tm, tn, e_mm);
  }
  __builtin_amdgcn_s_waitcnt(0x0070);   // the re-reads still in flight target this workgroup's LDS
#undef MOEP_LOAD1
#undef MOEP_ADVANCE_LOADER
#undef MOEP_NEXT_LOAD_TILE
#undef MOEP_ZERO_ACC
#undef MOEP_RB
#undef MOEP_RA
#undef MOEP_MFMA
#undef MOEP_READS_LOADS
#undef MOEP_READS
#undef MOEP_SCHED
#undef MOEP_STEP
}

// Per-device launch state, filled on a device's first launch under a mutex (first calls from several host
// threads are safe): the compute-unit count, and whether each instantiation's dynamic LDS limit has been raised.
constexpr int kMaxDevices = 64;
struct DeviceState {
  int compute_units = 0;
  bool attr_set[3][2] = {};
};
std::mutex g_dev_mu;
DeviceState g_dev[kMaxDevices];

template <int EPI, bool GROUPED>
int launch(const KArgs& k, hipStream_t s) {
  int dev = 0, cus = 0;
  MOEP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MOEP_EUNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices - 1);
  {
    std::lock_guard<std::mutex> lk(g_dev_mu);
    DeviceState& d = g_dev[dev];
    if (!d.compute_units) {
      int v = 0;
      MOEP_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
      d.compute_units = v > 0 ? v : 256;
    }
    if (!d.attr_set[EPI][GROUPED]) {   // raising the dynamic LDS limit is per function and device, once
      MOEP_HIP(hipFuncSetAttribute((const void*)gemm_packed_kernel<EPI, GROUPED>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
      d.attr_set[EPI][GROUPED] = true;
    }
    cus = d.compute_units;
  }
  const int64_t nblk = (int64_t)k.m_tiles * k.n_tiles * k.experts;
  int grid = cus & ~7;                        // one persistent workgroup per compute unit, a multiple of 8
  if (grid < 8) grid = 8;
  if (nblk < grid) grid = (int)nblk;          // a single round: any size
  hipLaunchKernelGGL((gemm_packed_kernel<EPI, GROUPED>), dim3(grid), dim3(THREADS), LDS_BYTES, s, k);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

int launch_pack(PackArgs p, int64_t tiles, int K, int experts, hipStream_t s, const char* name) {
  if (K <= 0 || K % 64) return fail(MOEP_EUNSUPPORTED, "%s: K=%d must be a positive multiple of 64", name, K);
  if (tiles <= 0 || experts <= 0) return MOEP_OK;
  if (((uintptr_t)p.W0 | (uintptr_t)p.W1 | (uintptr_t)p.dst) & 15)
    return fail(MOEP_EUNSUPPORTED, "%s: operands must be 16-byte aligned", name);
  if (tiles >= ((int64_t)1 << 31) || K / 64 > 65535 || experts > 65535) return fail(MOEP_EUNSUPPORTED, "%s: too large", name);
  p.nsl = K / 32;
  Timed t(name, s);
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)tiles, K / 64, experts), dim3(256), 0, s, p);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace

size_t packed_a_bytes(int64_t rows, int K) {
  return (size_t)ceil_div(rows, 256) * 256 * (size_t)K * 2;
}

size_t packed_b_bytes(int N, int K, bool gate_up_pair) {
  return (size_t)ceil_div(N, gate_up_pair ? 128 : 256) * 256 * (size_t)K * 2;
}

int launch_pack_a_bf16(const void* X, int64_t ld, int64_t rows, int K, void* dst, hipStream_t s, const char* name) {
  if (ld % 8) return fail(MOEP_EUNSUPPORTED, "%s: leading dimension must be a multiple of 8", name);
  PackArgs p = {};
  p.W0 = (const u32x4*)X; p.dst = (u32x4*)dst; p.ld_chunks = ld / 8; p.rows = rows; p.mode = 0;
  return launch_pack(p, ceil_div(rows, 256), K, 1, s, name);
}

int launch_pack_a_gathered_bf16(const void* X, int64_t ld, const int32_t* rows_of, const int32_t* tile_expert,
                                const int32_t* tile_row0, const int32_t* seg_end, const int32_t* tiles_in_use,
                                int64_t max_tiles, int K, void* dst, hipStream_t s, const char* name) {
  if (ld % 8) return fail(MOEP_EUNSUPPORTED, "%s: leading dimension must be a multiple of 8", name);
  PackArgs p = {};
  p.W0 = (const u32x4*)X; p.dst = (u32x4*)dst; p.ld_chunks = ld / 8; p.mode = 3;
  p.rows_of = rows_of; p.tile_expert = tile_expert; p.tile_row0 = tile_row0; p.seg_end = seg_end;
  p.tiles_in_use = tiles_in_use;
  return launch_pack(p, max_tiles, K, 1, s, name);
}

int launch_pack_b_bf16(const void* W0, const void* W1, int N, int K, int experts, void* dst, hipStream_t s,
                       const char* name) {
  PackArgs p = {};
  p.W0 = (const u32x4*)W0; p.W1 = (const u32x4*)W1; p.dst = (u32x4*)dst;
  p.ld_chunks = K / 8; p.rows = N; p.mode = W1 ? 2 : 1;
  p.src_expert_chunks = (int64_t)N * (K / 8);
  p.dst_expert_chunks = (int64_t)(packed_b_bytes(N, K, W1 != nullptr) / 16);
  return launch_pack(p, ceil_div(N, W1 ? 128 : 256), K, experts, s, name);
}

int launch_gemm_bf16_packed(const PackedGemmArgs& g, hipStream_t s, const char* name) {
  if (g.K <= 0 || g.K % 64) return fail(MOEP_EUNSUPPORTED, "%s: K=%d must be a positive multiple of 64", name, g.K);
  if (g.N <= 0 || g.N % 32) return fail(MOEP_EUNSUPPORTED, "%s: N=%d must be a positive multiple of 32", name, g.N);
  if (g.M <= 0) return MOEP_OK;
  if (((uintptr_t)g.A | (uintptr_t)g.B | (uintptr_t)g.C) & 15)
    return fail(MOEP_EUNSUPPORTED, "%s: operands must be 16-byte aligned", name);
  if (g.epilogue != EPI_SWIGLU && (g.ldc % 8 || g.ldc < g.N)) return fail(MOEP_EINVAL, "%s: bad leading dimension", name);
  const bool grouped = g.tile_expert != nullptr;
  if (grouped && (!g.tile_row0 || !g.seg_end || !g.tiles_in_use || !g.tile_order || g.max_m_tiles <= 0))
    return fail(MOEP_EINVAL, "%s: incomplete tile map", name);
  if (g.epilogue == EPI_ROWSCALE_F32 && !g.row_scale) return fail(MOEP_EINVAL, "%s: row_scale is NULL", name);
  KArgs k = {};
  k.A = (const char*)g.A; k.B = (const char*)g.B; k.C = g.C;
  k.M = g.M; k.ldc = g.ldc; k.N = g.N; k.nsl = g.K / 32;
  k.tile_expert = g.tile_expert; k.tile_row0 = g.tile_row0; k.seg_end = g.seg_end; k.tiles_in_use = g.tiles_in_use;
  k.b_expert_bytes = (int64_t)packed_b_bytes(g.N, g.K, g.epilogue == EPI_SWIGLU);
  k.row_scale = g.row_scale;
  if (g.experts < 1 || (grouped && g.experts != 1)) return fail(MOEP_EINVAL, "%s: bad batch count %d", name, g.experts);
  k.experts = g.experts; k.a_expert_bytes = g.a_expert_bytes; k.c_expert_bytes = g.c_expert_bytes;
  if (g.row_dest && (g.epilogue != EPI_ROWSCALE_F32 || !g.direct_out || ((uintptr_t)g.direct_out & 15)))
    return fail(MOEP_EINVAL, "%s: row_dest needs the row-scaled epilogue and a 16-byte aligned direct_out", name);
  k.row_dest = g.row_dest; k.direct_out = (uint16_t*)g.direct_out;
  k.tile_order = grouped ? g.tile_order : nullptr;
  if ((g.a_expert_bytes | g.c_expert_bytes) & 15) return fail(MOEP_EUNSUPPORTED, "%s: per-expert strides must be multiples of 16 bytes", name);
  const int64_t m_tiles = grouped ? g.max_m_tiles : ceil_div(g.M, 256);
  const int64_t n_tiles = ceil_div(g.N, g.epilogue == EPI_SWIGLU ? 128 : 256);
  if (m_tiles * n_tiles * g.experts >= ((int64_t)1 << 31)) return fail(MOEP_EUNSUPPORTED, "%s: too many tiles", name);
  k.m_tiles = (int)m_tiles; k.n_tiles = (int)n_tiles;
  Timed t(name, s);
  if (grouped) {
    switch (g.epilogue) {
      case EPI_STORE: return launch<EPI_STORE, true>(k, s);
      case EPI_SWIGLU: return launch<EPI_SWIGLU, true>(k, s);
      case EPI_ROWSCALE_F32: return launch<EPI_ROWSCALE_F32, true>(k, s);
    }
  } else {
    switch (g.epilogue) {
      case EPI_STORE: return launch<EPI_STORE, false>(k, s);
      case EPI_SWIGLU: return launch<EPI_SWIGLU, false>(k, s);
    }
  }
  return fail(MOEP_EINVAL, "%s: unsupported epilogue %d", name, g.epilogue);
}

}  // namespace moep
