// Grouped SwiGLU FFN on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// One kernel template covers the five products of the layer:
//   GATEUP  G = X Wg^T, U = X Wu^T, A = silu(G) U      (A, B both K-contiguous)
//   DOWN    Y = A Wd^T                                  (A, B both K-contiguous)
//           (DOWN_FOLD: also out[t] = res[t] + w[t] Y[p], the combine of a one-slot layer)
//   DA      dA = dY Wd  -> A, dG, dU                    (B stored [K][N])
//   DX      dX = dG Wg + dU Wu                          (B stored [K][N], two K phases)
//   DW      dW[e] = P_e^T Q_e over the rows of expert e (A, B both stored [K][M/N])
//
// Tiling: a 256x256 output tile per workgroup of eight wavefronts (4x2, 64x128
// each, as 4x8 v_mfma_f32_16x16x32_bf16 blocks = 128 accumulator registers per
// lane), K in steps of 64 through two LDS stages.  The 16x16x32 instruction is used
// because the part is power-limited under this load: with random operands and two
// wavefronts per SIMD it sustains about a quarter more than 32x32x16 (measured: 80 %
// against 55-65 % of the nominal rate in a register-only loop); one wavefront alone
// issues it at only 60 %, so two share each SIMD.  Operand tiles go from global memory
// straight into LDS (buffer loads with an LDS destination, 1 KB per wavefront
// instruction), one such load every third MFMA slot: no staging registers, no LDS
// store instructions, and no burst of memory instructions that would hold up a
// wavefront's MFMAs.  The tiles are unpadded and swizzled instead: the loads place
// each 16-byte piece where the fragment reads are free of bank conflicts.  Tiles whose
// memory layout has K contiguous are kept [row][k] in LDS; tiles whose memory layout
// has the row index contiguous are kept [k][row] and read with ds_read_b64_tr_b16,
// which hands each lane four consecutive k of one row -- so no operand is ever
// transposed in HBM or by scalar LDS traffic.
//
// Ragged rows: the row-tile list is derived on the device from seg_offsets, so
// no host synchronisation is needed.  One persistent workgroup per compute unit
// walks the tile list; each XCD (workgroup ids congruent modulo 8) takes a share
// balanced by cost, ordered so that neighbours share operand tiles in that XCD's L2.
// Wavefronts with no valid rows or columns in a ragged tile skip their MFMAs.  When the
// last round of a row-segmented product would fill at most half of the chip, its tiles
// are split along k over several XCDs and a small second kernel adds the fp32 partial
// tiles in a fixed order (ffn_split_reduce_kernel).
#include <type_traits>
#include <utility>

#include "common.h"
#include "ffn.h"
#include "profile.h"

namespace dynmo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kMfmaThreads = 512;              // eight wavefronts: two per SIMD
constexpr int kWaves = kMfmaThreads / 64;
constexpr int kPieces = 32 / kWaves;           // 1 KB pieces of an operand tile per wavefront
constexpr int kTileBytes = 256 * 64 * 2;       // one operand tile (256 rows x 64 k, bf16), unpadded
constexpr int kStageBytes = 2 * kTileBytes;    // A then B
constexpr int kEpPitch = 132;                  // floats per row of an epilogue LDS patch (128 + 4: rows 4 apart are 16 banks apart)
constexpr int kEpRows = 16;                    // rows a wavefront passes through its patch at a time
constexpr int kEpWaveBytes = kEpRows * kEpPitch * 4;
// The epilogue patches lie behind stage 0, which is free while they are in use: the next
// tile's first k tile is loaded into it meanwhile.
constexpr int kEpBase = kStageBytes;
constexpr int kLdsBytes = kEpBase + kWaves * kEpWaveBytes;  // >= the two stages
constexpr int kTableBytes = 64 * 8 * 4;        // the per-expert tile table, kept behind them
constexpr int kDumpBytes = kWaves * 256;       // where the four-byte loads of the L2 prefetch drop their data
constexpr int kLdsTotal = kLdsBytes + kTableBytes + kDumpBytes;
constexpr int kXcds = 8;
constexpr int kMaxPersistent = 256;          // persistent workgroups per launch (one per compute unit)
constexpr int kMinSplitKt = 16;              // a k chunk of a split tile is at least this many k tiles long
constexpr int kMaxSplitTiles = kMaxPersistent / 2;     // tiles of a last round that is worth splitting
constexpr size_t kPartialFloats = (size_t)BM * BN;     // one workgroup's fp32 partial tile
constexpr int kSplitHdrInts = 4 + 4 * kMaxSplitTiles;  // {split, patches, slots, tiles} + {m0, m_end, n0, -} per tile

static_assert(2 * kStageBytes <= kLdsBytes, "the two stages must fit in front of the tile table");
static_assert(kLdsTotal <= 160 * 1024, "LDS of one compute unit");
static_assert(kPieces * kWaves == 32, "a tile is 32 pieces of 1 KB");

// MODE_DOWN_FOLD is MODE_DOWN with the weighted combine of a one-slot layer in its stores;
// MODE_DX_FOLD is MODE_DX with the scatter back to token order (weight 1) in its stores
enum { MODE_GATEUP = 0, MODE_DOWN = 1, MODE_DA = 2, MODE_DX = 3, MODE_DW = 4, MODE_DOWN_FOLD = 5, MODE_DX_FOLD = 6 };

struct GemmParams {
  const int32_t* seg;
  int E;
  int M;  // rows of the output (MODE_DW only; the other modes take rows from seg)
  int N;  // columns of the output (for GATEUP: F, and a tile spans 128 of them twice)
  int K;  // contraction length per phase (MODE_DW: taken from seg)
  const bf16_t* A1;
  const bf16_t* A2;
  long lda;
  const bf16_t* B1;
  const bf16_t* B2;
  long ldb;
  long b_expert_stride;
  bf16_t* C0;
  bf16_t* C1;
  bf16_t* C2;
  long ldc;
  const bf16_t* G;
  const bf16_t* U;
  float* partial;     // kMaxPersistent fp32 partial tiles, then kSplitHdrInts ints (modes that may split k)
  const int32_t* gather;  // MODE_GATEUP: row p of operand A is row gather[p] / gather_div of A1, or nullptr
  int gather_div;
  // MODE_DOWN_FOLD / MODE_DX_FOLD (k = 1): row p also goes to row t = scatter[p] of out as
  // res[t] + scale[t] * value (res nullptr = 0; res may be out; scale nullptr = 1); C0 may then be nullptr
  const int32_t* scatter;
  const float* scale;
  const bf16_t* res;
  bf16_t* out;
};

// ---- global memory -> LDS ---------------------------------------------------------
// An operand tile is 256 "rows" x 64 k = 32 pieces of 1 KB.  One buffer load with an
// LDS destination moves a piece: lane l fetches 16 bytes from its own global offset and
// the hardware drops them at (LDS base of the piece) + 16 l.  A piece outside the valid
// rows / k range is given an offset beyond the buffer's record count, for which the
// hardware delivers zeros, so the loads are branch-free.  Every offset that is not masked
// this way lies inside the operand.  The buffer base already points at the tile's
// (row0, k0) element.
//
// LDS layouts (unpadded; the swizzles make the fragment reads below conflict-free):
//   [row][k]: 128 bytes per row; the 16-byte piece with k = 8 c .. 8 c + 7 of row r sits at
//             r * 128 + ((c ^ ((r >> 1) & 7)) << 4)
//   [k][row]: 512 bytes per k-row in eight 64-byte blocks of 32 rows; block b of k-row k
//             sits at k * 512 + (((b & 4) | ((b ^ k) & 3)) << 6), and its two 32-byte halves
//             (16 rows each) are swapped when bit 3 of k is set
constexpr uint32_t kOob = 0x80000000u;

// raw buffer descriptor (wave-uniform): base address, stride 0, record count in bytes
typedef uint32_t desc_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ desc_t make_desc(const bf16_t* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  desc_t d;
  d.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
  d.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
  d.z = __builtin_amdgcn_readfirstlane(bytes);
  d.w = 0x00020000u;
  return d;
}

// One piece: global -> LDS.  Written as assembly so that the compiler sees neither a
// load (it would count it against its own waits) nor an LDS write (it would make every
// transposed LDS read wait for all outstanding loads); the k loop waits for these loads
// itself, once per k tile.  The memory clobber keeps LDS reads from moving across it.
// The LDS destination is `lds_base` (wave-uniform, in a scalar register) + LDS_CONST.
template <int LDS_CONST>
__device__ __forceinline__ void load_to_lds(desc_t d, uint32_t lds_base, uint32_t global_offset) {
  asm volatile("s_add_i32 m0, %0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_base), "v"(global_offset), "s"(d), "n"(LDS_CONST)
               : "memory", "scc");
}

// A prefetch into L2: four bytes per lane (one lane per 128-byte line) through the same path
// as the real loads, so that it retires in order with them; the data is dropped in LDS.
__device__ __forceinline__ void touch_to_lds(desc_t d, uint32_t lds_offset, uint32_t global_offset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :
               : "s"(lds_offset), "v"(global_offset), "s"(d)
               : "memory");
}

// Waits of the k loop, written out because the loads above are invisible to the compiler.
__device__ __forceinline__ void wait_loads_and_lds() { __builtin_amdgcn_s_waitcnt(0x0070); }  // vmcnt(0) lgkmcnt(0)
// all loads but the youngest (the L2 prefetch issued after a k tile's pieces), and every LDS read
__device__ __forceinline__ void wait_pieces_and_lds() { __builtin_amdgcn_s_waitcnt(0x0071); }  // vmcnt(1) lgkmcnt(0)
template <int N>
__device__ __forceinline__ void wait_loads_but() {  // at most N loads still in flight
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
__device__ __forceinline__ void wg_barrier() { __builtin_amdgcn_s_barrier(); }

// The thread index behind a compiler barrier.  Offsets derived from it are recomputed where
// they are used (once per output tile) instead of being computed at kernel entry and kept
// in scratch memory across the k loop, whose own registers fill the whole file.
__device__ __forceinline__ int tid_now() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

// Per-lane global offsets of the pieces a wavefront moves: piece j of wavefront w is piece
// w * kPieces + j of the tile.  Row validity does not change along k, so it is folded into
// the offsets once per output tile; the k validity is applied per k tile (it only bites in
// a ragged last tile).
struct Pieces {
  uint32_t off[kPieces];  // byte offset from the tile's (row0, k0) element, or kOob
  int kpos[kPieces];      // k index of the lane's 16 bytes inside the 64-wide k tile
};

// [row][k] memory: piece q holds LDS rows 8 q .. 8 q + 7; lane l fills slot l % 8 of row
// 8 q + l / 8, which the swizzle assigns to k piece (l % 8) ^ ((row >> 1) & 7).
// `wrap` = 128 for the gate/up pairing (LDS rows 128..255 are rows 0..127 of a second matrix).
__device__ __forceinline__ Pieces pieces_rowk(uint32_t ld_bytes, int rows_left, int wrap) {
  Pieces ps;
  const int tid = tid_now();
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int j = 0; j < kPieces; ++j) {
    const int lrow = (wave * kPieces + j) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((lrow >> 1) & 7);
    const int row = lrow % wrap;
    ps.off[j] = row < rows_left ? (uint32_t)row * ld_bytes + c * 16 : kOob;
    ps.kpos[j] = c * 8;
  }
  return ps;
}

// [k][row] memory: piece q holds k-rows 2 q and 2 q + 1; lane l fills 16-byte slot l % 32 of
// k-row 2 q + l / 32, i.e. quarter (l % 4) of stored block (l % 32) / 4 (quarters 0, 1 and
// 2, 3 are the block's two halves).
__device__ __forceinline__ Pieces pieces_krow(uint32_t ld_bytes, int rows_left) {
  Pieces ps;
  const int tid = tid_now();
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int j = 0; j < kPieces; ++j) {
    const int k = (wave * kPieces + j) * 2 + (lane >> 5);
    const int slot = lane & 31, stored = slot >> 2;
    const int blk = (stored & 4) | ((stored ^ k) & 3);
    const int quarter = (slot & 3) ^ (((k >> 3) & 1) << 1);
    const int col = blk * 32 + quarter * 8;
    ps.off[j] = col < rows_left ? (uint32_t)k * ld_bytes + col * 2 : kOob;
    ps.kpos[j] = k;
  }
  return ps;
}

// [row][k] memory whose rows are fetched through an index: LDS row r is row
// rowmap[row0 + r] / rowdiv of the operand, so the offsets are taken from the operand's
// first row (the buffer base then points at (row 0, k0)).
__device__ __forceinline__ Pieces pieces_rowk_gather(uint32_t ld_bytes, int row0, int rows_left,
                                                     const int32_t* __restrict__ rowmap, int rowdiv) {
  Pieces ps;
  const int tid = tid_now();
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int j = 0; j < kPieces; ++j) {
    const int lrow = (wave * kPieces + j) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((lrow >> 1) & 7);
    ps.off[j] = kOob;
    if (lrow < rows_left) ps.off[j] = (uint32_t)(rowmap[row0 + lrow] / rowdiv) * ld_bytes + c * 16;
    ps.kpos[j] = c * 8;
  }
  return ps;
}

// ---- LDS -> MFMA operand fragments ---------------------------------------------
// Operand of v_mfma_f32_16x16x32_bf16: lane l holds, for row (l % 16) of the 16-row
// block, the eight k values (l / 16) * 8 .. + 7 of the 32-wide k step.
//
// Per-lane LDS addresses (of the stage being read) from which every fragment of a k tile is
// reached by a compile-time constant.  [row][k] tiles: one address per 32-wide k step (the
// swizzle mixes the k piece into the address; the 16-row block adds block * 2048).
// [k][row] tiles: one address per 16-row block (the swizzle mixes the block into the address;
// the k step adds step * 32 * 512).  `first16` is the wavefront's first 16-row block, its n-th
// block lies STRIDE blocks further on each time.
// The k loop moves the addresses from stage to stage in place (shift()).
template <bool TRANS, int BLOCKS>
struct FragAddr {
  static constexpr int kCount = TRANS ? BLOCKS : 2;
  uint32_t a[kCount];
  __device__ __forceinline__ void shift(uint32_t delta) {
#pragma unroll
    for (int i = 0; i < kCount; ++i) a[i] += delta;
  }
};

template <bool TRANS, int BLOCKS, int STRIDE>
__device__ __forceinline__ FragAddr<TRANS, BLOCKS> frag_addr(uint32_t stage, int first16) {
  FragAddr<TRANS, BLOCKS> fa;
  const int lane = tid_now() & 63;
  const int s = lane & 15, g = lane >> 4;
  if constexpr (!TRANS) {
#pragma unroll
    for (int h = 0; h < 2; ++h) fa.a[h] = stage + (uint32_t)((first16 * 16 + s) * 128 + (((h * 4 + g) ^ ((s >> 1) & 7)) << 4));
  } else {
    // ds_read_b64_tr_b16 works on groups of 16 lanes: lane s of a group points at four
    // consecutive rows (s % 4) * 4 .. + 3 of k-row (s / 4); afterwards lane i of the group
    // holds row i for those four k-rows.  Group g reads k-rows 8 g .. 8 g + 7 (two reads).
    const int k = g * 8 + (s >> 2);
#pragma unroll
    for (int n = 0; n < BLOCKS; ++n) {
      const int blk = (first16 + n * STRIDE) >> 1, half = (first16 + n * STRIDE) & 1;
      const int stored = (blk & 4) | ((blk ^ k) & 3);
      fa.a[n] = stage + (uint32_t)(k * 512 + stored * 64 + (((g & 1) ^ half) << 5) + (s & 3) * 8);
    }
  }
  return fa;
}

// A fragment in registers: one 16-byte LDS read for [row][k] tiles, two transposing 8-byte
// reads for [k][row] tiles.
template <bool TRANS>
struct Frag {
  bf16x8_t v;
  __device__ __forceinline__ bf16x8_t operand() const { return v; }
};
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <>
struct Frag<true> {
  u32x2_t lo, hi;
  __device__ __forceinline__ bf16x8_t operand() const {
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
  }
};
template <bool TRANS>
constexpr int kReadsPerFrag = TRANS ? 2 : 1;

// Reads the wavefront's IDX-th fragment, which lies ROW16 16-row blocks behind its first one, for
// the 32-wide k step H into `f`; TILE_OFF = the operand tile's offset inside a stage.  Written
// as assembly with the fragment as an in-out operand: the new value then takes the registers
// of the old one (left to itself the compiler gives every read of the unrolled k tile fresh
// registers, twice the fragments' share of the file, and spills loop invariants instead).
// The compiler therefore does not know these reads; wait_lds_but() below stands in for its waits.
template <bool TRANS, int IDX, int ROW16, int H, int TILE_OFF, int BLOCKS>
__device__ __forceinline__ void read_frag(Frag<TRANS>& f, const FragAddr<TRANS, BLOCKS>& fa) {
  if constexpr (!TRANS) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(f.v) : "v"(fa.a[H]), "n"(TILE_OFF + ROW16 * 2048) : "memory");
  } else {
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "+v"(f.lo) : "v"(fa.a[IDX]), "n"(TILE_OFF + H * 32 * 512) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "+v"(f.hi) : "v"(fa.a[IDX]), "n"(TILE_OFF + H * 32 * 512 + 4 * 512) : "memory");
  }
}

// Waits until at most N of this wavefront's LDS reads are outstanding (they complete in
// order).  The callers fence it with __builtin_amdgcn_sched_barrier(0) so that the MFMAs that
// need the data stay behind it.
template <int N>
__device__ __forceinline__ void wait_lds_but() {
  constexpr int n = N < 15 ? N : 15;
  __builtin_amdgcn_s_waitcnt(0xc07f | (n << 8));  // lgkmcnt(n), no wait on the other counters
}

// ---- tile schedule ---------------------------------------------------------------
struct Tile {
  int e;       // expert
  int m0;      // first output row (absolute row for the segmented modes)
  int m_end;   // end of valid rows
  int n0;      // first output column
  int k_begin, k_end;  // the expert's row range (the contraction range of MODE_DW)
};

// The tile list is never materialised.  All tiles of expert 0 come first, then
// expert 1, ...; inside an expert they go in the order of tile_in_expert() below, chosen
// so that the 32 consecutive tiles the workgroups of an XCD hold at a time share
// operand tiles in L2.  How the list is dealt to the XCDs depends on what a tile costs:
//   * row-segmented products: every tile has the same k range; each XCD takes one
//     contiguous eighth of the whole list, or, with several experts (whose tiles cost
//     what their ragged last row tiles make them cost), every eighth run of 32 tiles;
//   * products that contract over an expert's rows: a tile costs in proportion to
//     the expert's row count, so each XCD takes an eighth of EVERY expert's tiles
//     (whole experts per XCD would leave the most loaded one working alone).
struct TileTable {
  int nt;     // column tiles (same for all experts)
  int total;  // tiles in the list decode_tile() indexes: the whole list for the row-segmented
              // products, this XCD's list for the others
};

constexpr int kTableStride = 8;  // ints per expert in the LDS table
// Per expert e, at table[kTableStride*e ..]: first row, end row, row tiles, number of
// tiles of experts 0..e in the list, and what to add to a list position to get the tile
// index inside the expert.  Built by the first wavefront into LDS (kept there so that
// it costs no registers during the main loop); callers synchronise before reading it.
__device__ __forceinline__ TileTable make_tile_table(int* table, const int32_t* __restrict__ seg, int E, bool dw, int M,
                                                     int N, int tile_n, int xcd) {
  const int lane = threadIdx.x & 63;
  TileTable tb;
  tb.nt = (N + tile_n - 1) / tile_n;
  int begin = 0, end = 0;
  if (lane < E) {
    begin = seg[lane];
    end = seg[lane + 1];
  }
  const int mt = dw ? (lane < E ? (M + BM - 1) / BM : 0) : (end - begin + BM - 1) / BM;
  const int n = mt * tb.nt;
  auto scan = [&](int v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(v, d, 64);
      if (lane >= d) v += o;
    }
    return v;
  };
  int run_off = 0, run_len = n;
  if (dw) {
    run_off = (int)((long)n * xcd / kXcds);
    run_len = (int)((long)n * (xcd + 1) / kXcds) - run_off;
  }
  const int cum = scan(run_len);
  tb.total = __builtin_amdgcn_readlane(cum, 63);
  if (threadIdx.x < 64) {
    int* row = table + kTableStride * lane;
    row[0] = begin;
    row[1] = end;
    row[2] = mt;
    row[3] = cum;
    row[4] = run_off - (cum - run_len);  // add a list position to get the tile index inside the expert
  }
  return tb;
}

// Tile r of an expert with mt row tiles and nt column tiles -> (row tile, column tile): the order
// in which the list walks an expert's tiles.  32 consecutive tiles run side by side in one XCD
// and should need few distinct operand tiles, wherever in the expert the run starts (the
// experts' tile counts are not multiples of 32).
//   * Many row tiles (`tall`): column tiles in groups of kGroupN, a group walked row tile by row
//     tile -- a run is 4 row tiles x 8 column tiles, 12 operand tiles, except where it wraps
//     from a group's last row tiles to the next group's first (once in mt / 4 runs).
//   * Few row tiles: that wrap would be in every run (20 operand tiles).  The row tiles go in
//     chunks of about `rows` (nearly equal heights) and a chunk is walked column tile by column
//     tile, all of its row tiles before the next column tile: a run covers the h row tiles of
//     the chunk and about 32 / h column tiles, wherever it starts.
//   * Fewer than 8 column tiles: row tile by row tile over the whole width.
constexpr int kGroupN = 8;
__device__ __forceinline__ void tile_in_expert(int mt, int nt, int r, bool tall, int rows, int& mi, int& ni) {
  mt = max(1, mt);
  if (nt < kGroupN) {
    mi = r / nt;
    ni = r - mi * nt;
    return;
  }
  if (tall) {
    const int group = r / (mt * kGroupN);
    const int within = r - group * (mt * kGroupN);
    const int gn = min(kGroupN, nt - group * kGroupN);
    mi = within / gn;
    ni = group * kGroupN + within - mi * gn;
    return;
  }
  const int chunks = max(1, (mt + rows / 2 - 1) / rows);
  const int h = mt / chunks, taller = mt % chunks;  // the first `taller` chunks have h + 1 rows
  const int tall_tiles = taller * (h + 1) * nt;
  int row0, height;
  if (r < tall_tiles) {
    const int c = r / ((h + 1) * nt);
    r -= c * (h + 1) * nt;
    row0 = c * (h + 1);
    height = h + 1;
  } else {
    r -= tall_tiles;
    const int c = r / (h * nt);
    r -= c * h * nt;
    row0 = taller * (h + 1) + c * h;
    height = h;
  }
  ni = r / height;
  mi = row0 + r - ni * height;
}
// The first order from 13 row tiles on.  Below that, chunks of about 4 row tiles (runs of 4 x 8), or of
// about 8 (runs of 8 x 4) where operand tiles are small enough to survive in L2 from one run to the
// next, so that consecutive runs keep 8 tiles instead of 4:
//   * a short contraction (`short_k`: at most kShortK);
//   * a token-contracted product whose output has more row tiles than column tiles (dWg, dWu: F x H) --
//     its k range is an expert's rows -- which takes this order whatever its height (measured: 6 %
//     faster than 4 x 8 runs that move along F; dWd, H x F, gets the same from the first order).
constexpr int kTallFrom = 13;
constexpr int kShortK = 1024;
constexpr int kMinTouchKt = 16;  // L2 prefetch: only for k ranges of at least that many k tiles
__device__ __forceinline__ void tile_in_expert(bool dw, bool short_k, int mt, int nt, int r, int& mi, int& ni) {
  const bool long_rows = dw && mt >= nt;
  tile_in_expert(mt, nt, r, !long_rows && mt >= kTallFrom, long_rows || short_k ? 8 : 4, mi, ni);
}

// pos = position in the list
__device__ __forceinline__ Tile decode_tile(const int* table, const TileTable& tb, int pos, bool dw, bool short_k, int M, int tile_n) {
  const int lane = threadIdx.x & 63;
  const unsigned long long mask = __ballot(table[kTableStride * lane + 3] > pos);
  const int e = __builtin_ctzll(mask);
  const int* row = table + kTableStride * e;
  const int begin = row[0], end = row[1], mt = row[2];
  const int r = pos + row[4];  // tile index inside expert e
  int mi, ni;
  tile_in_expert(dw, short_k, mt, tb.nt, r, mi, ni);
  Tile t;
  t.e = e;
  t.m0 = dw ? mi * BM : begin + mi * BM;
  t.m_end = dw ? M : end;
  t.n0 = ni * tile_n;
  t.k_begin = begin;  // MODE_DW contracts over the expert's rows
  t.k_end = end;
  return t;
}

template <int... Is, typename F>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), fully unrolled
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// The logistic function for results that are rounded to bf16: the hardware reciprocal (1 ulp) instead of a
// correctly rounded division, which is ten instructions per element in epilogues that are bound by their
// vector arithmetic.
__device__ __forceinline__ float sigmoid_bf16(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float silu_mul(float g, float u) { return g * sigmoid_bf16(g) * u; }
// swiglu_bwd() of ffn.h with that reciprocal
__device__ __forceinline__ void swiglu_bwd_bf16(float dA, float g, float u, float* a, float* dg, float* du) {
  const float s = sigmoid_bf16(g);
  const float gs = g * s;
  *a = gs * u;
  *dg = dA * u * (s * (1.f + g * (1.f - s)));
  *du = dA * gs;
}

// WHOLE_K: the contraction length is a multiple of the k tile, so the [row][k] operands need no
// per-lane k mask (the [k][row] operands never do: their k range is the buffer's record count).
template <int MODE, bool WHOLE_K>
__global__ __launch_bounds__(kMfmaThreads, 1) void ffn_mfma_kernel(const GemmParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr bool A_TRANS = MODE == MODE_DW;
  constexpr bool IS_DX = MODE == MODE_DX || MODE == MODE_DX_FOLD;
  constexpr bool FOLDS = MODE == MODE_DOWN_FOLD || MODE == MODE_DX_FOLD;
  constexpr bool B_TRANS = MODE == MODE_DA || IS_DX || MODE == MODE_DW;
  constexpr int TILE_N = MODE == MODE_GATEUP ? 128 : BN;  // output columns per tile

  // Persistent workgroups: workgroup b belongs to XCD b % 8 (the hardware deals
  // workgroup ids round-robin over the XCDs) and is the (b / 8)-th of its XCD.  The
  // workgroups of an XCD walk that XCD's tile list in lock step, so neighbouring
  // tiles run at the same time in one L2.
  int* table = (int*)(smem + kLdsBytes);
  const int xcd = blockIdx.x % kXcds, slots = gridDim.x / kXcds;
  const TileTable tb = make_tile_table(table, p.seg, p.E, MODE == MODE_DW, p.M, p.N, TILE_N, xcd);
  __syncthreads();
  const int n_end = p.N;
  const bool short_k = MODE != MODE_DW && p.K <= kShortK;
  // The SIMD favours its older wavefront, which then reaches each k-tile barrier well
  // before the younger one; a higher priority for the younger wavefronts evens that
  // out (measured: a few percent).
  if (threadIdx.x >= kMfmaThreads / 2) __builtin_amdgcn_s_setprio(1);
  // Who runs what.  Products that contract over an expert's rows: the XCD's own list,
  // one tile per workgroup and round.  Row-segmented products: XCD x takes the x-th
  // contiguous eighth of the whole list (one expert) or every eighth run of 32 tiles
  // (several experts; below).  If the last round of the grid would leave at
  // least half of the XCDs idle (`patches` XCD-sized patches of tiles, 2 * patches <= 8),
  // those last tiles are taken out of the eighths and each patch is run by `split` XCDs
  // at once, every one on its own chunk of the k range: a patch keeps the operand
  // sharing of an ordinary round.  The chunks leave fp32 partial tiles in global memory,
  // which a second small kernel adds up in chunk order and converts.
  constexpr bool CAN_SPLIT = MODE == MODE_DOWN || MODE == MODE_DOWN_FOLD || IS_DX;
  const int slot = blockIdx.x / kXcds;
  int first = 0, mine = tb.total;  // this XCD's run of the list
  int split = 1, patches = 0, tail_tiles = 0;
  if (MODE != MODE_DW) {
    const int all = tb.total;
    if (CAN_SPLIT && p.partial != nullptr) {
      tail_tiles = all % (int)gridDim.x;
      patches = (tail_tiles + slots - 1) / slots;
      const int kts = (p.K + BK - 1) / BK * (IS_DX ? 2 : 1);
      if (tail_tiles > 0 && 2 * patches <= kXcds) split = max(1, min(kXcds / patches, kts / kMinSplitKt));
      if (split == 1) tail_tiles = 0;
    }
    const int per = (all - tail_tiles + kXcds - 1) / kXcds;
    first = min(xcd * per, all - tail_tiles);
    mine = min(per, all - tail_tiles - first);
  }
  // In round r the XCD's workgroups take its tiles r * slots .. + slots - 1, workgroup `slot` the one at
  // (slot + 5 r) mod slots of them.  The rotation changes nothing about which tiles run side by side; it
  // spreads the cheap ragged row tiles, which recur at a fixed place of that window when an expert has a
  // multiple of four row tiles (a multiple of eight places otherwise: hence a step that is not), over the
  // workgroups, whose tile counts are fixed.
  auto place = [&](int round) { return (slot + 5 * round) % slots; };
  // Row-segmented products over several experts: the runs of `slots` consecutive tiles go round robin to
  // the XCDs instead (run g to XCD g % 8).  A contiguous eighth holds whole experts, and an expert's tiles
  // cost what its ragged last row tile makes them cost: on a Mixtral-shaped layer the XCDs finished up to
  // 7 % apart.  Dealt round robin every XCD gets the same mix (that layer: gate/up -2 %, down -6 %, dA
  // -5 %).  A single expert keeps the eighths: there the XCDs that walk the same rows side by side share
  // them through the Infinity Cache (dense dA: 12 % slower round robin).
  const bool rr = MODE != MODE_DW && p.E > 1;
  const int main_tiles = rr ? tb.total - tail_tiles : mine;
  auto run_base = [&](int round) { return rr ? (round * kXcds + xcd) * slots : first + round * slots; };
  auto run_len = [&](int round) { return max(0, min(slots, (rr ? main_tiles : first + mine) - run_base(round))); };
  const int runs = (main_tiles + slots - 1) / slots;
  const int xcd_rounds = rr ? (runs > xcd ? (runs - xcd + kXcds - 1) / kXcds : 0) : (mine + slots - 1) / slots;
  const int my_rounds = xcd_rounds > 0 && place(xcd_rounds - 1) >= run_len(xcd_rounds - 1) ? xcd_rounds - 1 : xcd_rounds;
  const int tail_tile = (xcd / split) * slots + slot;  // index among the split tiles
  const bool has_part = split > 1 && tail_tile < tail_tiles;
  if (CAN_SPLIT && p.partial != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
    int32_t* hdr = (int32_t*)(p.partial + kMaxPersistent * kPartialFloats);
    hdr[0] = split;
    hdr[1] = patches;
    hdr[2] = slots;
    hdr[3] = tail_tiles;
  }
  const int wave_u = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // the gate/up pairing: LDS rows 128..255 of operand B (the upper four wavefronts' pieces) come from the second matrix
  const bool second_b = MODE == MODE_GATEUP && wave_u >= kWaves / 2;
  const bool gathered = MODE == MODE_GATEUP && p.gather != nullptr;
  const uint32_t lda_b = (uint32_t)p.lda * 2, ldb_b = (uint32_t)p.ldb * 2;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;  // LDS addresses are 32-bit offsets
  auto pieces_a = [&](const Tile& tt) {
    return A_TRANS   ? pieces_krow(lda_b, tt.m_end - tt.m0)
           : gathered ? pieces_rowk_gather(lda_b, tt.m0, tt.m_end - tt.m0, p.gather, p.gather_div)
                      : pieces_rowk(lda_b, tt.m_end - tt.m0, 256);
  };
  auto pieces_b = [&](const Tile& tt) {
    return B_TRANS ? pieces_krow(ldb_b, n_end - tt.n0) : pieces_rowk(ldb_b, n_end - tt.n0, MODE == MODE_GATEUP ? 128 : 256);
  };
  // operand descriptors of one k tile (wave-uniform), and how many k are left in it
  struct KTile {
    desc_t a, b;
    int k_left;
  };
  // The k range a workgroup covers of tile tt: all of it, or its chunk of a split tile.
  struct KRange {
    int k_begin, k_end, kt_per_phase, kt_lo, kt_hi;
  };
  auto krange = [&](const Tile& tt, bool parted_t) {
    KRange r;
    r.k_begin = MODE == MODE_DW ? tt.k_begin : 0;
    r.k_end = MODE == MODE_DW ? tt.k_end : p.K;
    r.kt_per_phase = (r.k_end - r.k_begin + BK - 1) / BK;
    const int n_kt = r.kt_per_phase * (IS_DX ? 2 : 1);
    const int chunk_t = parted_t ? xcd % split : 0;
    r.kt_lo = parted_t ? chunk_t * n_kt / split : 0;
    r.kt_hi = parted_t ? (chunk_t + 1) * n_kt / split : n_kt;
    return r;
  };
  // The k tiles of an output tile are loaded strictly one after the other, so their
  // descriptors come from an iterator that only adds strides (all of it scalar work: a
  // from-scratch address computation per k tile sat in front of the k loop's MFMAs).
  struct KIter {
    const bf16_t* a;   // (row0, k) elements of the next k tile's operand tiles
    const bf16_t* b;
    int k_left;        // valid k from there to the end of the k range (of this phase)
    int tiles_left;    // k tiles until this workgroup's share of the k range ends
    int to_switch;     // MODE_DX: k tiles until the second phase starts
    const bf16_t* a2;  // MODE_DX: where the second phase starts
    const bf16_t* b2;
  };
  auto uniform_ptr = [](const bf16_t* q) {
    const uint64_t v = (uint64_t)q;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const bf16_t*)(((uint64_t)hi << 32) | lo);
  };
  // positioned at k tile kt of tile tt (`second`: operand B of the gate/up pairing comes from the second matrix)
  auto kiter_at = [&](const Tile& tt, const KRange& r, int kt, bool second) {
    const int ph = IS_DX && kt >= r.kt_per_phase ? 1 : 0;
    const int k0 = r.k_begin + (kt - ph * r.kt_per_phase) * BK;
    auto addr_a = [&](int phase, int k) {
      const bf16_t* A = phase == 0 ? p.A1 : p.A2;
      return uniform_ptr(A_TRANS ? A + (long)k * p.lda + tt.m0 : A + (gathered ? 0 : (long)tt.m0 * p.lda) + k);
    };
    auto addr_b = [&](int phase, int k) {
      const bf16_t* B = ((phase == 1 || second) ? p.B2 : p.B1) + (MODE == MODE_DW ? 0 : (long)tt.e * p.b_expert_stride);
      return uniform_ptr(B_TRANS ? B + (long)k * p.ldb + tt.n0 : B + (long)tt.n0 * p.ldb + k);
    };
    KIter it;
    it.a = addr_a(ph, k0);
    it.b = addr_b(ph, k0);
    it.k_left = __builtin_amdgcn_readfirstlane(r.k_end - k0);
    it.tiles_left = __builtin_amdgcn_readfirstlane(r.kt_hi - kt);
    it.to_switch = IS_DX && ph == 0 ? __builtin_amdgcn_readfirstlane(r.kt_per_phase - kt) : 0x40000000;
    it.a2 = IS_DX ? addr_a(1, 0) : nullptr;
    it.b2 = IS_DX ? addr_b(1, 0) : nullptr;
    return it;
  };
  // the descriptors of the k tile the iterator stands at; moves it on to the next one
  auto knext = [&](KIter& it) {
    KTile q;
    q.k_left = it.tiles_left > 0 ? it.k_left : 0;
    // record counts: nothing past the k range is fetched (zeros land in LDS instead); a [k][row]
    // operand's k-rows are whole records, so its count is also the k mask of a ragged last tile
    const uint32_t k_rows = (uint32_t)max(0, min(q.k_left, BK));
    const uint32_t any = q.k_left > 0 ? 0x7ffffffeu : 0u;
    q.a = make_desc(it.a, A_TRANS ? k_rows * lda_b : any);
    q.b = make_desc(it.b, B_TRANS ? k_rows * ldb_b : any);
    it.a += A_TRANS ? (long)BK * p.lda : BK;
    it.b += B_TRANS ? (long)BK * p.ldb : BK;
    it.k_left -= BK;
    it.tiles_left -= 1;
    if (IS_DX) {
      it.to_switch -= 1;
      if (it.to_switch == 0) {
        it.a = it.a2;
        it.b = it.b2;
        it.k_left = p.K;
      }
    }
    return q;
  };
  // this wavefront's pieces of k tile q (pieces pa / pb) into the stage at LDS offset `stage`
  const uint32_t wave_pieces = wave_u * kPieces * 1024;  // this wavefront's pieces inside an operand tile
  auto dma_a = [&](const Pieces& pa, const KTile& q, uint32_t stage, auto J) {
    constexpr int j = decltype(J)::value;
    load_to_lds<j * 1024>(q.a, stage + wave_pieces, A_TRANS || WHOLE_K || pa.kpos[j] < q.k_left ? pa.off[j] : kOob);
  };
  auto dma_b = [&](const Pieces& pb, const KTile& q, uint32_t stage, auto J) {
    constexpr int j = decltype(J)::value;
    load_to_lds<kTileBytes + j * 1024>(q.b, stage + wave_pieces, B_TRANS || WHOLE_K || pb.kpos[j] < q.k_left ? pb.off[j] : kOob);
  };
  // L2 prefetch.  The workgroups of an XCD that run side by side share operand tiles (in a run
  // of 4 x 8 output tiles, 8 share each A tile and 4 each B tile) and ask for the same lines at
  // about the same time, so every one of them sees the full memory latency on every k tile.
  // Three k tiles ahead, each line is therefore asked for once, by one of the workgroups that
  // share it -- four bytes per 128-byte line, into a dump area; every wavefront issues one such
  // instruction per k tile (lanes without a line are masked), which keeps the wait counts
  // alike.  Purely a hint: nothing depends on the data.
  // Prefetched: the products whose operands are both [row][k] (gate/up and down: 9 to 12 % faster
  // when every expert has a multiple of four row tiles) and dX, both operands (Mixtral shape: 6 %
  // faster; only one of the two operands: 4 to 14 % slower than none).  Not prefetched: dA (+-2 %)
  // and the token-contracted products (2 to 3 % slower with it).
  constexpr bool TOUCHES = (!A_TRANS && !B_TRANS) || IS_DX;
  struct Touch {
    uint32_t off;  // this lane's line, as a byte offset from the tile's (row0, k0) element, or kOob
    bool second;   // gate/up pairing: this wavefront's lines are in the second matrix
  };
  // Who shares what is read off the tiles that really run side by side, not assumed: the experts'
  // tile counts are no multiples of 32, so a run starts anywhere in an expert's tile order and
  // may span two experts (a fixed partition by tile index left half of the B lines untouched in
  // such runs, and the prefetch gained nothing on a Mixtral-shaped layer with 3 to 9 row tiles per expert).  Lane j decodes the j-th tile of the
  // run this workgroup's tile belongs to (`base` = the run's first list position, `n_valid`
  // tiles, this workgroup's the `me`-th); tiles with the same expert and row tile share the A
  // tile, tiles with the same expert and column tile the B tile.
  auto touch_of = [&](const Tile& tt, int kts_of_tile, int base, int n_valid, int me) {
    if constexpr (!TOUCHES) return Touch{kOob, false};
    // nothing is touched when the k range (of a phase, for dX) is short (11 k tiles: 4 % slower with the prefetch than without)
    if (kts_of_tile < kMinTouchKt) return Touch{kOob, MODE == MODE_GATEUP && wave_u >= 6};
    const int tid = tid_now();
    const int lane = tid & 63, wave = tid >> 6;
    const int ni = tt.n0 / TILE_N, mi = (MODE == MODE_DW ? tt.m0 : tt.m0 - tt.k_begin) / BM;
    int e_j = -1, mi_j = 0, ni_j = 0;
    if (lane < n_valid) {
      const int pos = base + lane;
      int e = 0;
      for (int x = 0; x + 1 < p.E; ++x) e += table[kTableStride * x + 3] <= pos ? 1 : 0;
      const int* row = table + kTableStride * e;
      e_j = e;
      tile_in_expert(MODE == MODE_DW, short_k, row[2], tb.nt, pos + row[4], mi_j, ni_j);
    }
    const unsigned long long share_a = __ballot(e_j == tt.e && mi_j == mi);
    const unsigned long long share_b = __ballot(e_j == tt.e && ni_j == ni);
    const unsigned long long below = (1ull << me) - 1;
    const int cnt_a = max(1, __builtin_popcountll(share_a)), rank_a = __builtin_popcountll(share_a & below);
    const int cnt_b = max(1, __builtin_popcountll(share_b)), rank_b = __builtin_popcountll(share_b & below);
    Touch th;
    th.off = kOob;
    th.second = MODE == MODE_GATEUP && __builtin_amdgcn_readfirstlane(wave) >= 6;
    // The lines of an operand tile go round robin to its `cnt` sharers, this workgroup being the `rank`-th.
    // Wavefronts 0..3 cover the 256 lines of the A tile, 4..7 those of the B tile (gate/up: 4, 5 the gate
    // rows, 6, 7 the matching up rows).  (One contiguous block of lines per sharer instead measured the same,
    // +-1 %.)  A tile nobody else in the run uses is touched all the same, by its one user: left out, it runs
    // so much slower than its neighbours that a product of three rounds -- down on a Mixtral-shaped layer, where
    // ten of 576 tiles are in that position -- ends 20 % later.
    const int line = (wave & 3) * 64 + lane;
    if (wave < 4) {
      const int rows_left = tt.m_end - tt.m0;
      if (!A_TRANS) {
        if (line < rows_left && line % cnt_a == rank_a)
          th.off = (uint32_t)(gathered ? p.gather[tt.m0 + line] / p.gather_div : line) * lda_b;
      } else {
        // [k][row] tile: k-row line / 4, 64-row quarter line % 4 (128 bytes); the record count masks the k range
        if ((line & 3) * 64 < rows_left && line % cnt_a == rank_a) th.off = (uint32_t)(line >> 2) * lda_b + (line & 3) * 128;
      }
    } else {
      const int cols_left = n_end - tt.n0;
      if (!B_TRANS) {
        const int row = MODE == MODE_GATEUP ? line % 128 : line;
        if (row < cols_left && line % cnt_b == rank_b) th.off = (uint32_t)row * ldb_b;
      } else {
        if ((line & 3) * 64 < cols_left && line % cnt_b == rank_b) th.off = (uint32_t)(line >> 2) * ldb_b + (line & 3) * 128;
      }
    }
    return th;
  };
  const uint32_t lds_dump = lds0 + kLdsBytes + kTableBytes + wave_u * 256;
  auto touch = [&](const KTile& q, const Touch& th) {
    if constexpr (TOUCHES) touch_to_lds(wave_u >= 4 ? q.b : q.a, lds_dump, th.off);
  };
  // the k loop's wait for the pieces of the next k tile: the prefetch, if any, is the youngest load and may stay out
  auto wait_pieces = [&]() {
    if constexpr (TOUCHES) wait_pieces_and_lds();
    else wait_loads_and_lds();
  };
  const int n_rounds = my_rounds + (has_part ? 1 : 0);
  auto tile_at = [&](int round) {
    const bool parted_t = CAN_SPLIT && round == my_rounds;
    return decode_tile(table, tb, parted_t ? tb.total - tail_tiles + tail_tile : run_base(round) + place(round),
                       MODE == MODE_DW, short_k, p.M, TILE_N);
  };
  bool first_in_flight = false;  // the first k tile of the tile about to start is already on its way to stage 0
  for (int round = 0; round < n_rounds; ++round) {
  const bool parted = CAN_SPLIT && round == my_rounds;
  const int chunk = parted ? xcd % split : 0;
  const Tile t = tile_at(round);
  const KRange kr = krange(t, parted);
  const int kt_lo = kr.kt_lo, kt_hi = kr.kt_hi;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;  // 4 x 2 wavefronts, 64 x 128 outputs each

  // 16 x 16 blocks.  The wavefront's part is NOT a contiguous 64 rows: its row block i is the
  // tile's 16-row block 4 i + wm, so that in a ragged row tile (the valid rows are a prefix) every
  // wavefront keeps a share of the valid blocks -- ceil(valid blocks / 4) each -- instead of the
  // first one or two wavefronts of each column half doing all the work alone on their SIMDs.
  // Block (i, j) = rows 16 (4 i + wm) .., columns 16 j .. (+ 128 wn) of the tile.
  f32x4_t acc[4][8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

  // ---- main loop -------------------------------------------------------------
  // A hand-ordered software pipeline; __builtin_amdgcn_sched_barrier(0) after every
  // MFMA slot keeps the compiler from regrouping it.  Tile kt is in LDS stage kt % 2 and
  // the pieces of tile kt + 1 are in flight to the other stage on entry.  A k tile is two
  // 32-wide k steps of up to 32 MFMAs (the wavefront's 1..4 row blocks x 8 column blocks,
  // row-major).  Every fragment has one register set and is replaced as soon as its last MFMA
  // of the step has been issued (an A fragment after its row, a B fragment in the last row),
  // eight MFMA slots before it is needed again.  With four row blocks:
  //   step 0: MFMAs | fragments of step 1 as their registers fall free
  //   step 1, row 0: MFMAs
  //   wait for this wavefront's pieces of tile kt + 1 and for its LDS reads; barrier:
  //   now tile kt + 1 is complete and nobody reads the stage of tile kt any more
  //   step 1, rows 1..3: MFMAs | fragments of step 0 of tile kt + 1 as their registers fall
  //           free; one piece of tile kt + 2 every third MFMA into the stage of tile kt
  // so LDS latency is covered by MFMAs in flight (and by the SIMD's other wavefront), a
  // piece has a whole k tile to land, and the memory instructions are spread out: a burst
  // of them would hold up the wavefront's own MFMAs.  Past the last tile the loads are
  // masked (zeros, no memory access), which keeps the loop body free of branches.
  Frag<A_TRANS> fa[4];
  Frag<B_TRANS> fb[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) fa[i] = Frag<A_TRANS>{};
#pragma unroll
  for (int j = 0; j < 8; ++j) fb[j] = Frag<B_TRANS>{};
  constexpr int RA = kReadsPerFrag<A_TRANS>, RB = kReadsPerFrag<B_TRANS>;
  const Pieces pa = pieces_a(t), pb = pieces_b(t);
  // first 16-row block of this wavefront in each operand tile (gate/up: 64 gate rows, and the 64 matching up rows 128 further on)
  FragAddr<A_TRANS, 4> fra = frag_addr<A_TRANS, 4, 4>(lds0, wave_u >> 1);
  FragAddr<B_TRANS, 8> frb = frag_addr<B_TRANS, 8, 1>(lds0, MODE == MODE_GATEUP ? (wave_u & 1) * 4 : (wave_u & 1) * 8);
  KIter kit = kiter_at(t, kr, kt_lo, second_b);  // the k tiles to load, in order
  // A fragment of row block I / B fragment of column block J for k step H
  // (the stage read is the one fra / frb point into)
  auto read_a = [&](auto I, auto H) {
    read_frag<A_TRANS, decltype(I)::value, 4 * decltype(I)::value, decltype(H)::value, 0>(fa[decltype(I)::value], fra);
  };
  auto read_b = [&](auto J, auto H) {
    constexpr int j = decltype(J)::value;
    constexpr int n16 = MODE == MODE_GATEUP ? (j & 3) + (j >> 2) * 8 : j;
    read_frag<B_TRANS, j, n16, decltype(H)::value, kTileBytes>(fb[j], frb);
  };
  auto mfma = [&](auto I, auto J) {
    constexpr int i = decltype(I)::value, j = decltype(J)::value;
    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i].operand(), fb[j].operand(), acc[i][j], 0, 0, 0);
  };
  const std::integral_constant<int, 0> c0;
  const std::integral_constant<int, 1> c1;
  const std::integral_constant<int, 2> c2_;

  // What this workgroup prefetches is worked out with the first two k tiles on their way, where it costs
  // no time -- unless that takes a global load itself (the gather indices), which would wait for them.
  auto touch_now = [&]() {
    return parted ? touch_of(t, min(kt_hi - kt_lo, kr.kt_per_phase), tb.total - tail_tiles + (xcd / split) * slots, min(slots, tail_tiles - (xcd / split) * slots), slot)
                  : touch_of(t, min(kt_hi - kt_lo, kr.kt_per_phase), run_base(round), run_len(round), place(round));
  };
  Touch th{kOob, false};
  if (gathered) th = touch_now();
  {
    const KTile q0 = knext(kit);
    if (!first_in_flight) {
      static_for<kPieces>([&](auto J) { dma_a(pa, q0, lds0, J); });
      static_for<kPieces>([&](auto J) { dma_b(pb, q0, lds0, J); });
    }
  }
  {
    const KTile q1 = knext(kit);
    static_for<kPieces>([&](auto J) { dma_a(pa, q1, lds0 + kStageBytes, J); });
    static_for<kPieces>([&](auto J) { dma_b(pb, q1, lds0 + kStageBytes, J); });
  }
  if (!gathered) th = touch_now();
  KIter kit_touch = kiter_at(t, kr, kt_lo + 2, th.second);  // the k tiles to prefetch, in order
  if constexpr (TOUCHES) touch(knext(kit_touch), th);
  wait_loads_but<2 * kPieces + (TOUCHES ? 1 : 0)>();  // the first tile has landed
  wg_barrier();
  const int valid16 = min(16, (t.m_end - t.m0 + 15) / 16);  // valid 16-row blocks of the tile (a prefix)
  const bool cols_ok = (MODE == MODE_GATEUP ? t.n0 + (wave_u & 1) * 64 : t.n0 + (wave_u & 1) * 128) < n_end;
  // row blocks this wavefront has work in: blocks wm, wm + 4, .. below valid16
  const int my_rows = __builtin_amdgcn_readfirstlane(cols_ok && valid16 > (wave_u >> 1) ? (valid16 - (wave_u >> 1) + 3) / 4 : 0);
  // The k loop of a wavefront with ROWS row blocks of work (1..4; 4 = the full part).
  // Order of a step's fragment reads: A 0 .. ROWS-2 (each after its row), B 0 .. 7 (in the last
  // row, each after its last MFMA), A ROWS-1.  Reads complete in order, so what a MFMA has to
  // wait for is the number of reads issued after its youngest fragment.
  auto work = [&](auto ROWS_C) {
    constexpr int ROWS = decltype(ROWS_C)::value, LAST = ROWS - 1;
    const std::integral_constant<int, LAST> c_last;
    static_for<LAST>([&](auto I) { read_a(I, c0); });
    static_for<8>([&](auto J) { read_b(J, c0); });
    read_a(c_last, c0);
    // all MFMAs of one k step; WHAT = 0: first step of a k tile (fragments of step 1 follow as registers fall
    // free), 1: row 0 of step 1 only, 2: rows 1.. of step 1 with the refill, 3: rows 1.. of step 1 without
    auto mfmas = [&](auto WHAT_C, uint32_t freed, const KTile& q2, const KTile& q3) {
      constexpr int WHAT = decltype(WHAT_C)::value;
      constexpr int FIRST_SLOT = WHAT >= 2 ? 8 : 0, END_SLOT = WHAT == 1 ? 8 : 8 * ROWS;
      constexpr int REFILL_SLOTS = 8 * ROWS - 8;  // MFMA slots behind the barrier (none if ROWS == 1)
      static_for<END_SLOT - FIRST_SLOT>([&](auto M) {
        constexpr int m = decltype(M)::value + FIRST_SLOT, i = m >> 3, j = m & 7;
        if constexpr (WHAT <= 1 && i == 0) {
          // row 0: B 0..3, then B 4, 5, then B 6, 7 (B j is followed by B j+1 .. 7 and A LAST); with one row
          // block, A LAST is A 0 itself, the youngest read of all
          if constexpr (ROWS == 1 && j == 0) {
            wait_lds_but<0>();
            __builtin_amdgcn_sched_barrier(0);
          } else if constexpr (ROWS > 1 && (j == 0 || j == 4 || j == 6)) {
            wait_lds_but<(7 - (j == 0 ? 3 : j + 1)) * RB + RA>();
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        if constexpr (WHAT != 1 && ROWS > 1 && m == 8 * LAST) {  // A LAST of this step is followed by A 0 .. LAST-1 of the next
          wait_lds_but<LAST * RA>();
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (WHAT == 2) {
          // one piece of the refill every REFILL_SLOTS / 8 slots, the L2 prefetch in the last slot
          constexpr int every = REFILL_SLOTS / 8, s = m - 8;
          if constexpr (s % every == 0) {
            constexpr int piece = s / every;
            if constexpr (piece < kPieces) dma_a(pa, q2, freed, std::integral_constant<int, piece>{});
            else dma_b(pb, q2, freed, std::integral_constant<int, piece - kPieces>{});
          }
        }
        mfma(std::integral_constant<int, i>{}, std::integral_constant<int, j>{});
        if constexpr (WHAT == 0 || WHAT == 2) {
          constexpr auto H = std::integral_constant<int, WHAT == 0 ? 1 : 0>{};
          if constexpr (i == LAST) read_b(std::integral_constant<int, j>{}, H);
          if constexpr (j == 7) read_a(std::integral_constant<int, i>{}, H);
        }
        if constexpr (WHAT == 2 && m == 8 * ROWS - 1) touch(q3, th);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    const std::integral_constant<int, 2> c2;
    auto step0 = [&]() { mfmas(c0, 0u, KTile{}, KTile{}); };
    auto step1_row0_and_barrier = [&]() {
      mfmas(c1, 0u, KTile{}, KTile{});
      wait_pieces();
      wg_barrier();
      __builtin_amdgcn_sched_barrier(0);
    };
    // behind the barrier: fra / frb move on to the next tile's stage; its first fragments and the refill of the
    // stage just freed go between the remaining MFMAs of step 1 (all at once if there are none)
    auto step1_rest = [&](uint32_t to_next, uint32_t freed, const KTile& q2, const KTile& q3) {
      fra.shift(to_next);
      frb.shift(to_next);
      if constexpr (ROWS == 1) {
        static_for<kPieces>([&](auto J) { dma_a(pa, q2, freed, J); });
        static_for<kPieces>([&](auto J) { dma_b(pb, q2, freed, J); });
        touch(q3, th);
        static_for<8>([&](auto J) { read_b(J, c0); });
        read_a(c0, c0);
        __builtin_amdgcn_sched_barrier(0);
      } else {
        if constexpr (LAST > 0) read_a(c0, c0);
        mfmas(c2, freed, q2, q3);
      }
    };
    __builtin_amdgcn_sched_barrier(0);
    step0();
    step1_row0_and_barrier();
    for (int kt = kt_lo; kt + 1 < kt_hi; ++kt) {
      const int stage = (kt - kt_lo) & 1;
      const uint32_t to_next = stage ? 0u - (uint32_t)kStageBytes : (uint32_t)kStageBytes;
      const KTile q2 = knext(kit);
      KTile q3{};
      if constexpr (TOUCHES) q3 = knext(kit_touch);
      step1_rest(to_next, lds0 + stage * kStageBytes, q2, q3);
      step0();
      step1_row0_and_barrier();
    }
    if constexpr (ROWS > 1) mfmas(std::integral_constant<int, 3>{}, 0u, KTile{}, KTile{});
  };
  if (my_rows == 0) {
    // No valid rows or columns in this wavefront's part: it only keeps up the staging -- moves its
    // pieces and meets the barriers -- and leaves the SIMD and the LDS to the others.
    for (int kt = kt_lo; kt < kt_hi; ++kt) {
      wait_pieces();
      wg_barrier();
      const uint32_t freed = lds0 + ((kt - kt_lo) & 1) * kStageBytes;
      const KTile q2 = knext(kit);
      static_for<kPieces>([&](auto J) { dma_a(pa, q2, freed, J); });
      static_for<kPieces>([&](auto J) { dma_b(pb, q2, freed, J); });
      if constexpr (TOUCHES) touch(knext(kit_touch), th);
    }
  } else if (kt_lo < kt_hi) {  // (an expert without rows has nothing to contract: its tiles of MODE_DW stay zero)
    if (my_rows == 4) work(std::integral_constant<int, 4>{});
    else if (my_rows == 3) work(std::integral_constant<int, 3>{});
    else if (my_rows == 2) work(c2_);
    else work(c1);
  }
  // every piece (masked ones included) has landed and nobody reads the stages any more
  wait_loads_and_lds();
  wg_barrier();
  // The epilogue uses patches behind stage 0, so the first k tile of this workgroup's next
  // tile can be on its way into stage 0 while the results are stored.
  first_in_flight = round + 1 < n_rounds;
  if (first_in_flight) {
    const Tile tn = tile_at(round + 1);
    const KRange rn = krange(tn, CAN_SPLIT && round + 1 == my_rounds);
    const Pieces pan = pieces_a(tn), pbn = pieces_b(tn);
    KIter kn = kiter_at(tn, rn, rn.kt_lo, second_b);
    const KTile qn = knext(kn);
    static_for<kPieces>([&](auto J) { dma_a(pan, qn, lds0, J); });
    static_for<kPieces>([&](auto J) { dma_b(pbn, qn, lds0, J); });
  }

  // ---- epilogue.  Accumulator element r of block (i, j) is row 16 (4 i + wm) + (lane/16)*4 + r,
  // column 128 wn + 16 j + lane%16 of the tile.  Each wavefront passes sixteen rows at a
  // time (the eight blocks of row block i; only the row blocks it has work in) through its own
  // LDS patch (fp32, padded rows) so that global memory sees 16-byte accesses along rows.  The patch belongs to the wavefront alone and a
  // wavefront's LDS accesses complete in order, so neither reusing the patch nor reading it
  // back needs a workgroup barrier.
  // The lane and wavefront indices are taken afresh behind a compiler barrier: the addresses
  // below would otherwise be computed before the k loop and kept in scratch memory across it.
  {
  int lane_again = threadIdx.x & 63, wave_again = threadIdx.x >> 6;
  asm volatile("" : "+v"(lane_again), "+v"(wave_again));
  const int lane = lane_again, wave = wave_again;
  const int wm = wave >> 1, wn = wave & 1;
  float* ep = (float*)(smem + kEpBase + wave * kEpWaveBytes);
  const bf16_t* __restrict__ Gs = p.G;
  const bf16_t* __restrict__ Us = p.U;
  bf16_t* __restrict__ C0 = p.C0 + (MODE == MODE_DW ? (long)t.e * p.M * p.N : 0);
  bf16_t* __restrict__ C1 = p.C1;
  bf16_t* __restrict__ C2 = p.C2;
  // a k chunk of a split tile leaves fp32 sums, row-major in tile coordinates
  float* __restrict__ part = CAN_SPLIT ? p.partial + (size_t)blockIdx.x * kPartialFloats : nullptr;
  if (CAN_SPLIT && parted && chunk == 0 && threadIdx.x == 0) {
    int32_t* desc = (int32_t*)(p.partial + kMaxPersistent * kPartialFloats) + 4 + 4 * tail_tile;
    desc[0] = t.m0;
    desc[1] = t.m_end;
    desc[2] = t.n0;
  }
  constexpr int kPasses = kEpRows / 4;  // 64 lanes cover 4 rows x 128 columns (gate/up: 8 rows x 64 + 64) per pass
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i >= my_rows) break;
    const int tile_row = (i * 4 + wm) * kEpRows;  // first of the sixteen rows, inside the tile
    const int band_row = t.m0 + tile_row;
    // folded combine / scatter: the rows' token indices, then (once their accumulators have
    // left the registers) weights and residual rows, are requested all at once, so that their
    // latencies overlap each other and the LDS pass (out may alias res: every element is
    // read and written by the same thread only)
    int token[kPasses];
    float weight[kPasses];
    u32x4 resid[kPasses];
    const bool fold = FOLDS && !parted;
    if (fold) {
#pragma unroll
      for (int s = 0; s < kPasses; ++s) {
        const int row = band_row + s * 4 + (lane >> 4);
        token[s] = row < t.m_end ? p.scatter[row] : p.scatter[t.m0];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) ep[((lane >> 4) * 4 + r) * kEpPitch + j * 16 + (lane & 15)] = acc[i][j][r];
    if (fold) {
      const int col = t.n0 + wn * 128 + (lane & 15) * 8;
#pragma unroll
      for (int s = 0; s < kPasses; ++s) {
        weight[s] = p.scale ? p.scale[token[s]] : 1.f;
        resid[s] = u32x4{0u, 0u, 0u, 0u};
        if (p.res && col < n_end) resid[s] = *(const u32x4*)(p.res + (long)token[s] * p.ldc + col);
      }
    }
    if (MODE == MODE_GATEUP) {
      // LDS row: 64 gate columns then the 64 matching up columns
#pragma unroll
      for (int s = 0; s < kEpRows / 8; ++s) {
        const int rl = s * 8 + (lane >> 3), c0 = (lane & 7) * 8;
        const int row = band_row + rl, col = t.n0 + wn * 64 + c0;
        float g[8], u[8], a_[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          g[q] = ep[rl * kEpPitch + c0 + q];
          u[q] = ep[rl * kEpPitch + 64 + c0 + q];
          a_[q] = silu_mul(g[q], u[q]);
        }
        if (row < t.m_end && col < n_end) {
          const long o = (long)row * p.ldc + col;
          *(u32x4*)(C0 + o) = pack16<bf16_t>(g);
          *(u32x4*)(C1 + o) = pack16<bf16_t>(u);
          *(u32x4*)(C2 + o) = pack16<bf16_t>(a_);
        }
      }
    } else {
#pragma unroll
      for (int s = 0; s < kPasses; ++s) {
        const int rl = s * 4 + (lane >> 4), c0 = (lane & 15) * 8;
        const int row = band_row + rl, col = t.n0 + wn * 128 + c0;
        const bool ok = row < t.m_end && col < n_end;
        const long o = (long)row * p.ldc + col;
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = ep[rl * kEpPitch + c0 + q];
        if (CAN_SPLIT && parted) {
          float* dst = part + (tile_row + rl) * BN + wn * 128 + c0;
          *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
          *(float4*)(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
        } else if (MODE == MODE_DA) {
          if (ok) {
            float g[8], u[8], a_[8], dg[8], du[8];
            unpack16<bf16_t>(*(const u32x4*)(Gs + o), g);
            unpack16<bf16_t>(*(const u32x4*)(Us + o), u);
#pragma unroll
            for (int q = 0; q < 8; ++q) swiglu_bwd_bf16(v[q], g[q], u[q], &a_[q], &dg[q], &du[q]);
            *(u32x4*)(C0 + o) = pack16<bf16_t>(dg);
            *(u32x4*)(C1 + o) = pack16<bf16_t>(du);
            *(u32x4*)(C2 + o) = pack16<bf16_t>(a_);
          }
        } else if (ok) {
          if (!FOLDS || C0) *(u32x4*)(C0 + o) = pack16<bf16_t>(v);
          if (FOLDS) {
            float r[8];
            unpack16<bf16_t>(resid[s], r);
#pragma unroll
            for (int q = 0; q < 8; ++q) r[q] += weight[s] * v[q];
            *(u32x4*)(p.out + (long)token[s] * p.ldc + col) = pack16<bf16_t>(r);
          }
        }
      }
    }
  }
  }
  __syncthreads();  // the LDS patches overlap stage 1, which the next tile's second k tile goes to
  }  // tile loop
}

// Second pass of a product whose last round was split along k: adds the chunks'
// partial tiles in chunk order, converts and stores.  One workgroup per 16 rows of a tile
// (a whole tile per workgroup leaves most compute units idle when few tiles were split);
// the grid covers the most tiles a split can have, and workgroups beyond what the first
// pass recorded in the header, or wholly below a ragged tile's last row, return at once.
constexpr int kReduceRows = 16;                      // rows of a tile per workgroup
constexpr int kReduceParts = BM / kReduceRows;       // workgroups per tile
constexpr int kReduceIters = kReduceRows / 4;        // 256 threads cover 4 rows x 256 columns per step

__global__ __launch_bounds__(256) void ffn_split_reduce_kernel(const float* __restrict__ partial, bf16_t* __restrict__ C,
                                                               long ldc, int N, const int32_t* __restrict__ scatter,
                                                               const float* __restrict__ scale, const bf16_t* res,
                                                               bf16_t* out) {
  const int32_t* hdr = (const int32_t*)(partial + kMaxPersistent * kPartialFloats);
  const int split = hdr[0], slots = hdr[2], tiles = hdr[3];
  const int u = blockIdx.x / kReduceParts, part = blockIdx.x % kReduceParts;
  if (split <= 1 || u >= tiles) return;
  const int32_t* desc = hdr + 4 + 4 * u;
  const int m0 = desc[0], m_end = desc[1], n0 = desc[2];
  if (m0 + part * kReduceRows >= m_end) return;
  // chunk c of split tile u was run by workgroup (u % slots) of XCD (u / slots) * split + c
  const float* src = partial + (size_t)((u % slots) * kXcds + (u / slots) * split) * kPartialFloats;
  const int col = (threadIdx.x & 63) * 4;
  const bool cols_ok = n0 + col < N;
  // folded combine: token index and weight of each of this thread's rows, requested at once
  int token[kReduceIters];
  float weight[kReduceIters];
  if (scatter) {
#pragma unroll
    for (int it = 0; it < kReduceIters; ++it) {
      const int row = m0 + part * kReduceRows + it * 4 + (threadIdx.x >> 6);
      token[it] = scatter[row < m_end ? row : m0];
    }
#pragma unroll
    for (int it = 0; it < kReduceIters; ++it) weight[it] = scale ? scale[token[it]] : 1.f;
  }
#pragma unroll
  for (int it = 0; it < kReduceIters; ++it) {
    const int rl = part * kReduceRows + it * 4 + (threadIdx.x >> 6);
    const int row = m0 + rl;
    const bool ok = row < m_end && cols_ok;
    if (!ok) continue;
    // all chunks' loads are issued before the first add; the sum runs in chunk order
    float4 v[kXcds];
#pragma unroll
    for (int c = 0; c < kXcds; ++c)
      if (c < split) v[c] = *(const float4*)(src + (size_t)c * kPartialFloats + rl * BN + col);
    uint2 q = make_uint2(0u, 0u);
    if (scatter && res) q = *(const uint2*)(res + (long)token[it] * ldc + n0 + col);
    float4 sum = v[0];
#pragma unroll
    for (int c = 1; c < kXcds; ++c)
      if (c < split) {
        sum.x += v[c].x;
        sum.y += v[c].y;
        sum.z += v[c].z;
        sum.w += v[c].w;
      }
    uint2 o;
    if (C) {
      o.x = pack_bf16x2(sum.x, sum.y);
      o.y = pack_bf16x2(sum.z, sum.w);
      *(uint2*)(C + (long)row * ldc + n0 + col) = o;
    }
    if (scatter) {  // the combine of a one-slot layer, as in the first pass's own stores
      const float w = weight[it];
      o.x = pack_bf16x2(__uint_as_float(q.x << 16) + w * sum.x, __uint_as_float(q.x & 0xffff0000u) + w * sum.y);
      o.y = pack_bf16x2(__uint_as_float(q.y << 16) + w * sum.z, __uint_as_float(q.y & 0xffff0000u) + w * sum.w);
      *(uint2*)(out + (long)token[it] * ldc + n0 + col) = o;
    }
  }
}

// Scratch of the products that may split k: the partial tiles, then the header.
size_t ffn_mfma_scratch_bytes() { return kMaxPersistent * kPartialFloats * 4 + kSplitHdrInts * sizeof(int32_t); }

// Workgroups are persistent: one per compute unit (the LDS and register use allow
// no more), capped by the number of tiles the shapes can produce.
constexpr int kMaxDevices = 64;

static int current_device() {
  int dev = 0;
  return hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices ? dev : 0;
}

static int persistent_blocks(int max_tiles) {
  static int cus_of[kMaxDevices] = {};  // per device, filled on first use
  int& cus = cus_of[current_device()];
  if (cus == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, current_device()) != hipSuccess || n <= 0) n = 256;
    cus = n / kXcds * kXcds;
    if (cus < kXcds) cus = kXcds;
    if (cus > kMaxPersistent) cus = kMaxPersistent;
  }
  const int want = (max_tiles + kXcds - 1) / kXcds * kXcds;
  return want < cus ? want : cus;
}

template <int MODE, bool WHOLE_K>
static int32_t launch_mfma_as(const GemmParams& p, int max_tiles, KernelId id, hipStream_t st) {
  static bool attr_set[kMaxDevices] = {};  // the LDS size is a per-device function attribute
  bool& done = attr_set[current_device()];
  if (!done) {
    DYNMO_HIP_TRY(hipFuncSetAttribute((const void*)ffn_mfma_kernel<MODE, WHOLE_K>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal));
    done = true;
  }
  if (max_tiles <= 0) return DYNMO_OK;
  // a product that may split k always brings every compute unit: few tiles is when it splits
  const bool may_split = (MODE == MODE_DOWN || MODE == MODE_DOWN_FOLD || MODE == MODE_DX || MODE == MODE_DX_FOLD) && p.partial != nullptr;
  const int blocks = persistent_blocks(may_split ? kMaxPersistent : max_tiles);
  ProfScope prof(id, st);
  ffn_mfma_kernel<MODE, WHOLE_K><<<dim3(blocks), dim3(kMfmaThreads), kLdsTotal, st>>>(p);
  DYNMO_LAUNCH_CHECK();
  if (may_split) {
    ffn_split_reduce_kernel<<<dim3(kReduceParts * kMaxSplitTiles), dim3(256), 0, st>>>(p.partial, p.C0, p.ldc, p.N, p.scatter,
                                                                            p.scale, p.res, p.out);
    DYNMO_LAUNCH_CHECK();
  }
  return DYNMO_OK;
}

template <int MODE>
static int32_t launch_mfma(const GemmParams& p, int max_tiles, KernelId id, hipStream_t st) {
  // MODE_DW contracts over an expert's rows, which both of its operands hold as [k][row] records
  if constexpr (MODE != MODE_DW) {
    if (p.K % BK == 0) return launch_mfma_as<MODE, true>(p, max_tiles, id, st);
  }
  return launch_mfma_as<MODE, false>(p, max_tiles, id, st);
}

bool ffn_mfma_supported(const dynmo_desc* d) {
  return d->dtype == DYNMO_BF16 && d->H % 8 == 0 && d->F % 8 == 0 &&
         (int64_t)max_m_tiles(d, BM) * ((d->F + 127) / 128) < (1 << 30);
}

int32_t ffn_fwd_mfma(const dynmo_desc* d, const void* x_p, const int32_t* gather, const int32_t* seg, const void* Wg,
                     const void* Wu, const void* Wd, void* y_p, void* G, void* U, void* A, void* scratch,
                     const FoldedCombine* fc, hipStream_t st) {
  const int mt = max_m_tiles(d, BM);
  const long FH = (long)d->F * d->H;
  GemmParams p = {};
  p.seg = seg;
  p.E = d->E;
  // G, U, A = gate/up projections
  p.N = d->F;
  p.K = d->H;
  p.A1 = (const bf16_t*)x_p;
  p.gather = gather;
  p.gather_div = d->k;
  p.lda = d->H;
  p.B1 = (const bf16_t*)Wg;
  p.B2 = (const bf16_t*)Wu;
  p.ldb = d->H;
  p.b_expert_stride = FH;
  p.C0 = (bf16_t*)G;
  p.C1 = (bf16_t*)U;
  p.C2 = (bf16_t*)A;
  p.ldc = d->F;
  int32_t rc = launch_mfma<MODE_GATEUP>(p, mt * ((d->F + 127) / 128), K_FFN_GATEUP, st);
  if (rc) return rc;
  // Y = A Wd^T
  GemmParams q = {};
  q.partial = (float*)scratch;
  q.seg = seg;
  q.E = d->E;
  q.N = d->H;
  q.K = d->F;
  q.A1 = (const bf16_t*)A;
  q.lda = d->F;
  q.B1 = (const bf16_t*)Wd;
  q.ldb = d->F;
  q.b_expert_stride = FH;
  q.C0 = (bf16_t*)y_p;
  q.ldc = d->H;
  if (fc) {
    q.scatter = fc->scatter;
    q.scale = fc->scale;
    q.res = (const bf16_t*)fc->res;
    q.out = (bf16_t*)fc->out;
    return launch_mfma<MODE_DOWN_FOLD>(q, mt * ((d->H + BN - 1) / BN), K_FFN_DOWN, st);
  }
  return launch_mfma<MODE_DOWN>(q, mt * ((d->H + BN - 1) / BN), K_FFN_DOWN, st);
}

int32_t ffn_bwd_mfma(const dynmo_desc* d, const void* dy_p, const void* x_p, const void* G, const void* U,
                     const int32_t* seg, const void* Wg, const void* Wu, const void* Wd, void* dx_p, void* dWg,
                     void* dWu, void* dWd, void* dG, void* dU, void* A, void* scratch, const FoldedCombine* fc,
                     hipStream_t st) {
  const int mt = max_m_tiles(d, BM);
  const long FH = (long)d->F * d->H;
  const int tH = (d->H + BN - 1) / BN, tF = (d->F + BN - 1) / BN;
  int32_t rc;
  {  // dA = dY Wd, epilogue -> A, dG, dU
    GemmParams p = {};
    p.seg = seg;
    p.E = d->E;
    p.N = d->F;
    p.K = d->H;
    p.A1 = (const bf16_t*)dy_p;
    p.lda = d->H;
    p.B1 = (const bf16_t*)Wd;  // [H][F]: k = h rows, n = f contiguous
    p.ldb = d->F;
    p.b_expert_stride = FH;
    p.C0 = (bf16_t*)dG;
    p.C1 = (bf16_t*)dU;
    p.C2 = (bf16_t*)A;
    p.ldc = d->F;
    p.G = (const bf16_t*)G;
    p.U = (const bf16_t*)U;
    if ((rc = launch_mfma<MODE_DA>(p, mt * tF, K_FFN_DA, st))) return rc;
  }
  // weight gradients: contraction over the rows of each expert
  auto dw = [&](const void* P, int M, const void* Q, int N, void* out, KernelId id) -> int32_t {
    GemmParams p = {};
    p.seg = seg;
    p.E = d->E;
    p.M = M;
    p.N = N;
    p.A1 = (const bf16_t*)P;
    p.lda = M;
    p.B1 = (const bf16_t*)Q;
    p.ldb = N;
    p.C0 = (bf16_t*)out;
    p.ldc = N;
    return launch_mfma<MODE_DW>(p, d->E * ((M + BM - 1) / BM) * ((N + BN - 1) / BN), id, st);
  };
  // Order: the three weight gradients first, dX last, so that the pass that follows the
  // call (the scatter of dx_p back to token order) finds dx_p still in the last-level cache.
  if ((rc = dw(dy_p, d->H, A, d->F, dWd, K_FFN_DWD))) return rc;
  if ((rc = dw(dG, d->F, x_p, d->H, dWg, K_FFN_DWG))) return rc;
  if ((rc = dw(dU, d->F, x_p, d->H, dWu, K_FFN_DWU))) return rc;
  {  // dX = dG Wg + dU Wu
    GemmParams p = {};
    p.partial = (float*)scratch;
    p.seg = seg;
    p.E = d->E;
    p.N = d->H;
    p.K = d->F;
    p.A1 = (const bf16_t*)dG;
    p.A2 = (const bf16_t*)dU;
    p.lda = d->F;
    p.B1 = (const bf16_t*)Wg;  // [F][H]: k = f rows, n = h contiguous
    p.B2 = (const bf16_t*)Wu;
    p.ldb = d->H;
    p.b_expert_stride = FH;
    p.C0 = (bf16_t*)dx_p;
    p.ldc = d->H;
    if (fc) {
      p.scatter = fc->scatter;
      p.scale = fc->scale;
      p.res = (const bf16_t*)fc->res;
      p.out = (bf16_t*)fc->out;
      return launch_mfma<MODE_DX_FOLD>(p, mt * tH, K_FFN_DX, st);
    }
    return launch_mfma<MODE_DX>(p, mt * tH, K_FFN_DX, st);
  }
}

}  // namespace dynmo
