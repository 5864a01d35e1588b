// Linear-layer contractions (forward, input gradient, weight gradient) for gfx950.
//
// bf16 path: persistent MFMA kernels.  gemm_bf16_kernel serves every form: a workgroup of 8
// waves (256x256 tile, 128x64 per wave) or 4 waves (128x128 tile, 64x64 per wave) walks
// output tiles; gemm_bf16_kc4w_kernel (described at its definition) takes the whole 256x256
// tiles of the form with both operands K-contiguous.  In both,
// the grid is sized to the module's CU quota.  Each output element is produced by exactly
// one wave that accumulates k in ascending order with v_mfma_f32_32x32x16_bf16, so the
// bits of the result do not depend on the grid, the tile shape, the tile order or the CU.
//
// Data movement (gemm_bf16_kernel)
//   * HBM -> LDS directly (buffer_load ... lds): no register staging and no LDS write
//     instructions.  A wave instruction fills 1 KB of consecutive LDS; each lane chooses
//     which 16 bytes of the tile it requests, which realises the bank swizzle.  The
//     descriptor's bounds check returns zeros for rows past the end, so ragged tiles need
//     no branches.
//   * an operand whose contraction index is contiguous in HBM sits in LDS as rows of 32
//     k-values (64 bytes), 16-byte chunks XOR-swizzled by (row/4)%4, and is read with
//     ds_read_b128.  An operand whose contraction index is the strided one (the weight in
//     the forward pass, both operands of the weight gradient) sits in LDS as it is in HBM,
//     k-row by k-row with 64-byte chunks XOR-swizzled by k%4, and its fragments come out
//     with the transposing read ds_read_b64_tr_b16 (two per fragment).
//   * five LDS stages: while K-tile t is multiplied, t+1 is visible (its first fragments
//     are fetched before the barrier), t+2 is complete or landing and t+3 / t+4 are in
//     flight.  One barrier per K-tile; before it every wave waits (vmcnt) for its own
//     requests of tile t+2.  The stream of K-tiles runs across output tiles, so a new
//     output tile starts without a pipeline refill.
//   * fragments are double-buffered in registers: the reads for the next batch of MFMAs
//     are issued under the current batch, one fragment and one request per MFMA slot
//     (a scheduling barrier after every slot keeps the written order).
//   * accumulators are kept transposed (the weight-side fragment is MFMA's first operand),
//     so a lane owns four consecutive output columns per register group; the epilogue
//     (bias, residual, bf16 rounding) is staged through the free LDS stage into
//     row-contiguous 16-byte stores that fill whole 128-byte lines of the output.
//   * tiles are handed out so that the workgroups running on one XCD at the same time
//     form a 4 x 8 patch of the tile grid and share operand panels in that XCD's L2.
//
// fp32 path (and shapes the MFMA path does not cover): a plain LDS-tiled FMA kernel with
// arbitrary strides; ascending-k accumulation as well.
#include <stdlib.h>
#include <algorithm>
#include <mutex>
#include <type_traits>
#include "activations.h"
#include "kernels.h"
#include "tile_queue.h"

namespace {

#pragma clang diagnostic ignored "-Winline-asm"   // m0 is named as a clobber on purpose

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int BK = 32;            // k-values per LDS tile row (64 bytes)
constexpr unsigned kOob = 0xFFFFFFF0u;   // byte offset beyond any descriptor's range

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
constexpr int NS = 5;             // LDS stages
constexpr int AHEAD = 4;          // K-tiles between the load cursor and the compute cursor

// Requests one operand tile (ROWS x BK) from HBM straight into an LDS stage: every wave
// instruction moves 64 x 16 bytes to 1 KB of consecutive LDS; which 16 bytes of the tile a
// lane asks for is free, and that choice realises the swizzle.
//   K-contiguous operand: LDS rows of 64 bytes (32 k-values of one tile row), the four
//     16-byte chunks of row r stored at position chunk ^ (r/4)%4.
//   K-strided operand: LDS rows of ROWS*2 bytes (one k-row of the tile), the 64-byte chunks
//     of k-row k stored at position chunk ^ k%4; fragments come out with transposing reads.
// GU (K-strided operand only): the tile's columns are not consecutive columns of the matrix.
// The matrix is [gate | up] halves of gu_f columns each; 32-column group c of the tile is
// group c/2 of the gate half (c even) or of the up half (c odd), counted from column x0/2,
// so that a wave's two 32-column accumulator blocks hold a gate column and its up column
// in the same lane and register.
template <int ROWS, bool KC, int NWAVES, bool GU = false>
struct DmaLoader {
  static constexpr int NI = ROWS / 16 / NWAVES;     // wave instructions per wave and K-tile
  static constexpr int ROWB = ROWS * 2;             // strided: bytes per k-row
  static constexpr int RPI = 1024 / ROWB;           // strided: k-rows per wave instruction
  struct Tile { unsigned org; unsigned oobmask; };

  unsigned rel[NI];     // byte offset of instruction j's chunk relative to the tile origin at K-tile 0
  unsigned kstep;       // bytes between consecutive K-tiles
  int kofs;             // KC: first k of this lane's chunk
  int xofs[NI];         // strided: first tile column of this lane's chunk
  int wave_base;        // LDS byte offset of this wave's first instruction inside the operand area

  __device__ __forceinline__ void init(int64_t ld, int gu_f = 0) {
    static_assert(!(GU && KC), "the gate/up column map exists for the K-strided operand");
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    wave_base = w * NI * 1024;
    kofs = 0;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      if constexpr (KC) {
        const int r = 16 * (w * NI + j) + (lane >> 2), pos = lane & 3;
        const int ch = pos ^ ((r >> 2) & 3);
        kofs = ch * 8;
        rel[j] = (unsigned)(((int64_t)r * ld + ch * 8) * 2);
        xofs[j] = 0;
        kstep = BK * 2;
      } else {
        const int byte = 16 * lane;
        const int kr = (w * NI + j) * RPI + byte / ROWB, bp = byte % ROWB;
        const int c64 = (bp >> 6) ^ (kr & 3), p = (bp & 63) >> 4;
        xofs[j] = c64 * 32 + p * 8;
        int64_t gcol = xofs[j];
        if constexpr (GU) gcol = (c64 >> 1) * 32 + p * 8 + (int64_t)(c64 & 1) * gu_f;
        rel[j] = (unsigned)(((int64_t)kr * ld + gcol) * 2);
        kstep = (unsigned)(BK * ld * 2);
      }
    }
  }

  __device__ __forceinline__ Tile tile(int64_t ld, int x0, int X) const {
    Tile tl;
    tl.oobmask = 0;
    if constexpr (KC) tl.org = (unsigned)((int64_t)x0 * ld * 2);
    else if constexpr (GU) tl.org = (unsigned)x0;      // column x0/2 of each half, 2 bytes each; halves are whole tiles wide
    else {
      tl.org = (unsigned)(x0 * 2);
#pragma unroll
      for (int j = 0; j < NI; ++j) if (x0 + xofs[j] >= X) tl.oobmask |= 1u << j;
    }
    return tl;
  }

  // K-tile kt (absolute index) of tile tl -> operand area `dst` of a stage; zeros when
  // !valid, at or past kt_lim, or outside the matrix (rows past the end fall outside the
  // descriptor's range).  prep() holds what the NI requests of one K-tile share; issue_j()
  // makes request j, so that the caller can spread the requests over its instruction stream.
  struct Prep { bool oob; unsigned base; };
  __device__ __forceinline__ Prep prep(const Tile& tl, int kt, int K, int kt_lim, bool valid) const {
    Prep p;
    p.oob = !valid || kt >= kt_lim;
    if constexpr (KC) p.oob = p.oob || (kt * BK + kofs) >= K;
    p.base = tl.org + (unsigned)kt * kstep;
    return p;
  }
  __device__ __forceinline__ void issue_j(i32x4 rsrc, const Tile& tl, const Prep& p, int j, unsigned dst) const {
    const unsigned off = (p.oob || ((tl.oobmask >> j) & 1)) ? kOob : p.base + rel[j];
    // m0 = LDS byte address of lane 0's 16 bytes; lane l lands at m0 + 16*l.  Written as
    // assembly so that the compiler's wait-count pass does not see an LDS write and put a
    // full vmcnt(0) in front of every following LDS read; completion is waited for by
    // hand (wait_loads in the kernel).  The compiler itself never uses m0 in this file.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 : : "s"(dst + (unsigned)(wave_base + j * 1024)), "v"(off), "s"(rsrc) : "m0");
  }
  __device__ __forceinline__ void issue(i32x4 rsrc, const Tile& tl, int kt, int K, int kt_lim,
                                        bool valid, unsigned dst) const {
    const Prep p = prep(tl, kt, K, kt_lim, valid);
#pragma unroll
    for (int j = 0; j < NI; ++j) issue_j(rsrc, tl, p, j, dst);
  }
};

// Fragment addresses of one operand inside its stage area: NF blocks of 32 tile rows
// starting at row w0, for lane (lr = lane%32, hb = lane/32).
template <int ROWS, bool KC, int NF>
struct FragReader {
  int addr[KC ? 1 : NF];
  int ch[2];
  __device__ __forceinline__ void init(int w0) {
    const int lane = threadIdx.x & 63;
    if constexpr (KC) {
      const int lr = lane & 31, hb = lane >> 5, sw = (lr >> 2) & 3;
      addr[0] = (w0 + lr) * 64;
      ch[0] = ((hb ^ sw) & 3) << 4; ch[1] = (((2 + hb) ^ sw) & 3) << 4;
    } else {
      const int G = lane >> 4, i = lane & 15, hh = G >> 1, q = i >> 2, g = i & 3;
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const int c64 = (w0 + 32 * f) >> 5;
        addr[f] = (8 * hh + q) * (ROWS * 2) + ((c64 ^ q) << 6) + 32 * (G & 1) + 8 * g;
      }
      ch[0] = 0; ch[1] = 0;
    }
  }
  // fragment f for k-step ks (0/1) of the K-tile in operand area `base`
  __device__ __forceinline__ bf16x8 read(const lds_byte* base, int f, int ks) const {
    if constexpr (KC) {
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(base + addr[0] + f * 32 * 64 + ch[ks]);
    } else {
      const lds_byte* p = base + addr[f] + ks * 16 * (ROWS * 2);
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * (ROWS * 2)));
      typedef __attribute__((ext_vector_type(8))) short s16x8;
      const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// Position `tile` of the tile list -> (tile row, tile column).  The list is panel-major: panels
// of 8 tile columns, row-major inside a panel, so 32 consecutive entries form a 4 x 8 patch that
// shares operand panels in one XCD's L2.  Above that, tile rows are taken in super-blocks of
// `row_block` rows (all panels of a super-block before the next super-block), sized on the
// host so that the row operand of a super-block (row_block x 256 rows x K) stays in the
// last-level cache: it is then re-read from there, not from HBM, once per panel (measured on
// the 7B-shaped products: +3 % forward, +4 % input gradient; the board is power-bound and HBM
// reads cost energy).  Both kernels and both launches of a mixed plan use this one order.
__device__ __forceinline__ void tile_coords(int tile, int tiles_m, int tiles_n, int row_block, int* row, int* col) {
  const int per_sb = row_block * tiles_n;
  const int sb = tile / per_sb, rem = tile - sb * per_sb;
  const int rows_sb = min(row_block, tiles_m - sb * row_block);
  const int panel = rem / (rows_sb * 8);
  const int pw = min(8, tiles_n - panel * 8);
  const int in_panel = rem - panel * rows_sb * 8;
  *row = sb * row_block + in_panel / pw;
  *col = panel * 8 + in_panel % pw;
}

// Tile rows per super-block: the row operand of a super-block (rows x 256 x K bf16) is kept to
// about half of the 256 MB last-level cache, in whole 4-row patches.  Depends on K alone.
#ifndef MOSAIC_LLC_ROW_BYTES
#define MOSAIC_LLC_ROW_BYTES (128 << 20)
#endif
// Only products with many tile rows are cut (tiles_m counts 256-row tiles): with 64 rows or
// fewer, two rounds of 256 tiles already span every row and the plain order re-reads nothing
// that a cut would save (the weight-gradient form of the 7B shape, 16 tile rows, lost 3 % to a
// cut of 8 rows).
static inline int row_block_for(int64_t K, int64_t tiles_m) {
  if (tiles_m <= 64) return (int)((tiles_m + 3) / 4 * 4);
  int64_t rb = (int64_t)MOSAIC_LLC_ROW_BYTES / (512 * (K > 0 ? K : 1)) / 4 * 4;
  if (rb < 4) rb = 4;
  return (int)std::min<int64_t>(rb, (tiles_m + 3) / 4 * 4);
}

// One unit of work: an output tile, or (SPLITK) one K-piece of an output tile.
struct WorkItem {
  int m0, n0, kt0, kt_end, split, tl;      // tl: position of the item's coarse tile in this launch's range
  bool valid;
};

// SPLITK: the K range is cut into `ksplit` contiguous pieces of `ktiles_per` K-tiles; piece s
// of the launch's t-th tile is accumulated by its own workgroup and stored in fp32 to
// P[s][t][BM][BN]; a second kernel adds the pieces in ascending s.  Which tiles are cut and
// into how many pieces depends on the problem shape only.
//
// A workgroup streams the K-tiles of ALL its work items through one pipeline: a load
// cursor runs AHEAD K-tiles ahead of the compute cursor and crosses item boundaries, so
// the first tiles of the next item are already in LDS while the epilogue of the current one
// runs (the other wave on the SIMD keeps the matrix cores busy meanwhile).
//
// ACT (forward form only): the epilogue also writes an activation of the output to C2, so the
// pass that would read the output back is never launched.  ACT_GELU: C2 = gelu(C), same shape.
// ACT_SWIGLU: C is [gate | up] with gu_f columns each and C2[M, gu_f] = silu(gate) * up; the
// weight tile's columns are gathered so that a wave holds matching gate and up columns
// (DmaLoader GU).  The activation is taken of the bf16 value that is stored to C, as the
// separate pass would.
constexpr int ACT_NONE = 0, ACT_GELU = 1, ACT_SWIGLU = 2;
struct ActArgs {
  int act = ACT_NONE;
  bf16* C2 = nullptr;
  int64_t ldc2 = 0;
  uint32_t c2_bytes = 0;
  int gu_f = 0;
  int row_block = 1 << 20;   // tile rows per super-block of the tile order (set by the launcher)
};

template <int BM, int BN, int NWM, int NWN, bool A_KC, bool B_KC, bool SPLITK, int ACT = ACT_NONE>
__global__ __launch_bounds__(64 * NWM * NWN, 2) void gemm_bf16_kernel(
    const bf16* __restrict__ A, const bf16* __restrict__ B, bf16* __restrict__ C,
    const bf16* __restrict__ bias, const bf16* __restrict__ R, int M, int N, int K,
    int64_t lda, int64_t ldb, int64_t ldc, uint32_t a_bytes, uint32_t b_bytes, uint32_t c_bytes,
    int tiles_m, int tiles_n, int tile_begin, int tile_count, int sub, int ksplit, int ktiles_per,
    float* __restrict__ P, TileQueueArgs tq, ActArgs aa) {
  static_assert(ACT == ACT_NONE || (A_KC && !B_KC && !SPLITK), "activation epilogues exist for the forward form");
  constexpr int NT = 64 * NWM * NWN;
  constexpr int WM = BM / NWM, WN = BN / NWN;   // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int STAGE = (BM + BN) * 64;     // bytes per LDS stage
  extern __shared__ __align__(16) unsigned char smem[];

  const __amdgpu_buffer_rsrc_t ra = make_rsrc(A, a_bytes), rb = make_rsrc(B, b_bytes);
  const __amdgpu_buffer_rsrc_t rc = make_rsrc(C, c_bytes);
  const __amdgpu_buffer_rsrc_t rr = make_rsrc(R, R ? c_bytes : 0u);
  const __amdgpu_buffer_rsrc_t rbias = make_rsrc(bias, bias ? (uint32_t)N * 2u : 0u);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / NWN) * WM, wn = (wave % NWN) * WN;
  const int lr = lane & 31, hb = lane >> 5;
  lds_byte* const lds = (lds_byte*)smem;
  const int nk_all = (K + BK - 1) / BK;

  // Work order.  The output is cut into coarse tiles of (sub*BM) x (sub*BN), listed
  // panel-major: panels of 8 coarse-tile columns, row-major inside a panel, so 32 consecutive
  // entries form a 4 x 8 patch that shares operand panels.  This launch covers entries
  // [tile_begin, tile_begin + tile_count) of that list, each as sub*sub tiles of BM x BN
  // (sub = 2: the 128x128 kernel finishing the quarter tiles of the 256x256 tiles that did
  // not fill a whole round of the large kernel), once per split piece (split-major).  The
  // flat list of these items is handed out by the work queue (tile_queue.h): a chunk of as
  // many consecutive items as an XCD has resident workgroups goes to the list of one XCD, so
  // the workgroups of an XCD work on one patch at a time and reuse each other's panels in
  // that XCD's L2.
  const int per_split = tile_count * sub * sub;
  auto decode = [&](int item) -> WorkItem {
    WorkItem it;
    it.valid = item >= 0; it.m0 = 0; it.n0 = 0; it.kt0 = 0; it.kt_end = 0; it.split = 0; it.tl = 0;
    if (!it.valid) return it;
    it.split = item / per_split;
    const int fine = item - it.split * per_split;
    const int quad = fine % (sub * sub);
    it.tl = fine / (sub * sub);
    const int tile = tile_begin + it.tl;
    it.kt0 = it.split * ktiles_per;
    it.kt_end = SPLITK ? min(nk_all, it.kt0 + ktiles_per) : nk_all;
    int trow, tcol;
    tile_coords(tile, tiles_m, tiles_n, aa.row_block, &trow, &tcol);
    it.m0 = (trow * sub + quad / sub) * BM;
    it.n0 = (tcol * sub + quad % sub) * BN;
    return it;
  };

  // stage ring: K-tile number t of the stream lives in stage t % NS
  int si = 0;                                   // stage of the compute cursor's K-tile
  auto stg = [&](int ahead) { const int i = si + ahead; return (i >= NS ? i - NS : i) * STAGE; };

  // Drawing items.  Thread 0 talks to the queue and hands the item to the workgroup through
  // four bytes of the LDS stage that is free between two pipeline steps (the kernel's LDS is
  // otherwise full).  A draw is a round trip to memory.  The first item is drawn at the start;
  // the second when the load cursor asks for it (once per workgroup, in mid-pipeline: drawn
  // earlier, a workgroup that started first would take items from workgroups that have not
  // started yet); from then on one item is claimed at the start of every epilogue and resolved
  // at its end, so the round trip hides under the epilogue.  `drawn` holds an item drawn
  // ahead; `lq` the items the load cursor has entered and the compute cursor has not.
  TileQueueCursor qc;
  bool drained = false;
  int drawn = -1;
  bool have_drawn = false;
  // Claiming under the epilogue takes the item after the next, a whole tile before it is needed.
  // That is harmless while the list is long, but near its end a workgroup a few microseconds
  // ahead of the others would take two of the last items and leave another workgroup with
  // none (measured: a launch of exactly two rounds took three).  So an item comes with a
  // flag: `ahead_ok` says that the list it came from (this XCD's own) still held two rounds of
  // work after the claim; without it the next item is drawn when the load cursor asks for it.
  bool ahead_ok = false;
  auto publish = [&](int v) -> int {           // v is thread 0's (item | flag << 30); returns the item to every thread
    volatile int* mail = reinterpret_cast<volatile int*>(smem + stg(AHEAD));
    if (threadIdx.x == 0) *mail = v;
    __syncthreads();
    const int r = __builtin_amdgcn_readfirstlane(*mail);
    __syncthreads();                           // read by all before the stage is filled again
    if (r < 0) { drained = true; ahead_ok = false; return -1; }
    ahead_ok = (r >> 30) != 0;
    return r & 0x3fffffff;
  };
  int home_list = -1;                          // thread 0: the list of the XCD this workgroup runs on
  auto flagged = [&](int item, int left) -> int {
    if (item < 0) return -1;
    return item | ((qc.list == home_list && left >= 2 * tq.chunk) ? (1 << 30) : 0);
  };
  auto draw_sync = [&]() -> int {
    if (drained) return -1;
    if (tq.mode == TQ_ROUNDS) {                // static rounds: every thread computes its item
      const int r = tq_rounds_item(tq, ++qc.round);
      if (r < 0) drained = true;
      return r;
    }
    int v = -1;
    if (threadIdx.x == 0) { int left = 0; const int it = tq_resolve(tq, qc, tq_claim(tq, qc), &left); v = flagged(it, left); }
    return publish(v);
  };
  auto draw_first = [&]() -> int {
    if (tq.mode == TQ_ROUNDS) {
      const int r = tq_first_item(tq, qc);
      if (r < 0) drained = true;
      return r;
    }
    int v = -1;
    if (threadIdx.x == 0) {
      qc.init();
      home_list = qc.list;
      int left = 0;
      const int it = tq_resolve(tq, qc, tq_claim(tq, qc), &left);
      v = flagged(it, left);
    }
    const int r = publish(v);
    if (tq.mode != TQ_QUEUE) drained = true;   // one item per workgroup at most
    return r;
  };
  auto next_drawn = [&]() -> int {             // the next item in draw order
    if (have_drawn) { have_drawn = false; return drawn; }
    return draw_sync();
  };
  int lq0 = -1, lq1 = -1, lq2 = -1, lq3 = -1, lq4 = -1, lq5 = -1, lqn = 0;
  auto lq_push = [&](int v) {
    lq0 = lqn == 0 ? v : lq0; lq1 = lqn == 1 ? v : lq1; lq2 = lqn == 2 ? v : lq2;
    lq3 = lqn == 3 ? v : lq3; lq4 = lqn == 4 ? v : lq4; lq5 = lqn == 5 ? v : lq5;
    ++lqn;
  };
  auto lq_pop = [&]() -> int {
    const int v = lq0;
    lq0 = lq1; lq1 = lq2; lq2 = lq3; lq3 = lq4; lq4 = lq5; lq5 = -1;
    --lqn;
    return v;
  };

  WorkItem cur = decode(draw_first());
  if (!cur.valid) {                // a workgroup that started after the queue ran dry
    if (threadIdx.x == 0) tq_leave(tq);
    return;
  }

  typedef DmaLoader<BM, A_KC, NWM * NWN> LA;
  typedef DmaLoader<BN, B_KC, NWM * NWN, ACT == ACT_SWIGLU> LB;
  LA la; LB lb;
  la.init(lda); lb.init(ldb, aa.gu_f);
  constexpr int NLOADS = LA::NI + LB::NI;      // requests per lane and K-tile

  // load cursor: the next K-tile to request
  WorkItem lit = cur;
  int lkt = cur.kt0;
  typename LA::Tile lta = la.tile(lda, lit.m0, M);
  typename LB::Tile ltb = lb.tile(ldb, lit.n0, N);
  // buffer descriptors for the direct-to-LDS requests: base, no stride, size in bytes, raw 32-bit format
  auto desc = [](const void* p, uint32_t bytes) {
    i32x4 d;
    d.x = (int)(uint32_t)(uintptr_t)p; d.y = (int)((uint32_t)((uintptr_t)p >> 32) & 0xffffu);
    d.z = (int)bytes; d.w = 0x00020000;
    return d;
  };
  const i32x4 da = desc(A, a_bytes), db = desc(B, b_bytes);
  const unsigned lds0 = (unsigned)(uintptr_t)lds;      // LDS byte address of the dynamic segment
  auto issue = [&](int stage) {
    la.issue(da, lta, lkt, K, lit.kt_end, lit.valid, lds0 + (unsigned)stage);
    lb.issue(db, ltb, lkt, K, lit.kt_end, lit.valid, lds0 + (unsigned)(stage + BM * 64));
  };
  auto load_cursor_next_item = [&]() {
    const int item = next_drawn();
    if (item >= 0) lq_push(item);
    lit = decode(item);
    lkt = lit.kt0;
    lta = la.tile(lda, lit.m0, M);
    ltb = lb.tile(ldb, lit.n0, N);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // vmcnt(n) alone: lgkmcnt and expcnt fields at "no wait"
  auto wait_loads = [](auto n) { constexpr int N = decltype(n)::value; __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14)); };

  // prologue: the first AHEAD K-tiles of the stream are requested; the first two must have
  // landed before anyone reads
#pragma unroll
  for (int u = 0; u < AHEAD; ++u) {
    issue(u * STAGE);
    if (++lkt >= lit.kt_end && lit.valid) load_cursor_next_item();
  }
  wait_loads(std::integral_constant<int, 2 * NLOADS>{});
  __syncthreads();

  FragReader<BM, A_KC, TM> fra; FragReader<BN, B_KC, TN> frb;
  fra.init(wm); frb.init(wn);
  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  auto frags = [&](bf16x8* fa, bf16x8* fb, int stage, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = fra.read(lds + stage, i, ks);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = frb.read(lds + stage + BM * 64, j, ks);
  };
  frags(fa0, fb0, 0, 0);

  // Epilogue of one work item.  acc[i][j][4g+e] is output (row m0+wm+32i+lr, column
  // n0+wn+32j+8g+4hb+e): a lane holds 4-column pieces of 32 different rows, which would
  // reach memory as 8-byte fragments.  The accumulators therefore pass through a 4 KB
  // per-wave patch of the LDS stage that is free between two pipeline steps (XOR swizzled)
  // and leave row-contiguous.
  // Three variants, chosen by a uniform branch, so that each holds no request it does not
  // need.  The compiler's wait before a use of a loaded value counts every request of the
  // wave in issue order, stores included: a bias or residual request issued between two
  // stores makes the block that uses it wait until all earlier blocks' stores have been
  // acknowledged.
  //   EPI_PLAIN: no bias, no residual - stores only, nothing waits        (finish_rows)
  //   EPI_BIAS:  every bias value is requested before the first store     (finish_rows)
  //   EPI_RES:   residual (and bias, if any: a null bias reads zeros through its empty
  //              descriptor); the requests for block b+1 are issued before block b is stored,
  //              so a wait never covers the newest stores                 (finish_impl)
  // finish_impl moves one 32x32 block at a time in fp32 and adds bias and residual in
  // row-contiguous layout (fp32, one rounding); split-K pieces take the same path and leave
  // as fp32.
  constexpr int EPI_PLAIN = 0, EPI_BIAS = 1, EPI_RES = 2;
  auto finish_impl = [&](const WorkItem& it, int free_stage, auto mode_) {
    constexpr int MODE = decltype(mode_)::value;
    float* patch = reinterpret_cast<float*>(smem + free_stage) + wave * 1024;
    // The lane index passes through an empty asm so that the write-back offsets are computed
    // here, per tile, instead of being kept in registers across the K loop.
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int elr = ln & 31, ehb = ln >> 5;
    // Blocks leave in the order b = i * TN + j (row block i outer, column block j inner):
    // the two 64-byte halves of a 128-byte line of C belong to column blocks j, j+1 of the
    // same rows and are stored back to back, so they meet in the L2 before the line is
    // written out.
    // byte offset in C (and in the residual) of the 8 columns this lane writes back for row
    // half q of block b; rows past M fall outside the descriptor's range
    auto out_off = [&](int b, int q) -> unsigned {
      const int row = it.m0 + wm + 32 * (b / TN) + (ln >> 2) + 16 * q;
      const int col = it.n0 + wn + 32 * (b % TN) + 8 * (ln & 3);
      return (col < N) ? (unsigned)(((int64_t)row * ldc + col) * 2) : kOob;
    };
    // bias for the 8 columns this lane writes back in column block j (same for every row block)
    auto bias_req = [&](int j) -> u32x4 {
      const int col = it.n0 + wn + 32 * j + 8 * (ln & 3);
      return __builtin_amdgcn_raw_buffer_load_b128(rbias, col < N ? col * 2 : (int)kOob, 0, 0);
    };
    u32x4 rnext[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    u32x4 braw[MODE == EPI_BIAS ? TN : 1] = {};
    u32x4 bnext = {0u, 0u, 0u, 0u};
    if constexpr (MODE == EPI_BIAS) {
#pragma unroll
      for (int j = 0; j < TN; ++j) braw[j] = bias_req(j);
    }
    if constexpr (MODE == EPI_RES) {
      bnext = bias_req(0);
#pragma unroll
      for (int q = 0; q < 2; ++q) rnext[q] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)out_off(0, q), 0, 0);
    }
#pragma unroll
    for (int b = 0; b < TM * TN; ++b) {
      const int i = b / TN, j = b % TN;
      const int cb = it.n0 + wn + 32 * j;                 // first column of the block
      const int rb0 = it.m0 + wm + 32 * i;                // first row of the block
      float bvals[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) bvals[e] = 0.f;
      if constexpr (MODE != EPI_PLAIN) {
        const bf16x8 bv = __builtin_bit_cast(bf16x8, MODE == EPI_BIAS ? braw[MODE == EPI_BIAS ? j : 0] : bnext);
#pragma unroll
        for (int e = 0; e < 8; ++e) bvals[e] = (float)bv[e];
      }
      {
        // accumulator layout -> LDS: row lr, column group cg = 2g + hb (4 columns each)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int cg = (2 * g + ehb) ^ ((elr >> 1) & 7);
          float4 v = make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
          *reinterpret_cast<float4*>(patch + elr * 32 + cg * 4) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if constexpr (SPLITK) {
          float* Ps = P + ((int64_t)it.split * tile_count + it.tl) * (BM * BN);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int r = (ln >> 3) + 8 * q, cgl = ln & 7;
            const float4 v = *reinterpret_cast<const float4*>(patch + r * 32 + ((cgl ^ ((r >> 1) & 7)) * 4));
            const int row = rb0 + r, col = cb + 4 * cgl;
            if (row < M && col < N) *reinterpret_cast<float4*>(Ps + (row - it.m0) * BN + (col - it.n0)) = v;
          }
        } else {
          float4 v0[2], v1[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int r = (ln >> 2) + 16 * q, c8 = ln & 3;
            const int sx = (r >> 1) & 7;
            v0[q] = *reinterpret_cast<const float4*>(patch + r * 32 + (((2 * c8) ^ sx) * 4));
            v1[q] = *reinterpret_cast<const float4*>(patch + r * 32 + (((2 * c8 + 1) ^ sx) * 4));
          }
          const u32x4 rcur[2] = {rnext[0], rnext[1]};
          if constexpr (MODE == EPI_RES) {
            if (b + 1 < TM * TN) {
#pragma unroll
              for (int q = 0; q < 2; ++q) rnext[q] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)out_off(b + 1, q), 0, 0);
              bnext = bias_req((b + 1) % TN);
            }
          }
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const bf16x8 rv = __builtin_bit_cast(bf16x8, rcur[q]);
            const float vals[8] = {v0[q].x, v0[q].y, v0[q].z, v0[q].w, v1[q].x, v1[q].y, v1[q].z, v1[q].w};
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              // one order of additions in every variant (value + bias + residual; the absent
              // terms are exact zeros), so the variant never changes a bit
              float v = vals[e];
              if constexpr (MODE != EPI_PLAIN) v += bvals[e];
              if constexpr (MODE == EPI_RES) v += (float)rv[e];
              o[e] = (bf16)v;
            }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), rc, (int)out_off(b, q), 0, 0);
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    __syncthreads();               // the patch lives in the stage the next step overwrites
  };
  // Plain and bias variants when the wave tile is 64 columns wide: the two column blocks of
  // a row block are rounded to bf16 in accumulator layout (bias added in fp32 first) and
  // pass through the patch together as 32 rows of 128 bytes, 16-byte chunks XOR-swizzled
  // by (row/2)%8; they leave as whole 128-byte lines, 8 rows per store instruction.
  auto finish_rows = [&](const WorkItem& it, int free_stage, auto mode_) {
    constexpr int MODE = decltype(mode_)::value;
    static_assert(TN % 2 == 0, "row-wide epilogue moves 64-column halves of the wave tile");
    unsigned char* patch = smem + free_stage + wave * 4096;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int elr = ln & 31, ehb = ln >> 5;
    // bias of the columns this lane holds in accumulator layout: block j, group g -> 4 values
    u32x2 braw[MODE == EPI_BIAS ? TN * 4 : 1] = {};
    if constexpr (MODE == EPI_BIAS) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int col = it.n0 + wn + 32 * j + 8 * g + 4 * ehb;
          braw[4 * j + g] = __builtin_amdgcn_raw_buffer_load_b64(rbias, col < N ? col * 2 : (int)kOob, 0, 0);
        }
    }
    const int wr = elr * 128 + ehb * 8, wsx = (elr >> 1) & 7;
    const int c16 = ln & 7;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int h = 0; h < TN / 2; ++h) {         // 64-column halves of the wave tile
        const int ocol = it.n0 + wn + 64 * h + 8 * c16;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            bf16x4 o;
            bf16x4 bv = {};
            if constexpr (MODE == EPI_BIAS) bv = __builtin_bit_cast(bf16x4, braw[4 * (2 * h + j) + g]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float v = acc[i][2 * h + j][4 * g + e];
              if constexpr (MODE == EPI_BIAS) v += (float)bv[e];
              o[e] = (bf16)v;
            }
            *reinterpret_cast<bf16x4*>(patch + wr + (((4 * j + g) ^ wsx) << 4)) = o;
          }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        u32x4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int r = (ln >> 3) + 8 * q;
          v[q] = *reinterpret_cast<const u32x4*>(patch + r * 128 + ((c16 ^ ((r >> 1) & 7)) << 4));
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = it.m0 + wm + 32 * i + (ln >> 3) + 8 * q;
          const unsigned off = (ocol < N) ? (unsigned)(((int64_t)row * ldc + ocol) * 2) : kOob;
          __builtin_amdgcn_raw_buffer_store_b128(v[q], rc, (int)off, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    __syncthreads();               // the patch lives in the stage the next step overwrites
  };
  // Activation variants (forward form, no residual): every row block passes through the patch
  // twice, first the output itself (bias added in fp32, rounded to bf16) on its way to C, then
  // the activation of those rounded values on its way to C2.  The bias descriptor of a null
  // bias is empty and reads zeros.
  auto finish_act = [&](const WorkItem& it, int free_stage) {
    static_assert(ACT == ACT_NONE || TN == 2, "a wave holds two 32-column blocks");
    constexpr bool GU = ACT == ACT_SWIGLU;
    unsigned char* patch = smem + free_stage + wave * 4096;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int elr = ln & 31, ehb = ln >> 5;
    const __amdgpu_buffer_rsrc_t rc2 = make_rsrc(aa.C2, aa.c2_bytes);
    // first column in C of the wave's accumulator block 0 and block 1
    const int zc0 = GU ? (it.n0 >> 1) + (wn >> 1) : it.n0 + wn;
    const int zc1 = GU ? zc0 + aa.gu_f : zc0 + 32;
    u32x2 braw[8];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = (j ? zc1 : zc0) + 8 * g + 4 * ehb;
        braw[4 * j + g] = __builtin_amdgcn_raw_buffer_load_b64(rbias, col < N ? col * 2 : (int)kOob, 0, 0);
      }
    const int wr = elr * 128 + ehb * 8, wsx = (elr >> 1) & 7;
    const int c16 = ln & 7;
    // column this lane writes back (16 bytes = 8 columns of patch chunk c16), in C and in C2
    const int zcol = c16 < 4 ? zc0 + 8 * c16 : zc1 + 8 * (c16 - 4);
    const int acol = GU ? (c16 < 4 ? zc0 + 8 * c16 : -1) : zcol;
    const int a_n = GU ? aa.gu_f : N;
    // the value stored to C for accumulator register (i, j, 4g+e)
    auto zval = [&](int i, int j, int g, int e) -> float {
      const bf16x4 bv = __builtin_bit_cast(bf16x4, braw[4 * j + g]);
      return (float)(bf16)(acc[i][j][4 * g + e] + (float)bv[e]);
    };
    auto patch_sync = [&]() {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // patch (32 rows of 128 bytes, chunks XOR-swizzled) -> rows of `rsrc`, 8 rows per instruction
    auto drain = [&](int i, __amdgpu_buffer_rsrc_t rsrc, int64_t ld, int col, int ncols) {
      u32x4 v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r = (ln >> 3) + 8 * q;
        v[q] = *reinterpret_cast<const u32x4*>(patch + r * 128 + ((c16 ^ ((r >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = it.m0 + wm + 32 * i + (ln >> 3) + 8 * q;
        const unsigned off = (col >= 0 && col < ncols) ? (unsigned)(((int64_t)row * ld + col) * 2) : kOob;
        __builtin_amdgcn_raw_buffer_store_b128(v[q], rsrc, (int)off, 0, 0);
      }
    };
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)zval(i, j, g, e);
          *reinterpret_cast<bf16x4*>(patch + wr + (((4 * j + g) ^ wsx) << 4)) = o;
        }
      patch_sync();
      drain(i, rc, ldc, zcol, N);
      patch_sync();
      if constexpr (GU) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)swiglu_f(zval(i, 0, g, e), zval(i, 1, g, e));
          *reinterpret_cast<bf16x4*>(patch + wr + ((g ^ wsx) << 4)) = o;
        }
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)gelu_f(zval(i, j, g, e));
            *reinterpret_cast<bf16x4*>(patch + wr + (((4 * j + g) ^ wsx) << 4)) = o;
          }
      }
      patch_sync();
      drain(i, rc2, aa.ldc2, acol, a_n);
      patch_sync();
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    __syncthreads();               // the patch lives in the stage the next step overwrites
  };
  // Only the forward form meets a bias without a residual often enough to hold a variant for
  // it; elsewhere such a call takes EPI_RES, whose empty residual descriptor reads zeros.
  constexpr bool BIAS_VARIANT = A_KC && !B_KC;
  const int epi_mode = SPLITK ? EPI_PLAIN : (R != nullptr) ? EPI_RES
                     : (bias != nullptr) ? (BIAS_VARIANT ? EPI_BIAS : EPI_RES) : EPI_PLAIN;
  auto finish = [&](const WorkItem& it, int free_stage) {
    if constexpr (SPLITK) {
      finish_impl(it, free_stage, std::integral_constant<int, EPI_PLAIN>{});
    } else if constexpr (ACT != ACT_NONE) {
      finish_act(it, free_stage);
    } else {
      if (epi_mode == EPI_RES) { finish_impl(it, free_stage, std::integral_constant<int, EPI_RES>{}); return; }
      if constexpr (BIAS_VARIANT) {
        if (epi_mode == EPI_BIAS) { finish_rows(it, free_stage, std::integral_constant<int, EPI_BIAS>{}); return; }
      }
      finish_rows(it, free_stage, std::integral_constant<int, EPI_PLAIN>{});
    }
  };

  int kt = cur.kt0;
  // One pipeline step, straight-line: the K-tile AHEAD of the compute cursor is requested
  // into the stage that was read last step, the current K-tile is multiplied, and before
  // the barrier every wave waits for its own requests of the K-tile two ahead, so that
  // after the barrier that tile is complete for all waves.
  // Written slot by slot: one MFMA, then at most a fragment read and a request, then a
  // scheduling barrier that keeps the compiler from regrouping them.  A wave that is alone
  // on its SIMD has nobody to cover a clump of requests or a wait for a read it has just
  // issued, so every fragment is read a whole batch of MFMAs before its first use and the
  // requests are spread over the first batch.
  // The barrier is the bare instruction.  What it has to order: (1) requests into the
  // stage read in this step are issued in the next step, after every wave has passed this
  // barrier, and all reads of that stage feed MFMAs that precede the barrier in program
  // order (the scheduling barriers keep them there), so those reads have returned;
  // (2) each wave has waited for its own requests of the K-tile two ahead before it
  // arrives, so after the barrier that tile is complete.
  constexpr int NM = TM * TN, NF = TM + TN;
  auto read_frag = [&](bf16x8* fa, bf16x8* fb, int stage, int ks, int r) {
    // fragment order: weight-side block 0, the TM activation-side blocks, the other weight-side blocks
    if (r == 0) fb[0] = frb.read(lds + stage + BM * 64, 0, ks);
    else if (r <= TM) fa[r - 1] = fra.read(lds + stage, r - 1, ks);
    else fb[r - TM] = frb.read(lds + stage + BM * 64, r - TM, ks);
  };
  auto step = [&]() {
    const int rd = stg(0), nx = stg(1), ldst = stg(AHEAD);
    const typename LA::Prep pa = la.prep(lta, lkt, K, lit.kt_end, lit.valid);
    const typename LB::Prep pb = lb.prep(ltb, lkt, K, lit.kt_end, lit.valid);
    const unsigned dsta = lds0 + (unsigned)ldst, dstb = dsta + BM * 64;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < NM; ++q) {
      const int i = q % TM, j = q / TM;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb0[j], fa0[i], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int r = (q * NF + NM - 1) / NM; r < ((q + 1) * NF + NM - 1) / NM; ++r) read_frag(fa1, fb1, rd, 1, r);   // k-step 1 of this K-tile
#pragma unroll
      for (int l = q * NLOADS / NM; l < (q + 1) * NLOADS / NM; ++l) {
        if (l < LA::NI) la.issue_j(da, lta, pa, l, dsta);
        else lb.issue_j(db, ltb, pb, l - LA::NI, dstb);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < NM; ++q) {
      const int i = q % TM, j = q / TM;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb1[j], fa1[i], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int r = (q * NF + NM - 1) / NM; r < ((q + 1) * NF + NM - 1) / NM; ++r) read_frag(fa0, fb0, nx, 0, r);   // k-step 0 of the next K-tile
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_loads(std::integral_constant<int, 2 * NLOADS>{});
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    si = si + 1 >= NS ? 0 : si + 1;
    ++lkt; ++kt;
  };
  while (true) {
    int n = cur.kt_end - kt;
    if (lit.valid) n = min(n, lit.kt_end - lkt);
    for (; n > 0; --n) step();
    if (lit.valid && lkt >= lit.kt_end) load_cursor_next_item();
    if (kt >= cur.kt_end) {
      // an item is claimed under the epilogue when none is drawn ahead
      const bool claim = tq.mode == TQ_QUEUE && !have_drawn && !drained && ahead_ok;
      unsigned entry = 0;
      if (claim && threadIdx.x == 0) entry = tq_claim(tq, qc);
      finish(cur, stg(NS - 1));
      if (claim) {
        int v = -1;
        if (threadIdx.x == 0) { int left = 0; const int it = tq_resolve(tq, qc, entry, &left); v = flagged(it, left); }
        drawn = publish(v);
        have_drawn = drawn >= 0;
      }
      if (lqn == 0) break;         // the load cursor has found the queue empty
      cur = decode(lq_pop());
      kt = cur.kt0;
    }
  }
  wait_loads(std::integral_constant<int, 0>{});
  if (threadIdx.x == 0) tq_leave(tq);
}

// Both operands K-contiguous (the input-gradient form), K a multiple of 128: 256x256x64 tile,
// four waves of 128x128 with the accumulators in the accumulator half of the register file.
// A row of a K-contiguous operand gives a whole 128-byte line per K-tile of 64, so the path
// to the L2 carries half the requests of the 32-wide K-tiles of the kernel above.  Operand
// tiles go global -> registers -> LDS: two register sets are in flight (K-tiles kt+1 and kt+2
// while kt is multiplied), LDS is double buffered, one barrier per K-tile.  Every output
// element is still accumulated in ascending k with v_mfma_f32_32x32x16_bf16 in steps of 16
// and rounded once after the same fp32 additions, so its bits equal the other kernel's.
//   LDS tile: rows of 128 bytes, 16-byte pieces XOR-swizzled by (row/2)%8; a fragment is one
//   ds_read_b128 per lane (row = lane%32, piece = 2*kstep + lane/32).
//   Slots: one MFMA each; the fragment reads of the next k-step sit in slots 0..7 of a
//   k-step, the LDS writes (each followed at once by the request that refills its
//   registers) in read-free slots of k-steps 0..2; the barrier comes before k-step 3, whose
//   slots read the first fragments of the next K-tile from the other LDS stage.
template <bool HAS_R>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kc4w_kernel(
    const bf16* __restrict__ A, const bf16* __restrict__ B, bf16* __restrict__ C, const bf16* __restrict__ R,
    int M, int N, int K, int64_t lda, int64_t ldb, int64_t ldc, uint32_t a_bytes, uint32_t b_bytes, uint32_t c_bytes,
    int tiles_m, int tiles_n, int tile_begin, int tile_count, int row_block, TileQueueArgs tq) {
  constexpr int TBM = 256, TBK = 64, OPB = TBM * TBK * 2, STG = 2 * OPB;
  extern __shared__ __align__(16) unsigned char smem[];
  lds_byte* const lds = (lds_byte*)smem;
  typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
  typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  const int lr = lane & 31, hb = lane >> 5;
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(A, a_bytes), rb = make_rsrc(B, b_bytes);
  const __amdgpu_buffer_rsrc_t rc = make_rsrc(C, c_bytes), rr = make_rsrc(R, HAS_R ? c_bytes : 0u);
  const int nk = K / TBK;                       // even: K is a multiple of 128
  // this thread's 8 pieces of an operand tile: piece c = tid + 256*i -> tile row tid/8 + 32*i,
  // 16 bytes tid%8.  The swizzle term (row/2)%8 is the same for all eight (32*i/2 is a
  // multiple of 8), so one LDS offset serves with immediates 4096*i; likewise for the
  // fragment rows lr + 32*i.
  const int grow0 = tid >> 3, gch = tid & 7;
  const int lwr0 = grow0 * 128 + ((gch ^ ((grow0 >> 1) & 7)) << 4);
  const int fro0 = lr * 128, frsw = (lr >> 1) & 7;
  // Items come from the work queue (tile_queue.h), in the same panel-major tile list as
  // gemm_bf16_kernel.  Thread 0 claims the next tile when the K loop is done and resolves the
  // claim after the epilogue, so the round trip hides under the epilogue.
  __shared__ int mail;
  TileQueueCursor qc;
  int item = tq_first(tq, qc, &mail);
  while (item >= 0) {
    const int tile = tile_begin + item;
    int trow, tcol;
    tile_coords(tile, tiles_m, tiles_n, row_block, &trow, &tcol);
    const int m0 = trow * TBM, n0 = tcol * TBM;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // byte offsets of this thread's pieces at K-tile 0; rows past the end fall outside the
    // descriptor's range and read zeros
    const unsigned oa0 = (unsigned)(((int64_t)(m0 + grow0) * lda) * 2 + gch * 16);
    const unsigned ob0 = (unsigned)(((int64_t)(n0 + grow0) * ldb) * 2 + gch * 16);
    const unsigned sa = (unsigned)(32 * lda * 2), sb = (unsigned)(32 * ldb * 2);     // 32 rows further
    // K-tiles past the end are requested too (their registers are never used): the piece
    // must not alias a valid row of the next K range, so it is sent out of range
    auto ga_load = [&](int i, int kt) -> u32x4 {
      return __builtin_amdgcn_raw_buffer_load_b128(ra, kt < nk ? (int)(oa0 + (unsigned)i * sa + (unsigned)kt * (TBK * 2)) : (int)kOob, 0, 0);
    };
    auto gb_load = [&](int i, int kt) -> u32x4 {
      return __builtin_amdgcn_raw_buffer_load_b128(rb, kt < nk ? (int)(ob0 + (unsigned)i * sb + (unsigned)kt * (TBK * 2)) : (int)kOob, 0, 0);
    };
    u32x4 ga0[8], gb0[8], ga1[8], gb1[8];
    bf16x8 fa[2][4], fb[2][4];
    // prologue: K-tile 0 -> register set 1 -> LDS stage 0 and K-tile 1 -> register set 0 are
    // requested together (one round trip, not two), then K-tile 2 -> register set 1
    __syncthreads();                    // the previous tile's epilogue is done with the LDS
#pragma unroll
    for (int i = 0; i < 8; ++i) { ga1[i] = ga_load(i, 0); gb1[i] = gb_load(i, 0); }
#pragma unroll
    for (int i = 0; i < 8; ++i) { ga0[i] = ga_load(i, 1); gb0[i] = gb_load(i, 1); }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<lds_u32x4*>(lds + lwr0 + 4096 * i) = ga1[i];
      *reinterpret_cast<lds_u32x4*>(lds + OPB + lwr0 + 4096 * i) = gb1[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) { ga1[i] = ga_load(i, 2); gb1[i] = gb_load(i, 2); }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[0][i] = *reinterpret_cast<const lds_bf16x8*>(lds + wm * 128 + fro0 + 4096 * i + ((hb ^ frsw) << 4));
      fb[0][i] = *reinterpret_cast<const lds_bf16x8*>(lds + OPB + wn * 128 + fro0 + 4096 * i + ((hb ^ frsw) << 4));
    }
    auto body = [&](int kt, auto sel_) {
      constexpr int SEL = decltype(sel_)::value;
      const int st = kt & 1;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int cur = ks & 1, nxt = cur ^ 1;
        // K-tile kt+1 is in LDS for everybody and nobody reads stage st after this k-step
        if (ks == 3) __syncthreads();
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int i = q & 3, j = q >> 2;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
          if (q < 8) {
            // fragments of the next k-step (of the next K-tile's first k-step when ks == 3)
            const int rs_ = ks < 3 ? st : st ^ 1, rk = ks < 3 ? ks + 1 : 0;
            if (q < 4) fa[nxt][q] = *reinterpret_cast<const lds_bf16x8*>(lds + rs_ * STG + wm * 128 + fro0 + 4096 * q + (((2 * rk + hb) ^ frsw) << 4));
            else fb[nxt][q - 4] = *reinterpret_cast<const lds_bf16x8*>(lds + rs_ * STG + OPB + wn * 128 + fro0 + 4096 * (q - 4) + (((2 * rk + hb) ^ frsw) << 4));
          }
          if ((ks < 2 && q >= 8 && q < 14) || (ks == 2 && q >= 8 && q < 12)) {
            // register set SEL (K-tile kt+1) -> the other LDS stage; the freed registers go
            // straight back out for K-tile kt+3
            const int w = ks * 6 + (q - 8), i8 = w >> 1;
            if ((w & 1) == 0) {
              u32x4& a_ = SEL ? ga1[i8] : ga0[i8];
              *reinterpret_cast<lds_u32x4*>(lds + (st ^ 1) * STG + lwr0 + 4096 * i8) = a_;
              a_ = ga_load(i8, kt + 3);
            } else {
              u32x4& b_ = SEL ? gb1[i8] : gb0[i8];
              *reinterpret_cast<lds_u32x4*>(lds + (st ^ 1) * STG + OPB + lwr0 + 4096 * i8) = b_;
              b_ = gb_load(i8, kt + 3);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    for (int kt = 0; kt < nk; kt += 2) {
      body(kt, std::integral_constant<int, 0>{});
      body(kt + 1, std::integral_constant<int, 1>{});
    }
    __syncthreads();                    // every wave is done reading fragments: LDS is free
    const unsigned entry = tq_claim_ahead(tq, qc);

    // Epilogue, one 32x32 block at a time through a 4 KB fp32 patch per wave (XOR swizzled),
    // leaving row-contiguous; the residual is added in fp32 in that layout, one rounding.
    // acc[i][j][4g+e] is output (row m0+wm+32i+lr, column n0+wn+32j+8g+4hb+e).
    {
      float* patch = reinterpret_cast<float*>(smem) + wave * 1024;
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int elr = ln & 31, ehb = ln >> 5;
      auto out_off = [&](int b, int q) -> unsigned {
        const int row = m0 + wm + 32 * (b >> 2) + (ln >> 2) + 16 * q;
        const int col = n0 + wn + 32 * (b & 3) + 8 * (ln & 3);
        return (col < N) ? (unsigned)(((int64_t)row * ldc + col) * 2) : kOob;
      };
      u32x4 rnext[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
      if constexpr (HAS_R) {
#pragma unroll
        for (int q = 0; q < 2; ++q) rnext[q] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)out_off(0, q), 0, 0);
      }
#pragma unroll
      for (int b = 0; b < 16; ++b) {
        const int i = b >> 2, j = b & 3;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int cg = (2 * g + ehb) ^ ((elr >> 1) & 7);
          float4 v = make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
          *reinterpret_cast<float4*>(patch + elr * 32 + cg * 4) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float4 v0[2], v1[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int r = (ln >> 2) + 16 * q, c8 = ln & 3, sx = (r >> 1) & 7;
          v0[q] = *reinterpret_cast<const float4*>(patch + r * 32 + (((2 * c8) ^ sx) * 4));
          v1[q] = *reinterpret_cast<const float4*>(patch + r * 32 + (((2 * c8 + 1) ^ sx) * 4));
        }
        const u32x4 rcur[2] = {rnext[0], rnext[1]};
        if constexpr (HAS_R) {
          if (b + 1 < 16) {
#pragma unroll
            for (int q = 0; q < 2; ++q) rnext[q] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)out_off(b + 1, q), 0, 0);
          }
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const bf16x8 rv = __builtin_bit_cast(bf16x8, rcur[q]);
          const float vals[8] = {v0[q].x, v0[q].y, v0[q].z, v0[q].w, v1[q].x, v1[q].y, v1[q].z, v1[q].w};
          bf16x8 o;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float v = vals[e];
            if constexpr (HAS_R) { v += 0.f; v += (float)rv[e]; }   // value + (absent bias) + residual
            o[e] = (bf16)v;
          }
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), rc, (int)out_off(b, q), 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
    item = tq_next(tq, qc, entry, &mail);
  }
  tq_done(tq);
}

// out = bf16( P[0] + P[1] + ... ) in ascending piece order, for the tiles [tile_begin,
// tile_begin + tile_count) of the 256x256 tile list that the split launch covered.  One block
// iteration takes four rows of one tile (256 float4), so the tile's place is found once per
// iteration.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ P, bf16* __restrict__ C,
                                                            int M, int N, int64_t ldc, int ksplit, int tiles_m,
                                                            int tiles_n, int tile_begin, int tile_count, int row_block) {
  const int64_t piece = (int64_t)tile_count * 65536;
  const int units = tile_count * 64;
  for (int u = blockIdx.x; u < units; u += gridDim.x) {
    const int tl = u >> 6;
    int trow, tcol;
    tile_coords(tile_begin + tl, tiles_m, tiles_n, row_block, &trow, &tcol);
    const int r = (u & 63) * 4 + (threadIdx.x >> 6), c = (threadIdx.x & 63) * 4;
    const int row = trow * 256 + r, col = tcol * 256 + c;
    if (row >= M || col >= N) continue;
    const float* src = P + (int64_t)tl * 65536 + r * 256 + c;
    float4 a = *reinterpret_cast<const float4*>(src);
    for (int s = 1; s < ksplit; ++s) {
      const float4 b = *reinterpret_cast<const float4*>(src + s * piece);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    bf16x4 o;
    o[0] = (bf16)a.x; o[1] = (bf16)a.y; o[2] = (bf16)a.z; o[3] = (bf16)a.w;
    *reinterpret_cast<bf16x4*>(C + (int64_t)row * ldc + col) = o;
  }
}

// ------------------------------------------------------------------ generic FMA kernel
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    const T* __restrict__ A, const T* __restrict__ B, T* __restrict__ C, const T* __restrict__ bias,
    const T* __restrict__ R, int M, int N, int K, int64_t sam, int64_t sak, int64_t sbk, int64_t sbn,
    int64_t ldc, int tiles_m, int tiles_n) {
  constexpr int TS = 64, KS = 16;
  __shared__ float As[KS][TS + 1];
  __shared__ float Bs[KS][TS + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int ntiles = tiles_m * tiles_n;
  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int tn_i = tile / tiles_m, tm_i = tile - tn_i * tiles_m;
    const int m0 = tm_i * TS, n0 = tn_i * TS;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < K; k0 += KS) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int idx = threadIdx.x + 256 * q;     // 0..1023
        // A tile: prefer the contiguous index to vary fastest across threads
        int am, ak;
        if (sak == 1) { ak = idx % KS; am = idx / KS; } else { am = idx % TS; ak = idx / TS; }
        const int gm = m0 + am, gk = k0 + ak;
        As[ak][am] = (gm < M && gk < K) ? to_f32(A[(int64_t)gm * sam + (int64_t)gk * sak]) : 0.f;
        int bn, bk;
        if (sbk == 1) { bk = idx % KS; bn = idx / KS; } else { bn = idx % TS; bk = idx / TS; }
        const int gn = n0 + bn, gk2 = k0 + bk;
        Bs[bk][bn] = (gn < N && gk2 < K) ? to_f32(B[(int64_t)gk2 * sbk + (int64_t)gn * sbn]) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < KS; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = m0 + ty * 4 + i;
      if (row >= M) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = n0 + tx * 4 + j;
        if (col >= N) continue;
        float v = acc[i][j];
        if (bias) v += to_f32(bias[col]);
        if (R) v += to_f32(R[(int64_t)row * ldc + col]);
        C[(int64_t)row * ldc + col] = from_f32<T>(v);
      }
    }
  }
}


// One launch of the MFMA kernel over coarse tiles [tile_begin, tile_begin + tile_count) of the
// panel-major list of (sub*BM) x (sub*BN) tiles; tile_count < 0 means all of them.
template <int BM, int BN, int NWM, int NWN, bool A_KC, bool B_KC, bool SPLITK = false, int ACT = ACT_NONE>
mosaic_status launch_mfma(hipStream_t s, int quota, int M, int N, int K, const bf16* A, int64_t lda,
                          const bf16* B, int64_t ldb, bf16* C, int64_t ldc, const bf16* bias, const bf16* R,
                          uint32_t a_bytes, uint32_t b_bytes, uint32_t c_bytes, int ksplit = 1,
                          int ktiles_per = 0, float* P = nullptr, int sub = 1, int tile_begin = 0,
                          int tile_count = -1, const ActArgs& aa = ActArgs()) {
  constexpr size_t smem = (size_t)NS * (BM + BN) * 64;
  auto kern = gemm_bf16_kernel<BM, BN, NWM, NWN, A_KC, B_KC, SPLITK, ACT>;
  static std::once_flag attr_once;   // per instantiation; launches come from several host threads
  static hipError_t attr_rc = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  });
  MOSAIC_HIP(attr_rc);
  const int tiles_m = (int)ceil_div(M, BM * sub), tiles_n = (int)ceil_div(N, BN * sub);
  if (tile_count < 0) tile_count = tiles_m * tiles_n - tile_begin;
  if (tile_count <= 0) return MOSAIC_OK;
  const int wg_per_cu = (BM == 256) ? 1 : 2;
  const int64_t items = (int64_t)tile_count * sub * sub * ksplit;
  if (items > INT32_MAX) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "too many output tiles");
  TileQueueArgs tq;
  int grid;
  MOSAIC_TRY(tile_queue_plan(s, quota, wg_per_cu, items, 0, false, &tq, &grid));
  ActArgs ka = aa;
  // coarse tile rows are BM * sub rows high; every launch over one product (whole rounds,
  // quarter tiles, split tiles) walks the same tile list
  ka.row_block = row_block_for(K, ceil_div((int64_t)M, 256)) * 256 / (BM * sub);
  kern<<<grid, 64 * NWM * NWN, smem, s>>>(A, B, C, bias, R, M, N, K, lda, ldb, ldc, a_bytes, b_bytes, c_bytes,
                                          tiles_m, tiles_n, tile_begin, tile_count, sub, ksplit, ktiles_per, P, tq, ka);
  MOSAIC_LAUNCH_CHECK();
  if (SPLITK) {
    static_assert(!SPLITK || (BM == 256 && BN == 256), "the reduce kernel walks 256x256 tiles");
    const int g2 = grid_for(quota, 8, (int64_t)tile_count * 64);
    splitk_reduce_kernel<<<g2, 256, 0, s>>>(P, C, M, N, ldc, ksplit, tiles_m, tiles_n, tile_begin, tile_count, ka.row_block);
    MOSAIC_LAUNCH_CHECK();
  }
  return MOSAIC_OK;
}

// The four-wave kernel for the K-contiguous x K-contiguous form: whole tiles only (sub = 1).
mosaic_status launch_kc4w(hipStream_t s, int quota, int M, int N, int K, const bf16* A, int64_t lda, const bf16* B,
                          int64_t ldb, bf16* C, int64_t ldc, const bf16* R, uint32_t a_bytes, uint32_t b_bytes,
                          uint32_t c_bytes, int tile_begin, int tile_count) {
  constexpr size_t smem = 2 * 2 * 256 * 64 * 2;        // two stages of two 256 x 64 operand tiles
  static std::once_flag attr_once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kc4w_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (attr_rc == hipSuccess)
      attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kc4w_kernel<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  });
  MOSAIC_HIP(attr_rc);
  const int tiles_m = (int)ceil_div(M, 256), tiles_n = (int)ceil_div(N, 256);
  if (tile_count < 0) tile_count = tiles_m * tiles_n - tile_begin;
  if (tile_count <= 0) return MOSAIC_OK;
  TileQueueArgs tq;
  int grid;
  MOSAIC_TRY(tile_queue_plan(s, quota, 1, tile_count, 0, false, &tq, &grid));
  const int rb = row_block_for(K, tiles_m);
  if (R) gemm_bf16_kc4w_kernel<true><<<grid, 256, smem, s>>>(A, B, C, R, M, N, K, lda, ldb, ldc, a_bytes, b_bytes, c_bytes,
                                                             tiles_m, tiles_n, tile_begin, tile_count, rb, tq);
  else gemm_bf16_kc4w_kernel<false><<<grid, 256, smem, s>>>(A, B, C, R, M, N, K, lda, ldb, ldc, a_bytes, b_bytes, c_bytes,
                                                            tiles_m, tiles_n, tile_begin, tile_count, rb, tq);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

// A/B switches for kernel timing, compiled in only with -DMOSAIC_TUNING (never in the library
// that ships): MOSAIC_GEMM_KC4W=0 sends the input-gradient form back to the eight-wave kernel,
// MOSAIC_GEMM_TILE=256 / 128 / 1 forces the all-256, all-128 or mixed tile plan (the bits are
// the same either way); MOSAIC_SPLITK=n forces the piece count of a weight gradient's cut tail
// (0: no cut; the bits differ with n).
#ifdef MOSAIC_TUNING
bool kc4w_enabled() {
  static int v = -1;
  if (v < 0) { const char* e = getenv("MOSAIC_GEMM_KC4W"); v = e ? atoi(e) : 1; }
  return v != 0;
}
int forced_tile() {
  static int v = -1;
  if (v < 0) { const char* e = getenv("MOSAIC_GEMM_TILE"); v = e ? atoi(e) : 0; }
  return v;
}
#else
constexpr bool kc4w_enabled() { return true; }
constexpr int forced_tile() { return 0; }
#endif

// Splitting the weight-gradient form along K.  Its contraction runs over the tokens and is
// long; its output has few tiles.  Two cases, both decided by the shape alone (256 = CUs of the
// device the kernels are written for; never the quota, so the bits stay quota-independent):
//  - up to 128 tiles of 256x256: every tile is cut, into about as many work items as CUs;
//  - more: the tiles that do not fill a round of 256 (the tail of the tile list) are cut when
//    the contraction is at least 16384 long and the cut is priced well below the alternatives,
//    one more round of large tiles or the tail as quarter tiles.  Prices in microseconds on the
//    whole device: a 256x256 tile takes 25.5 ns per unit of K, a work item 12 us on top
//    (pipeline fill, fp32 store of its piece), the pass that adds the pieces reads them at
//    3.5 TB/s after 8 us; two small workgroups per CU take 1.8 quarter units each (as in
//    launch_mfma_shape).  Measured, pieces forced to 2 .. 8: the gate/up gradient at T=32768
//    (1376 tiles, 96 in the tail) 4845 us uncut, 4624 in 5 pieces (the plan's choice; 2 and 8
//    pieces within 15 us of it); the same at T=16384 2405 -> 2315; the down-projection gradient
//    (688 tiles, 176 in the tail, else a third round of large tiles) 2410 -> 2362 in 4 pieces
//    and slower in any other count; at T=8192 no cut gains anything (331 us either way for 96
//    tail tiles, 178 -> 211 and worse for a lone round of 192 tiles): pieces of a few thousand
//    tokens are mostly fill and drain.
// *first: first tile of the list that is cut; returns the piece count (1: nothing is cut).
int splitk_plan(int64_t M, int64_t N, int64_t K, int* first) {
  const int64_t t256 = ceil_div(M, 256) * ceil_div(N, 256);
  *first = 0;
  if (N % 4) return 1;
  if (t256 <= 128) {
    if (K < 2048) return 1;
    int64_t s = 256 / t256;
    if (s > 8) s = 8;
    while (s > 1 && ceil_div(K, s) < 512) --s;
    return (int)s;
  }
  const int64_t tail = t256 % 256;
  if (tail == 0 || K < 16384) return 1;
  const double tile_us = 25.5e-3 * (double)K;
  int best = 1;
  double best_us = 1e30;
  for (int s = 2; s <= 8 && K / s >= 1024; ++s) {
    const double pieces = (double)(tail * s);
    const double us = (double)ceil_div(tail * s, 256) * (tile_us / s + 12.0) + pieces * 262144.0 / 3.5e6 + 8.0;
    if (us < best_us - 1e-9) { best_us = us; best = s; }
  }
  const int64_t q = 4 * tail, full = q / 512, rem = q % 512;
  const double quarter_us = ((double)full * 2.0 * 1.8 + (rem == 0 ? 0.0 : rem <= 256 ? 1.2 * 1.8 : 2.0 * 1.8)) / 4.0 * tile_us;
  const double other_us = std::min(tile_us, quarter_us);            // one more round of large tiles, or quarter tiles
#ifdef MOSAIC_TUNING
  if (const char* e = getenv("MOSAIC_SPLITK")) { const int f = atoi(e); if (f <= 1) return 1; *first = (int)(t256 - tail); return f; }
#endif
  if (best == 1 || best_us >= 0.92 * other_us) return 1;
  *first = (int)(t256 - tail);
  return best;
}

template <bool A_KC, bool B_KC>
mosaic_status launch_mfma_shape(hipStream_t s, int quota, int M, int N, int K, const bf16* A, int64_t lda,
                                const bf16* B, int64_t ldb, bf16* C, int64_t ldc, const bf16* bias, const bf16* R,
                                uint32_t a_bytes, uint32_t b_bytes, uint32_t c_bytes, void* splitk_scratch,
                                const ActArgs& aa = ActArgs()) {
  // tiles [split_first, t256) of the tile list are cut along K (weight-gradient form only); the
  // tiles before them are planned below as if they were the whole product
  int64_t t256 = ceil_div(M, 256) * ceil_div(N, 256);
  const int64_t t256_all = t256;
  int sk = 1, split_first = 0;
  if constexpr (!A_KC && !B_KC) {
    if (splitk_scratch && !bias && !R) sk = splitk_plan(M, N, K, &split_first);
  }
  auto launch_split = [&]() -> mosaic_status {
    const int per = (int)ceil_div(ceil_div(K, BK), sk);
    return launch_mfma<256, 256, 2, 4, A_KC, B_KC, true>(s, quota, M, N, K, A, lda, B, ldb, C, ldc, bias, R, a_bytes, b_bytes, c_bytes,
                                                         sk, per, (float*)splitk_scratch, 1, split_first, (int)(t256_all - split_first));
  };
  const bool part = sk > 1;          // the plans below cover tiles [0, t256) only
  if (part) {
    if (split_first == 0) return launch_split();
    t256 = split_first;
  }
  // Tile shape only decides which workgroup computes an element, never its bits.  Large
  // tiles halve LDS traffic per MFMA; small tiles fill the CUs when there are few large
  // ones.  Three plans, priced in units of a quarter of a 256x256 tile's time on one CU:
  //   all-256: whole rounds of 256x256 tiles, the last one possibly mostly idle;
  //   all-128: 128x128 tiles, two workgroups per CU;
  //   mixed:   the whole rounds with the large kernel, then the tiles of the partial round
  //            as quarter tiles with the small kernel.
  // rounds are counted with the CUs that are certain to run a workgroup at the same time
  const int launch_quota = quota;
  quota = tile_queue_sure_cus(quota);
  const int64_t t128 = part ? 4 * t256 : ceil_div(M, 128) * ceil_div(N, 128);
  auto cost_small = [&](int64_t tiles) {       // 128x128 tiles on `quota` CUs
    const int64_t full = tiles / (2 * (int64_t)quota), rem = tiles % (2 * (int64_t)quota);
    // a CU shared by two workgroups finishes both in about 2 x 1.35 units (more when the
    // operands need the transposing LDS writes), a workgroup alone in 1.6
    constexpr double pen = (A_KC && B_KC) ? 1.3 : (!A_KC && !B_KC) ? 1.8 : 1.45;
    return (double)full * 2.0 * pen + (rem == 0 ? 0.0 : rem <= quota ? 1.2 * pen : 2.0 * pen);
  };
  // whole 256x256 tiles of the K-contiguous x K-contiguous form go to the four-wave kernel
  // (its K-tiles are 64 wide and come in pairs; no bias in its epilogue); a round of it takes
  // about 3.7 units where the eight-wave kernel takes 4
  const bool kc4w = A_KC && B_KC && !bias && (K % 128 == 0) && kc4w_enabled();
  const double round256 = kc4w ? 3.7 : 4.0;
  const int64_t whole = t256 / quota, rest = t256 % quota;
  const double cost256 = (double)ceil_div(t256, quota) * round256;
  const double cost128 = cost_small(t128);
  const double cost_mix = (whole > 0 && rest > 0) ? (double)whole * round256 + cost_small(4 * rest) + 0.15 : 1e30;
  int plan = cost256 <= cost128 ? (cost256 <= cost_mix ? 256 : 0) : (cost128 <= cost_mix ? 128 : 0);
  if (forced_tile() == 128 || forced_tile() == 256) plan = forced_tile();
  if (forced_tile() == 1 && whole > 0 && rest > 0) plan = 0;
  // one launch of the eight-wave (big) or four-wave quarter-tile kernel over coarse tiles
  // [tile_begin, tile_begin + tile_count) (tile_count < 0: all), with the epilogue `aa` asks for
  auto launch_tiles = [&](auto big_, int sub, int tile_begin, int tile_count) -> mosaic_status {
    constexpr bool BIG = decltype(big_)::value;
    constexpr int TB = BIG ? 256 : 128, WN_ = BIG ? 4 : 2;
    if constexpr (A_KC && !B_KC) {
      if (aa.act == ACT_GELU)
        return launch_mfma<TB, TB, 2, WN_, A_KC, B_KC, false, ACT_GELU>(s, launch_quota, M, N, K, A, lda, B, ldb, C, ldc, bias, R, a_bytes, b_bytes,
                                                                        c_bytes, 1, 0, nullptr, sub, tile_begin, tile_count, aa);
      if (aa.act == ACT_SWIGLU)
        return launch_mfma<TB, TB, 2, WN_, A_KC, B_KC, false, ACT_SWIGLU>(s, launch_quota, M, N, K, A, lda, B, ldb, C, ldc, bias, R, a_bytes, b_bytes,
                                                                          c_bytes, 1, 0, nullptr, sub, tile_begin, tile_count, aa);
    }
    return launch_mfma<TB, TB, 2, WN_, A_KC, B_KC>(s, launch_quota, M, N, K, A, lda, B, ldb, C, ldc, bias, R, a_bytes, b_bytes, c_bytes, 1, 0,
                                                   nullptr, sub, tile_begin, tile_count);
  };
  if (plan == 256) {
    if (kc4w) return launch_kc4w(s, launch_quota, M, N, K, A, lda, B, ldb, C, ldc, R, a_bytes, b_bytes, c_bytes, 0, -1);
    MOSAIC_TRY(launch_tiles(std::true_type{}, 1, 0, part ? (int)t256 : -1));
    return part ? launch_split() : MOSAIC_OK;
  }
  if (plan == 128) {
    MOSAIC_TRY(part ? launch_tiles(std::false_type{}, 2, 0, (int)t256) : launch_tiles(std::false_type{}, 1, 0, -1));
    return part ? launch_split() : MOSAIC_OK;
  }
  const int head = (int)(whole * quota);
  mosaic_status st = kc4w ? launch_kc4w(s, launch_quota, M, N, K, A, lda, B, ldb, C, ldc, R, a_bytes, b_bytes, c_bytes, 0, head)
                          : launch_tiles(std::true_type{}, 1, 0, head);
  if (st != MOSAIC_OK) return st;
  MOSAIC_TRY(launch_tiles(std::false_type{}, 2, head, (int)rest));
  return part ? launch_split() : MOSAIC_OK;
}

}  // namespace

size_t gemm_splitk_scratch_bytes(int64_t M, int64_t N, int64_t K) {
  int first = 0;
  const int sk = splitk_plan(M, N, K, &first);
  const int64_t cut = ceil_div(M, 256) * ceil_div(N, 256) - first;      // whole 256x256 tiles, edge tiles too
  return sk > 1 ? (size_t)sk * (size_t)cut * 65536 * sizeof(float) : 0;
}

// fused != null: a forward-form call that also wants act(C) in C2; *fused says whether the
// launch took care of it
static mosaic_status launch_gemm_impl(hipStream_t s, int quota, int dtype, bool a_kc, bool b_kc, int64_t M, int64_t N,
                          int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                          int64_t ldc, const void* bias, const void* R, void* splitk_scratch,
                          int act, void* C2, int64_t ldc2, bool* fused) {
  if (fused) *fused = false;
  if (M < 0 || N < 0 || K < 0) MOSAIC_FAIL(MOSAIC_EINVAL, "negative GEMM size");
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "GEMM dimension too large");
  if (M == 0 || N == 0) return MOSAIC_OK;
  const bool vec_ok = (lda % 8 == 0) && (ldb % 8 == 0) && (K % 8 == 0 || (!a_kc && !b_kc)) &&
                      (a_kc || M % 8 == 0) && (b_kc || N % 8 == 0) &&
                      ((uintptr_t)A % 16 == 0) && ((uintptr_t)B % 16 == 0) && ((uintptr_t)C % 16 == 0) &&
                      (ldc % 8 == 0) && (N % 8 == 0) && K > 0 &&
                      (R == nullptr || (uintptr_t)R % 16 == 0) && (bias == nullptr || (uintptr_t)bias % 16 == 0);
  // extents in bytes as seen by the buffer descriptors (dense rows: ld >= logical width)
  const int64_t a_ext = a_kc ? ((M - 1) * lda + K) * 2 : ((K - 1) * lda + M) * 2;
  const int64_t b_ext = b_kc ? ((N - 1) * ldb + K) * 2 : ((K - 1) * ldb + N) * 2;
  const int64_t c_ext = ((M - 1) * ldc + N) * 2;
  const int64_t lim = (int64_t)1 << 31;
  if (dtype == MOSAIC_BF16 && vec_ok && a_ext < lim && b_ext < lim && c_ext < lim) {
    const uint32_t ab = (uint32_t)a_ext, bb = (uint32_t)b_ext, cb = (uint32_t)c_ext;
    const bf16 *a = (const bf16*)A, *b = (const bf16*)B, *bi = (const bf16*)bias, *r = (const bf16*)R;
    bf16* c = (bf16*)C;
    if (a_kc && !b_kc) {
      ActArgs aa;
      if (fused && C2 && !R && (uintptr_t)C2 % 16 == 0 && ldc2 % 8 == 0) {
        const int64_t n2 = act == MOSAIC_SWIGLU ? N / 2 : N;
        const int64_t c2_ext = ((M - 1) * ldc2 + n2) * 2;
        // gate and up halves must be whole quarter tiles wide: a tile then never straddles the halves
        const bool ok = c2_ext < lim && (act == MOSAIC_GELU || (act == MOSAIC_SWIGLU && N % 256 == 0));
        if (ok) {
          aa.act = act == MOSAIC_GELU ? ACT_GELU : ACT_SWIGLU;
          aa.C2 = (bf16*)C2; aa.ldc2 = ldc2; aa.c2_bytes = (uint32_t)c2_ext;
          aa.gu_f = act == MOSAIC_SWIGLU ? (int)(N / 2) : 0;
          *fused = true;
        }
      }
      return launch_mfma_shape<true, false>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r, ab, bb, cb, splitk_scratch, aa);
    }
    if (a_kc && b_kc) return launch_mfma_shape<true, true>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r, ab, bb, cb, splitk_scratch);
    if (!a_kc && !b_kc) return launch_mfma_shape<false, false>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r, ab, bb, cb, splitk_scratch);
    return launch_mfma_shape<false, true>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r, ab, bb, cb, splitk_scratch);
  }
  const int64_t sam = a_kc ? lda : 1, sak = a_kc ? 1 : lda;
  const int64_t sbk = b_kc ? 1 : ldb, sbn = b_kc ? ldb : 1;
  const int tiles_m = (int)ceil_div(M, 64), tiles_n = (int)ceil_div(N, 64);
  const int grid = grid_for(quota, 8, (int64_t)tiles_m * tiles_n);
  if (dtype == MOSAIC_BF16)
    gemm_generic_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)A, (const bf16*)B, (bf16*)C, (const bf16*)bias,
                                                   (const bf16*)R, (int)M, (int)N, (int)K, sam, sak, sbk, sbn, ldc, tiles_m, tiles_n);
  else
    gemm_generic_kernel<float><<<grid, 256, 0, s>>>((const float*)A, (const float*)B, (float*)C, (const float*)bias,
                                                    (const float*)R, (int)M, (int)N, (int)K, sam, sak, sbk, sbn, ldc, tiles_m, tiles_n);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_gemm(hipStream_t s, int quota, int dtype, bool a_kc, bool b_kc, int64_t M, int64_t N,
                          int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                          int64_t ldc, const void* bias, const void* R, void* splitk_scratch) {
  return launch_gemm_impl(s, quota, dtype, a_kc, b_kc, M, N, K, A, lda, B, ldb, C, ldc, bias, R, splitk_scratch, 0, nullptr, 0, nullptr);
}

mosaic_status launch_linear_act_fwd(hipStream_t s, int quota, int dtype, int act, int64_t T, int64_t k, int64_t n,
                                    const void* X, const void* W, const void* bias, void* Z, void* Aout) {
  if (act != MOSAIC_GELU && act != MOSAIC_SWIGLU && act != MOSAIC_GELU_TANH) MOSAIC_FAIL(MOSAIC_EINVAL, "unknown activation %d", act);
  if (act == MOSAIC_SWIGLU && (n % 2)) MOSAIC_FAIL(MOSAIC_EINVAL, "SwiGLU needs an even output width, got %lld", (long long)n);
  const int64_t na = act == MOSAIC_SWIGLU ? n / 2 : n;
  bool fused = false;
  MOSAIC_TRY(launch_gemm_impl(s, quota, dtype, true, false, T, n, k, X, k, W, n, Z, n, bias, nullptr, nullptr, act, Aout, na,
                              act == MOSAIC_GELU_TANH ? nullptr : &fused));
  if (fused || T == 0 || n == 0) return MOSAIC_OK;
  if (act == MOSAIC_SWIGLU) return launch_swiglu_fwd(s, quota, dtype, T, na, Z, Aout);
  if (act == MOSAIC_GELU_TANH) return launch_gelu_tanh_fwd(s, quota, dtype, T * n, Z, Aout);
  return launch_gelu_fwd(s, quota, dtype, T * n, Z, Aout);
}
