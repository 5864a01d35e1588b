// Flash-style attention for bf16 on the gfx950 matrix cores, head size 64 or 128.
//
// Forward: a workgroup of 4 or 8 waves owns 128 or 256 queries of one (sample, head), one
// wave per 32 queries, and streams key/value tiles of 64 through a ring of LDS stages with
// online softmax.  Scores are computed
// transposed, S^T = K Q^T, so that in the 32x32 accumulator layout a lane owns ONE query
// (column lane%32) and 16 keys (its registers): the row maximum and sum are in-lane
// reductions plus one exchange between the two half-waves, and the running rescale is a
// per-lane scalar.  The probabilities feed the second product O^T = V^T P^T straight from
// registers: MFMA's contraction index may be enumerated in any order as long as both
// operands agree, so V^T is read from LDS in the key order the accumulator layout
// dictates (two 4-key runs per 16-key step).
//
// Streamed tiles go from HBM straight into LDS (buffer_load ... lds), in natural row order
// with the 16-byte chunks of a row XOR-swizzled; a lane chooses which chunk it requests, so
// the swizzle costs nothing.  One copy of a tile serves both uses: as an operand whose
// contraction runs along the row it is read with ds_read_b128, as an operand whose
// contraction runs across rows (V in O^T = V^T P^T, K in dQ, Q and dO in dK / dV) with the
// transposing read ds_read_b64_tr_b16, two per fragment.  The swizzle makes both kinds of
// read conflict-free.
//
// Backward is split in two kernels so that every sum has one owner and a fixed order
// (bit-identical for any grid): the dK/dV kernel owns 128 or 256 keys and streams query
// tiles; the dQ kernel owns 128 or 256 queries and streams key tiles.  Both recompute P from the saved
// row log-sum-exp; D_i = sum_c dO_ic O_ic is formed by the dQ kernel, which runs first, from the
// dO fragments it holds, and read by the dK/dV kernel.
#include <algorithm>
#include <mutex>
#include "kernels.h"
#include "tile_queue.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#ifndef DKV_PF
#define DKV_PF 3
#endif
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Online softmax keeps, per row, a reference value m and sums of exp2(s - m).  Any m works
// (softmax is shift-invariant) as long as the exponentials stay in range, so the reference
// only follows the running maximum when some row's maximum has grown by more than this many
// powers of two: probabilities then reach at most 2^8, well inside bf16 and fp32, and the
// rescale of the running sums (one multiply per accumulator register) becomes rare instead
// of happening on almost every block of a long row.
constexpr float kLazyRescale = 8.0f;
// In the forward kernel's steady state a block's probabilities are formed before anyone has
// looked at its maximum; a block whose 16 probabilities per lane add up to more than this (or
// to NaN / infinity) is done again after the reference has been moved.  Far inside bf16 and fp32.
constexpr float kOptimisticSum = 1048576.0f;      // 2^20: some probability above 2^16
// The next work item is claimed this many streamed 64-row tiles before the end of the current
// one: late enough that a workgroup cannot take items from workgroups that have not started,
// early enough that most of the claim's round trip hides under the item's last tiles.
constexpr int kClaimTilesAhead = 4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

#pragma clang diagnostic ignored "-Winline-asm"   // m0 is named as a clobber on purpose

// A tile of RS rows x D bf16 columns in LDS, natural order, rows of 2*D bytes, filled by a
// workgroup of NW waves with direct-to-LDS requests.  Chunk c (16 bytes) of row r sits at position
// c ^ swz(r).  swz is chosen so that (a) sixteen lanes reading the same chunk of sixteen
// consecutive rows and (b) sixteen lanes of a transposing read (four consecutive rows x 32
// bytes, two neighbouring groups 32 bytes apart) both touch every bank once.
template <int RS, int D, int NW>
struct LdsTile {
  static constexpr int ROWB = 2 * D;                 // bytes per row
  static constexpr int BYTES = RS * ROWB;
  static constexpr int RPI = 1024 / ROWB;            // rows per wave instruction (1 KB)
  static constexpr int NI = BYTES / 1024 / NW;       // wave instructions per wave (NW waves)
  static_assert(NI >= 1, "tile too small for the workgroup");

  __device__ static __forceinline__ int swz(int r) {
    if constexpr (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
    else return (((r >> 1) & 1) << 2) | (((r >> 3) & 1) << 1) | ((r >> 2) & 1);
  }

  // per wave instruction: byte offset of this lane's 16-byte chunk inside a matrix whose
  // rows are rs_bytes apart (row of the tile times the stride, plus the swizzled column)
  unsigned loff[NI];
  int wave_base;
  __device__ __forceinline__ void init(unsigned rs_bytes) {
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    wave_base = w * NI * 1024;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int byte = 16 * lane;
      const int row = (w * NI + j) * RPI + byte / ROWB, pos = (byte % ROWB) >> 4;
      loff[j] = (unsigned)row * rs_bytes + (unsigned)((pos ^ swz(row)) * 16);
    }
  }
  // rows row0 .. row0+RS-1 of the matrix described by `desc` -> LDS byte address dst, where
  // base = row0 * row stride + byte offset of the first column (uniform over the workgroup);
  // rows beyond the descriptor's range arrive as zeros.  The whole offset travels in the
  // vector operand: the scalar offset field of the instruction is not range-checked.
  __device__ __forceinline__ void issue(i32x4 desc, unsigned base, unsigned dst) const {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const unsigned off = loff[j] + base;
      // m0 = LDS address of lane 0's 16 bytes; lane l lands at m0 + 16*l.  Assembly, so that
      // the compiler's wait-count pass does not put a vmcnt(0) in front of every LDS read;
      // completion is waited for by hand before the barrier that publishes the tile.
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   : : "s"(dst + (unsigned)(wave_base + j * 1024)), "v"(off), "s"(desc) : "m0");
    }
  }
  // fragment whose contraction runs along the row: row `row`, columns 16*s + 8*hb .. +7
  __device__ static __forceinline__ bf16x8 nat(const lds_byte* t, int row, int s, int hb) {
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(t + row * ROWB + (((2 * s + hb) ^ swz(row)) << 4));
  }
  // fragment whose contraction runs across rows: for the lane that owns column 32*cblk + lr
  // of MFMA's first operand, rows kb + 4*hb + {0..3} and kb + 8 + 4*hb + {0..3} -- the eight
  // streamed indices a lane of half hb holds in registers 8*s2 .. 8*s2+7 of a 32x32
  // accumulator block when kb = block base + 16*s2
  __device__ static __forceinline__ bf16x8 tr(const lds_byte* t, int cblk, int kb) {
    const int lane = threadIdx.x & 63;
    const int G = lane >> 4, i = lane & 15, hh = G >> 1, q = i >> 2, g = i & 3;
    const int r0 = kb + 4 * hh + q, r1 = r0 + 8;
    const int ch = 4 * cblk + 2 * (G & 1) + (g >> 1);
    const lds_byte* p0 = t + r0 * ROWB + ((ch ^ swz(r0)) << 4) + (g & 1) * 8;
    const lds_byte* p1 = t + r1 * ROWB + ((ch ^ swz(r1)) << 4) + (g & 1) * 8;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
};

// descriptor of the rows of one (sample, head) slice: base pointer, no stride, bytes up to
// the end of the slice's last row, raw 32-bit format
__device__ __forceinline__ i32x4 slice_desc(const bf16* p, int64_t rows, int64_t rs, int D) {
  i32x4 d;
  d.x = (int)(uint32_t)(uintptr_t)p; d.y = (int)((uint32_t)((uintptr_t)p >> 32) & 0xffffu);
  d.z = (int)(uint32_t)(((rows - 1) * rs + D) * 2); d.w = 0x00020000;
  return d;
}
// vmcnt(N) alone: all but the newest N requests of this wave have landed
template <int N>
__device__ __forceinline__ void wait_requests() {
  static_assert(N < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// Streamed tiles live in a ring of NST stages; tile t+PD is requested at the start of step t
// (its stage was last read in step t-1) and tile t+1 is waited for before the barrier that
// ends step t.  Requests are issued for every step, past the last tile too (they point
// outside the descriptor and fetch nothing), so that the wait count is a constant.
template <int NW> struct Ring { static constexpr int NST = (NW == 8) ? 4 : 2, PD = NST - 1; };

// registers 8*s2 .. 8*s2+7 of an accumulator block as a bf16 B-operand
__device__ __forceinline__ bf16x8 pack8(const float* v) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
  return o;
}
// streamed index (within a 32-block) held by register r of a lane of half hb
__device__ __forceinline__ int acc_row(int r, int hb) { return 8 * (r >> 2) + 4 * hb + (r & 3); }

// Work order.  All query tiles of one (sample, head) stream the same K and V rows (all key
// tiles the same Q and dO rows), so they should run at the same time on the same XCD and
// meet in its L2: handed out head by head otherwise, 512 resident workgroups stream 512
// different heads and every tile comes from HBM (the forward kernel then moves ~4.4 GB per
// millisecond and is bandwidth-bound).  Items come from the work queue (tile_queue.h) in blocks
// of `hb` heads: a block belongs to the list of one XCD and the workgroups of that XCD draw its
// tiles one after another.  Tiles cost unequally under a causal mask.  Inside a block the
// items are ordered tile-major, costliest tile position first (heavy_last: the last tile is the
// costliest), all heads of the block for one position before the next position: drawn in that
// order by whichever workgroup is free, the light tiles fill the gaps the heavy ones leave
// (longest-first list scheduling).  The host sizes a block to about two rounds of an XCD's
// workgroups, so several tiles of every head of the block are in flight together.  Without a
// mask all tiles cost the same and hb = 1 keeps a head's tiles together.
// Under static rounds (equal-cost tiles, or too few items for the queue to pay) hb = 1 and
// `mirror` flips the position inside the head on odd rounds when a round covers whole heads,
// so that a workgroup that drew a heavy tile next draws a light one.
__device__ __forceinline__ void attn_item(int item, int heads, int tiles, int hb, bool heavy_last, bool mirror, int* head, int* tile) {
  if (mirror) heavy_last = !heavy_last;
  const int per = hb * tiles, blk = item / per, within = item - blk * per;
  const int h0 = blk * hb, hn = min(hb, heads - h0);        // the last block may hold fewer heads
  const int pos = within / hn;
  *head = h0 + within - pos * hn;
  *tile = heavy_last ? tiles - 1 - pos : pos;
}

__device__ __forceinline__ bool attn_mirror(const TileQueueArgs& q, const TileQueueCursor& c, int tiles) {
  return q.mode == TQ_ROUNDS && (c.round & 1) && ((gridDim.x & 7) == 0 ? (gridDim.x >> 3) : gridDim.x) % tiles == 0;
}

// --------------------------------------------------------------------------- forward
// value of the other half-wave's lane (lane ^ 32) combined with this lane's: one cross-half swap,
// no LDS round trip
__device__ __forceinline__ float xhalf_max(float v) {
  typedef __attribute__((ext_vector_type(2))) unsigned u32x2_;
  const unsigned x = __builtin_bit_cast(unsigned, v);
  const u32x2_ r = __builtin_amdgcn_permlane32_swap(x, x, false, false);   // r[0] = lower half's value, r[1] = upper half's, in every lane
  return fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, r[1]));
}

// The key blocks of 32 are taken through a software pipeline that is skewed by one block, so
// that the three things a block needs run at the same time for three consecutive blocks:
// in slot i the matrix cores compute the scores of block i+1 (S = K Q^T) and add block i-1 to
// the output (O^T += V^T P^T) while the vector ALU turns the scores of block i into
// probabilities.  Inside one wave instructions issue in order, and a matrix instruction holds
// the matrix pipe for 32 cycles during which only instructions that follow it in program order
// can issue: the slot is therefore written, and pinned with scheduling barriers, as one matrix
// instruction, the read of an operand a few instructions ahead, a few vector instructions, and
// so on.  The arithmetic per block is that of the plain loop: scores, reference, probabilities,
// output, block by block in ascending order.
//
// LDS: a step covers two slots and reads the K rows of tile u+1 and the V rows of tile u (64
// keys each); these share a stage, two stages alternate, and the next step's rows are
// requested at the start of a step (their stage was last read in the step before).
template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_fwd_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ O,
                                                     float* __restrict__ lse, int B, int N, int H, int Hkv, int causal,
                                                     float scale_log2, int qtiles, int hblk, TileQueueArgs tq) {
  constexpr int RS = 64, NS = D / 16, NC = D / 32;
  typedef LdsTile<RS, D, NW> L;
  constexpr int STAGE = 2 * L::BYTES;                      // K rows of one tile | V rows of the tile before
  constexpr int QT = 32 * NW;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const lds_byte* smem = (const lds_byte*)smem_raw;        // [2][STAGE]
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  L ld;
  ld.init((unsigned)((H + 2 * Hkv) * D * 2));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * D, ko = H * D, vo = (H + Hkv) * D, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * D;
  __shared__ int mail;
  TileQueueCursor qc;
  int item = tq_first(tq, qc, &mail);
  while (item >= 0) {
    int head_, qt;
    attn_item(item, B * H, qtiles, hblk, causal != 0, attn_mirror(tq, qc, qtiles), &head_, &qt);
    const int hd = head_ % H, b = head_ / H;
    const int q0 = qt * QT, i0 = q0 + 32 * wave, i = i0 + lr;
    const bf16* rowb = qkv + (int64_t)b * N * rs;
    const bf16* base = rowb + hd * D;
    const int kvh = hd / GQ;
    bf16x8 qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (i < N) qf[s] = *reinterpret_cast<const bf16x8*>(base + (int64_t)i * rs + 16 * s + 8 * hb);
      else { for (int e = 0; e < 8; ++e) qf[s][e] = (bf16)0.f; }
    }
    f32x16 o[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[c][e] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const int kv_end = causal ? min(N, q0 + QT) : N;
    const int nt = (kv_end + RS - 1) / RS;                 // key tiles the workgroup streams
    // key blocks this wave multiplies: up to the end of the keys and, under a causal mask, up
    // to the block that holds its own diagonal; only the last of them can need the mask
    int nb = (kv_end + 31) / 32;
    if (causal) nb = min(nb, i0 / 32 + 1);
    const i32x4 dk_ = slice_desc(rowb + ko + kvh * D, N, rs, D), dv_ = slice_desc(rowb + vo + kvh * D, N, rs, D);
    const unsigned rsb = (unsigned)(rs * 2);
    auto request = [&](int u) {            // step u: K rows of tile u+1, V rows of tile u; tiles that do not exist point outside the slice
      const unsigned nbuf = lds0 + (unsigned)(((u + 1) & 1) * STAGE);
      const int krow = (u + 1 < nt) ? (u + 1) * RS : N;
      const int vrow = (u >= 0 && u < nt) ? u * RS : N;
      ld.issue(dk_, (unsigned)krow * rsb, nbuf);
      ld.issue(dv_, (unsigned)vrow * rsb, nbuf + L::BYTES);
    };
    __syncthreads();                      // previous item's readers are done with both stages
    request(-1);
    wait_requests<0>();
    __syncthreads();
    unsigned entry = 0;
    const int claim_at = nt > kClaimTilesAhead ? nt - kClaimTilesAhead : -1;
    f32x16 sc;                            // raw scores of the block whose probabilities are formed next
    bf16x8 pk0, pk1;                      // probabilities of the block whose output product is pending
#pragma unroll
    for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { pk0[e] = (bf16)0.f; pk1[e] = (bf16)0.f; }
    for (int u = -1; u < nt; ++u) {
      const lds_byte* ks = smem + ((u + 1) & 1) * STAGE;
      const lds_byte* vs = ks + L::BYTES;
      request(u + 1);
      if (u == claim_at) entry = tq_claim_ahead(tq, qc);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int bi = 2 * u + 1 + half;                  // the block whose probabilities this slot forms
        const bool do_s = bi + 1 < nb, do_x = bi >= 0 && bi < nb, do_pv = bi >= 1 && bi - 1 < nb;
        const int krow = 32 * half + lr, vrow = 32 * half;
        // o += V^T P^T for the pending block, one instruction after the other
        auto add_pv_now = [&]() {
#pragma unroll
          for (int c = 0; c < NC; ++c) {
            o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::tr(vs, c, vrow), pk0, o[c], 0, 0, 0);
            o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::tr(vs, c, vrow + 16), pk1, o[c], 0, 0, 0);
          }
        };
        // moves the reference of the running sums to the new row maximum
        auto rescale = [&](float mx) {
          const float mn = fmaxf(m, mx);
          const float mref0 = (mn == -INFINITY) ? 0.f : mn;
          const float corr = fast_exp2(m - mref0);               // m = -inf -> 0
          lsum *= corr;
#pragma unroll
          for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[c][e] *= corr;
          m = mn;
        };
        if (bi >= 1 && bi + 1 < nb) {
          // steady state: all three present, block bi is not the last one, so nothing is masked.
          // The probabilities are formed against the reference the row already has, without
          // looking at the block's maximum first; the reference is moved afterwards, and the
          // block's probabilities formed again, only if their sum shows that they have grown
          // beyond kOptimisticSum (rare: the reference then lags the row maximum by more than
          // sixteen powers of two).
          const float mref = (m == -INFINITY) ? 0.f : m;
          // Slot by slot: the matrix instruction, the read of the operand PFD slots ahead, and a
          // share of the vector work, which runs while the matrix instruction holds its pipe.
          // Score and output products alternate, so no instruction waits for the one just issued.
          constexpr int NM = NS + 2 * NC, PFD = 3, XPS = 16 / NM;   // NS == 2 * NC for both head sizes
          static_assert(NS == 2 * NC && 16 % NM == 0, "slots alternate score and output products");
          auto operand = [&](int k) -> bf16x8 {                  // k even: K fragment k/2; k odd: V fragment of output block k/4, key half (k/2)%2
            const int q = k >> 1;
            return (k & 1) ? L::tr(vs, q >> 1, vrow + 16 * (q & 1)) : L::nat(ks, krow, q, hb);
          };
          bf16x8 opb[PFD + 1];
#pragma unroll
          for (int k = 0; k < PFD; ++k) opb[k] = operand(k);
          f32x16 sn;
#pragma unroll
          for (int e = 0; e < 16; ++e) sn[e] = 0.f;
          float sv[16];
          float ps = 0.f;
          bf16x8 pn0, pn1;
          // the first operands are on their way: the vector work of the first slots runs now,
          // under their latency, instead of under matrix instructions that cannot start yet
          auto prob = [&](int k) {
#pragma unroll
            for (int x = 0; x < XPS; ++x) {
              const int r = k * XPS + x;
              sv[r] = fast_exp2(fmaf(sc[r], scale_log2, -mref));
              ps += sv[r];
            }
          };
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int k = 0; k < PFD; ++k) prob(k);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int k = 0; k < NM; ++k) {
            if (k + PFD < NM) opb[(k + PFD) % (PFD + 1)] = operand(k + PFD);
            const bf16x8 a = opb[k % (PFD + 1)];
            const int q = k >> 1;
            if (k & 1) o[q >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, (q & 1) ? pk1 : pk0, o[q >> 1], 0, 0, 0);
            else sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[q], sn, 0, 0, 0);
            if (k + PFD < NM) prob(k + PFD);
            if ((k + PFD + 1) * XPS == 8) pn0 = pack8(sv);
            if (k + PFD == NM - 1) pn1 = pack8(sv + 8);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (__any(!(ps <= kOptimisticSum))) {
            // o holds every block before bi now (the pending product has just been added)
            float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
            for (int r = 2; r < 16; ++r) mx = fmaxf(mx, sc[r]);
            rescale(xhalf_max(mx) * scale_log2);
            ps = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { sv[r] = fast_exp2(fmaf(sc[r], scale_log2, -m)); ps += sv[r]; }
            pn0 = pack8(sv); pn1 = pack8(sv + 8);
          }
          lsum += ps;
          sc = sn; pk0 = pn0; pk1 = pn1;
        } else if (do_s || do_x || do_pv) {
          // first and last slots of the wave: whatever of the three exists, one after the other
          const int jb = 32 * bi;
          float sv[16];
          bool pv_done = !do_pv;
          if (do_x) {
            float mx = -INFINITY;
            if ((jb + 32 > N) || (causal && jb + 31 > i0)) {     // block touches the diagonal or the end of the keys
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int j = jb + acc_row(r, hb);
                const bool masked = (j >= N) || (causal && j > i);
                sv[r] = masked ? -INFINITY : sc[r];
                mx = fmaxf(mx, sv[r]);
              }
            } else {
#pragma unroll
              for (int r = 0; r < 16; ++r) { sv[r] = sc[r]; mx = fmaxf(mx, sv[r]); }
            }
            mx = xhalf_max(mx) * scale_log2;                     // scale > 0: max commutes with it
            if (__any(mx > m + kLazyRescale)) {
              if (!pv_done) { add_pv_now(); pv_done = true; }   // o must hold every block before bi when it is rescaled
              rescale(mx);
            }
          }
          if (!pv_done) add_pv_now();
          if (do_x) {
            const float mref = (m == -INFINITY) ? 0.f : m;       // row with nothing visible yet
            float ps = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { sv[r] = fast_exp2(fmaf(sv[r], scale_log2, -mref)); ps += sv[r]; }
            lsum += ps;
            pk0 = pack8(sv); pk1 = pack8(sv + 8);
          }
          if (do_s) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
            for (int s = 0; s < NS; ++s) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::nat(ks, krow, s, hb), qf[s], sc, 0, 0, 0);
          }
        }
      }
      wait_requests<0>();                  // this wave's share of the next step's rows has landed
      __syncthreads();
    }
    const float ltot = lsum + __shfl_xor(lsum, 32, 64);
    if (i < N) {
      const float inv = 1.0f / ltot;
      bf16* orow = O + ((int64_t)b * N + i) * h + hd * D;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[c][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * c + 8 * g + 4 * hb) = v;
        }
      if (hb == 0) lse[((int64_t)b * H + hd) * N + i] = (m + log2f(ltot)) * kLn2;
    }
    item = tq_next(tq, qc, entry, &mail);
  }
  tq_done(tq);
}

// Forward kernel for head size 64, one key tile of 64 at a time: with four matrix instructions
// per score block the loop is bound by the vector ALU, not by the matrix cores, and three
// resident workgroups per CU (about 155 registers) serve it better than the skewed pipeline
// above, which needs about 190 (measured: 149 against 159 us at B8 N1500 H20, 25.6 against
// 27.7 us at B8 N576 H16).  Both blocks of a tile are multiplied before the first block's
// probabilities are formed, so the second block's scores are on the matrix cores meanwhile.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_fwd_tile_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ O,
                                                     float* __restrict__ lse, int B, int N, int H, int Hkv, int causal,
                                                     float scale_log2, int qtiles, int hblk, TileQueueArgs tq) {
  constexpr int RS = 64, NS = D / 16, NC = D / 32;
  typedef LdsTile<RS, D, NW> L;
  constexpr int STAGE = 2 * L::BYTES;                      // K | V
  constexpr int NST = Ring<NW>::NST, PD = Ring<NW>::PD, QT = 32 * NW, NREQ = 2 * L::NI;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const lds_byte* smem = (const lds_byte*)smem_raw;        // [NST][STAGE]
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  L ld;
  ld.init((unsigned)((H + 2 * Hkv) * D * 2));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * D, ko = H * D, vo = (H + Hkv) * D, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * D;
  __shared__ int mail;
  TileQueueCursor qc;
  int item = tq_first(tq, qc, &mail);
  while (item >= 0) {
    int head_, qt;
    attn_item(item, B * H, qtiles, hblk, causal != 0, attn_mirror(tq, qc, qtiles), &head_, &qt);
    const int hd = head_ % H, b = head_ / H;
    const int q0 = qt * QT, i0 = q0 + 32 * wave, i = i0 + lr;
    const bf16* rowb = qkv + (int64_t)b * N * rs;
    const bf16* base = rowb + hd * D;
    const int kvh = hd / GQ;
    bf16x8 qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (i < N) qf[s] = *reinterpret_cast<const bf16x8*>(base + (int64_t)i * rs + 16 * s + 8 * hb);
      else { for (int e = 0; e < 8; ++e) qf[s][e] = (bf16)0.f; }
    }
    f32x16 o[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[c][e] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const int kv_end = causal ? min(N, q0 + QT) : N;
    const int ntiles = (kv_end + RS - 1) / RS;
    const i32x4 dk_ = slice_desc(rowb + ko + kvh * D, N, rs, D), dv_ = slice_desc(rowb + vo + kvh * D, N, rs, D);
    const unsigned rsb = (unsigned)(rs * 2);
    auto request = [&](int tile) {         // tiles past the last one point outside the slice
      const unsigned nb = lds0 + (unsigned)((tile % NST) * STAGE);
      const int row0 = tile < ntiles ? tile * RS : N;
      const unsigned at = (unsigned)row0 * rsb;
      ld.issue(dk_, at, nb);
      ld.issue(dv_, at, nb + L::BYTES);
    };
    __syncthreads();                      // previous item's readers are done with every stage
#pragma unroll
    for (int u = 0; u < PD; ++u) request(u);
    wait_requests<(PD - 1) * NREQ>();
    __syncthreads();
    unsigned entry = 0;
    const int claim_at = ntiles > kClaimTilesAhead ? ntiles - kClaimTilesAhead : 0;
    for (int t = 0; t < ntiles; ++t) {
      const lds_byte* ks = smem + (t % NST) * STAGE;
      const lds_byte* vs = ks + L::BYTES;
      request(t + PD);
      if (t == claim_at) entry = tq_claim_ahead(tq, qc);
      const int j0 = t * RS;
      // A 32-key block is visible to this wave when it starts before the end of the keys and
      // (causal) not after the wave's last query; the second block of a tile is visible only
      // if the first is.
      auto visible = [&](int jb) { return jb < kv_end && !(causal && jb > i0 + 31); };
      // online-softmax update with one block of scores (raw dot products, this lane's query
      // against 16 keys): returns the probabilities as two B-operands
      auto softmax_block = [&](const f32x16& sacc, int jb, bf16x8& p0, bf16x8& p1) {
        float sv[16];
        float mx = -INFINITY;
        // only blocks that touch the diagonal or the end of the sequence need the mask
        const bool need_mask = (jb + 32 > N) || (causal && jb + 31 > i0);
        if (need_mask) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jb + acc_row(r, hb);
            const bool masked = (j >= N) || (causal && j > i);
            sv[r] = masked ? -INFINITY : sacc[r];
            mx = fmaxf(mx, sv[r]);
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) { sv[r] = sacc[r]; mx = fmaxf(mx, sv[r]); }
        }
        mx = xhalf_max(mx) * scale_log2;                           // scale > 0: max commutes with it
        const float mn = fmaxf(m, mx);
        if (__any(mx > m + kLazyRescale)) {
          const float mref0 = (mn == -INFINITY) ? 0.f : mn;
          const float corr = fast_exp2(m - mref0);               // m = -inf -> 0
          lsum *= corr;
#pragma unroll
          for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[c][e] *= corr;
          m = mn;
        }
        const float mref = (m == -INFINITY) ? 0.f : m;           // row with nothing visible yet
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sv[r] = fast_exp2(fmaf(sv[r], scale_log2, -mref)); ps += sv[r]; }
        lsum += ps;
        p0 = pack8(sv); p1 = pack8(sv + 8);
      };
      auto scores = [&](const bf16x8* kfr) {
        f32x16 sacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[s], qf[s], sacc, 0, 0, 0);
        return sacc;
      };
      auto add_pv = [&](const bf16x8 (*vfr)[2], const bf16x8& p0, const bf16x8& p1) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[c][0], p0, o[c], 0, 0, 0);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[c][1], p1, o[c], 0, 0, 0);
        }
      };
      if (visible(j0) && visible(j0 + 32)) {
        // Both blocks: the scores of the second block are on the matrix cores while the
        // first block's softmax runs on the vector ALU, and the first block's P V product
        // runs under the second block's softmax.  Fragment reads are issued a phase ahead.
        bf16x8 kfa[NS], kfb[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) kfa[s] = L::nat(ks, lr, s, hb);
#pragma unroll
        for (int s = 0; s < NS; ++s) kfb[s] = L::nat(ks, 32 + lr, s, hb);
        __builtin_amdgcn_sched_barrier(0);
        const f32x16 sa = scores(kfa);
        const f32x16 sb = scores(kfb);
        bf16x8 vfa[NC][2];
#pragma unroll
        for (int c = 0; c < NC; ++c) { vfa[c][0] = L::tr(vs, c, 0); vfa[c][1] = L::tr(vs, c, 16); }
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 p0, p1;
        softmax_block(sa, j0, p0, p1);
        bf16x8 vfb[NC][2];
#pragma unroll
        for (int c = 0; c < NC; ++c) { vfb[c][0] = L::tr(vs, c, 32); vfb[c][1] = L::tr(vs, c, 48); }
        add_pv(vfa, p0, p1);
        __builtin_amdgcn_sched_barrier(0);
        softmax_block(sb, j0 + 32, p0, p1);
        add_pv(vfb, p0, p1);
      } else if (visible(j0)) {
        bf16x8 kfr[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) kfr[s] = L::nat(ks, lr, s, hb);
        __builtin_amdgcn_sched_barrier(0);
        const f32x16 sa = scores(kfr);
        bf16x8 vfr[NC][2];
#pragma unroll
        for (int c = 0; c < NC; ++c) { vfr[c][0] = L::tr(vs, c, 0); vfr[c][1] = L::tr(vs, c, 16); }
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 p0, p1;
        softmax_block(sa, j0, p0, p1);
        add_pv(vfr, p0, p1);
      }
      wait_requests<(PD - 1) * NREQ>();    // this wave's share of the next tile has landed
      __syncthreads();
    }
    const float ltot = lsum + __shfl_xor(lsum, 32, 64);
    if (i < N) {
      const float inv = 1.0f / ltot;
      bf16* orow = O + ((int64_t)b * N + i) * h + hd * D;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[c][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * c + 8 * g + 4 * hb) = v;
        }
      if (hb == 0) lse[((int64_t)b * H + hd) * N + i] = (m + log2f(ltot)) * kLn2;
    }
    item = tq_next(tq, qc, entry, &mail);
  }
  tq_done(tq);
}

// ------------------------------------------------------------------------------- dQ
template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_bwd_dq_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ O,
                                                        const bf16* __restrict__ dO,
                                                        const float* __restrict__ lse, float* __restrict__ delta,
                                                        bf16* __restrict__ dqkv, int B, int N, int H, int Hkv, int causal,
                                                        float scale, int qtiles, int hblk, TileQueueArgs tq) {
  constexpr int RS = 64, NS = D / 16, NC = D / 32;
  typedef LdsTile<RS, D, NW> L;
  constexpr int STAGE = 2 * L::BYTES;                      // K | V
  constexpr int NST = Ring<NW>::NST, PD = Ring<NW>::PD, QT = 32 * NW, NREQ = 2 * L::NI;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const lds_byte* smem = (const lds_byte*)smem_raw;        // [NST][STAGE]
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  L ld;
  ld.init((unsigned)((H + 2 * Hkv) * D * 2));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * D, ko = H * D, vo = (H + Hkv) * D, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * D;
  const float scale_log2 = scale * kLog2e;
  __shared__ int mail;
  TileQueueCursor qc;
  int item = tq_first(tq, qc, &mail);
  while (item >= 0) {
    int head_, qt;
    attn_item(item, B * H, qtiles, hblk, causal != 0, attn_mirror(tq, qc, qtiles), &head_, &qt);
    const int hd = head_ % H, b = head_ / H;
    const int q0 = qt * QT, i0 = q0 + 32 * wave, i = i0 + lr;
    const bf16* rowb = qkv + (int64_t)b * N * rs;
    const bf16* base = rowb + hd * D;
    const int kvh = hd / GQ;
    const bf16* dob = dO + (int64_t)b * N * h + hd * D;
    const bf16* ob = O + (int64_t)b * N * h + hd * D;
    bf16x8 qf[NS], dof[NS];
    // delta_i = sum_c dO[i][c] * O[i][c] of this wave's rows is formed here, from the dO
    // fragments the wave holds anyway (a lane covers half of the columns, the other half
    // sits 32 lanes away), and stored for the dK/dV kernel, which runs after this one
    float dlt = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (i < N) {
        qf[s] = *reinterpret_cast<const bf16x8*>(base + (int64_t)i * rs + 16 * s + 8 * hb);
        dof[s] = *reinterpret_cast<const bf16x8*>(dob + (int64_t)i * h + 16 * s + 8 * hb);
        const bf16x8 of = *reinterpret_cast<const bf16x8*>(ob + (int64_t)i * h + 16 * s + 8 * hb);
#pragma unroll
        for (int e = 0; e < 8; ++e) dlt = fmaf((float)dof[s][e], (float)of[e], dlt);
      } else {
        for (int e = 0; e < 8; ++e) { qf[s][e] = (bf16)0.f; dof[s][e] = (bf16)0.f; }
      }
    }
    dlt += __shfl_xor(dlt, 32, 64);
    if (i < N && hb == 0) delta[((int64_t)b * H + hd) * N + i] = dlt;
    const float lse2 = (i < N) ? lse[((int64_t)b * H + hd) * N + i] * kLog2e : 0.f;
    f32x16 dq[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[c][e] = 0.f;
    const int kv_end = causal ? min(N, q0 + QT) : N;
    const int ntiles = (kv_end + RS - 1) / RS;
    const i32x4 dk_ = slice_desc(rowb + ko + kvh * D, N, rs, D), dv_ = slice_desc(rowb + vo + kvh * D, N, rs, D);
    const unsigned rsb = (unsigned)(rs * 2);
    auto request = [&](int tile) {
      const unsigned nb = lds0 + (unsigned)((tile % NST) * STAGE);
      const int row0 = tile < ntiles ? tile * RS : N;
      const unsigned at = (unsigned)row0 * rsb;
      ld.issue(dk_, at, nb);
      ld.issue(dv_, at, nb + L::BYTES);
    };
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PD; ++u) request(u);
    wait_requests<(PD - 1) * NREQ>();
    __syncthreads();
    unsigned entry = 0;
    const int claim_at = ntiles > kClaimTilesAhead ? ntiles - kClaimTilesAhead : 0;
    for (int t = 0; t < ntiles; ++t) {
      const lds_byte* ks = smem + (t % NST) * STAGE;
      const lds_byte* vs = ks + L::BYTES;
      request(t + PD);
      if (t == claim_at) entry = tq_claim_ahead(tq, qc);
      const int j0 = t * RS;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int jb = j0 + 32 * sub;
        if (jb >= kv_end || (causal && jb > i0 + 31)) continue;
        f32x16 sacc, pacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
        // The K and V fragments are read two MFMA pairs ahead of their use (the scheduling
        // barriers keep that distance): read right in front of the MFMA that consumes it, a
        // fragment costs the wave a full LDS round trip per pair.
        constexpr int PF = 2;
        bf16x8 kfr[NS], vfr[NS];
#pragma unroll
        for (int s = 0; s < PF; ++s) {
          kfr[s] = L::nat(ks, 32 * sub + lr, s, hb);
          vfr[s] = L::nat(vs, 32 * sub + lr, s, hb);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          if (s + PF < NS) {
            kfr[s + PF] = L::nat(ks, 32 * sub + lr, s + PF, hb);
            vfr[s + PF] = L::nat(vs, 32 * sub + lr, s + PF, hb);
          }
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[s], qf[s], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[s], dof[s], pacc, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        // the transposed K fragments of the first two dQ column blocks are on their way while
        // the probabilities are formed
        bf16x8 ta[NC], tb[NC];
#pragma unroll
        for (int c = 0; c < (NC < 2 ? NC : 2); ++c) { ta[c] = L::tr(ks, c, 32 * sub); tb[c] = L::tr(ks, c, 32 * sub + 16); }
        __builtin_amdgcn_sched_barrier(0);
        // only blocks that touch the diagonal or the end of the sequence need the mask: a
        // masked score becomes -inf, so its recomputed probability is exactly 0
        if ((jb + 32 > N) || (i0 + 32 > N) || (causal && jb + 31 > i0)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jb + acc_row(r, hb);
            if ((j >= N) || (i >= N) || (causal && j > i)) sacc[r] = -INFINITY;
          }
        }
        float ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) ds[r] = fast_exp2(fmaf(sacc[r], scale_log2, -lse2)) * (pacc[r] - dlt);
        const bf16x8 d0 = pack8(ds), d1 = pack8(ds + 8);
        __builtin_amdgcn_sched_barrier(0);
        // each accumulator takes its two products in the same order as before (k-half 0, then
        // k-half 1); the halves of different column blocks alternate, so no MFMA waits for
        // the one issued just before it
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          if (c + 2 < NC) { ta[c + 2] = L::tr(ks, c + 2, 32 * sub); tb[c + 2] = L::tr(ks, c + 2, 32 * sub + 16); }
          dq[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta[c], d0, dq[c], 0, 0, 0);
          if (c > 0) dq[c - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tb[c - 1], d1, dq[c - 1], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        dq[NC - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tb[NC - 1], d1, dq[NC - 1], 0, 0, 0);
      }
      wait_requests<(PD - 1) * NREQ>();
      __syncthreads();
    }
    if (i < N) {
      bf16* out = dqkv + ((int64_t)b * N + i) * rs + hd * D;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[c][4 * g + e] * scale);
          *reinterpret_cast<bf16x4*>(out + 32 * c + 8 * g + 4 * hb) = v;
        }
    }
    item = tq_next(tq, qc, entry, &mail);
  }
  tq_done(tq);
}

// --------------------------------------------------------------------------- dK, dV
template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_bwd_dkv_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dqkv, int B, int N, int H, int Hkv, int causal,
                                                         float scale, int ktiles, int hblk, TileQueueArgs tq) {
  constexpr int RS = 32, NS = D / 16, NC = D / 32;
  typedef LdsTile<RS, D, NW> L;
  constexpr int STAGE = 2 * L::BYTES;                      // Q | dO
  constexpr int NST = Ring<NW>::NST, PD = Ring<NW>::PD, KT = 32 * NW, NREQ = 2 * L::NI + 2;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const lds_byte* smem = (const lds_byte*)smem_raw;        // [NST][STAGE]
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  // the V rows of the owned keys stay in LDS for the whole item (as registers they would
  // push the kernel past its register budget and into scratch)
  typedef LdsTile<KT, D, NW> LV;
  const lds_byte* vblk = smem + NST * STAGE;
  const float* stat = reinterpret_cast<const float*>(smem_raw + NST * STAGE + LV::BYTES);  // [NST][2][64]: lse, delta
  L ld, ldo;           // lane offsets for the two row strides: q rows and dO rows
  ld.init((unsigned)((H + 2 * Hkv) * D * 2));
  ldo.init((unsigned)(H * D * 2));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * D, ko = H * D, vo = (H + Hkv) * D, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * D;
  const float scale_log2 = scale * kLog2e;
  __shared__ int mail;
  TileQueueCursor qc;
  int item = tq_first(tq, qc, &mail);
  while (item >= 0) {
    int head_, kt_i;
    attn_item(item, B * Hkv, ktiles, hblk, false, attn_mirror(tq, qc, ktiles), &head_, &kt_i);      // the first key tile has the most queries
    const int kvh = head_ % Hkv, b = head_ / Hkv;
    const int hd0 = kvh * GQ;                    // first query head of the group
    const int k0 = kt_i * KT, j0w = k0 + 32 * wave, j = j0w + lr;
    const bf16* rowb = qkv + (int64_t)b * N * rs;
    const bf16* base = rowb + hd0 * D;           // q columns of the group's heads are adjacent
    const bf16* dob = dO + (int64_t)b * N * h + hd0 * D;
    const float* lse_b = lse + ((int64_t)b * H + hd0) * N;
    const float* del_b = delta + ((int64_t)b * H + hd0) * N;
    bf16x8 kf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (j < N) kf[s] = *reinterpret_cast<const bf16x8*>(rowb + ko + kvh * D + (int64_t)j * rs + 16 * s + 8 * hb);
      else { for (int e = 0; e < 8; ++e) kf[s][e] = (bf16)0.f; }
    }
    f32x16 dk[NC], dv[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) { dk[c][e] = 0.f; dv[c][e] = 0.f; }
    const int q_begin = causal ? (k0 / RS) * RS : 0;
    const int ntq = (N - q_begin + RS - 1) / RS;       // query tiles of one head
    const int ntiles = ntq * GQ;                         // streamed for every query head of the group in turn
    // per-row statistics of streamed tile `tile` (lse, delta) take the same road as the tiles:
    // one 4-byte request per lane straight into the tile's stage slot.  Every wave issues
    // them (same values, same place) so that all waves count the same number of requests.
    auto desc_f32 = [&](const float* p) {
      i32x4 d;
      d.x = (int)(uint32_t)(uintptr_t)p; d.y = (int)((uint32_t)((uintptr_t)p >> 32) & 0xffffu);
      d.z = GQ * N * 4; d.w = 0x00020000;
      return d;
    };
    const i32x4 dl_ = desc_f32(lse_b), dd_ = desc_f32(del_b);
    // one descriptor spans the group's GQ adjacent heads; the head is a column offset
    const i32x4 dq_ = slice_desc(base, N, rs, GQ * D), do_ = slice_desc(dob, N, h, GQ * D);
    const unsigned rsb = (unsigned)(rs * 2), hsb = (unsigned)(h * 2);
    // Tiles are requested in order and the position of the next one advances by increments
    // instead of a division per request (tile -> head, block): 35 of the loop's 420
    // instructions (0.5 - 1 % of the kernel's time: the loop waits on LDS more than it issues).
    int rq_t = 0, rq_g = 0, rq_row = q_begin, rq_left = ntq;       // next tile: number, head, first row, blocks left in the head
    auto request_next = [&]() {
      const bool real = rq_t < ntiles;
      const unsigned nb = lds0 + (unsigned)((rq_t % NST) * STAGE);
      const int row0 = real ? rq_row : N;
      const unsigned col = real ? (unsigned)(rq_g * D * 2) : 0u;
      ld.issue(dq_, (unsigned)row0 * rsb + col, nb);
      ldo.issue(do_, (unsigned)row0 * hsb + col, nb + L::BYTES);
      const unsigned off = (real && lane < RS && rq_row + lane < N) ? (unsigned)(rq_g * N + rq_row + lane) * 4u : 0xFFFFFFF0u;
      const unsigned dst = lds0 + (unsigned)(NST * STAGE + LV::BYTES + (rq_t % NST) * 2 * 64 * 4);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds" : : "s"(dst), "v"(off), "s"(dl_) : "m0");
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds" : : "s"(dst + 256u), "v"(off), "s"(dd_) : "m0");
      ++rq_t;
      rq_row += RS;
      if (--rq_left == 0) { rq_left = ntq; rq_row = q_begin; ++rq_g; }
    };
    __syncthreads();
    {
      LV ldv;            // built here so that its per-lane offsets do not live across the tile loop
      ldv.init(rsb);
      ldv.issue(slice_desc(rowb + vo + kvh * D, N, rs, D), (unsigned)k0 * rsb, lds0 + NST * STAGE);
    }
#pragma unroll
    for (int u = 0; u < PD; ++u) request_next();
    wait_requests<(PD - 1) * NREQ>();
    __syncthreads();
    unsigned entry = 0;
    const int claim_at = ntiles > 2 * kClaimTilesAhead ? ntiles - 2 * kClaimTilesAhead : 0;   // tiles of 32 rows here
    int ib = q_begin, ib_left = ntq;                   // first query row of block t, blocks left in its head
    for (int t = 0; t < ntiles; ++t) {
      const int slot = t % NST;
      const lds_byte* qs = smem + slot * STAGE;
      const lds_byte* dos = qs + L::BYTES;
      const float* sl = stat + (slot * 2 + 0) * 64;
      const float* sd = stat + (slot * 2 + 1) * 64;
      request_next();                                  // block t + PD
      if (t == claim_at) entry = tq_claim_ahead(tq, qc);
      if (!(causal && ib + 31 < j0w) && j0w < N) {            // otherwise every (i, j) here is masked
        if constexpr (D == 128) {
          // at head size 128 the accumulators (128 registers), the K fragments (32) and the two
          // score blocks leave no room for operand buffers: reads stay next to their use and the
          // other wave of the SIMD covers their latency (with a lookahead the kernel spilled
          // into scratch inside this loop and ran 9 % slower)
          f32x16 sacc, pacc;
#pragma unroll
          for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::nat(qs, lr, s, hb), kf[s], sacc, 0, 0, 0);
            pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::nat(dos, lr, s, hb), LV::nat(vblk, 32 * wave + lr, s, hb), pacc, 0, 0, 0);
          }
          // only blocks that touch the diagonal or the end of the sequence need the mask: a
          // masked score becomes -inf, so its recomputed probability is exactly 0
          if ((ib + 32 > N) || (j0w + 32 > N) || (causal && j0w + 31 > ib)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int gi = ib + acc_row(r, hb);
              if ((gi >= N) || (j >= N) || (causal && j > gi)) sacc[r] = -INFINITY;
            }
          }
          // registers 4g .. 4g+3 of a lane hold query rows 8g + 4*hb + {0..3}: their statistics
          // are four consecutive floats, one 16-byte LDS read each
          float pv[16], ds[16];
          const float4* sl4 = reinterpret_cast<const float4*>(sl + 4 * hb);
          const float4* sd4 = reinterpret_cast<const float4*>(sd + 4 * hb);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 l4 = sl4[2 * g], d4 = sd4[2 * g];
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int r = 4 * g + e;
              const float p = fast_exp2(fmaf(sacc[r], scale_log2, -lv[e] * kLog2e));
              pv[r] = p;
              ds[r] = p * (pacc[r] - dv4[e]);
            }
          }
          const bf16x8 p0 = pack8(pv), p1 = pack8(pv + 8), d0 = pack8(ds), d1 = pack8(ds + 8);
          // From here on S, dP and the unpacked P and dS are dead: their registers hold a ring of
          // transposed fragments read DKV_PF matrix instructions ahead (left to itself the compiler
          // reads every fragment into the same four registers right in front of its instruction).
          // Product w of 4 * NC: column block w / 4; w % 4 = 0: dV, keys half 0; 1: dK, half 0;
          // 2: dV, half 1; 3: dK, half 1 (each accumulator takes half 0 first, as before).
          constexpr int PF = DKV_PF;
          auto tr_operand = [&](int w) -> bf16x8 {
            const int c = w >> 2, part = w & 3;
            return L::tr((part & 1) ? qs : dos, c, 16 * (part >> 1));
          };
          bf16x8 ta[PF + 1];
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int w = 0; w < PF; ++w) ta[w] = tr_operand(w);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int w = 0; w < 4 * NC; ++w) {
            if (w + PF < 4 * NC) ta[(w + PF) % (PF + 1)] = tr_operand(w + PF);
            const int c = w >> 2, part = w & 3;
            const bf16x8 a = ta[w % (PF + 1)];
            if (part == 0) dv[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p0, dv[c], 0, 0, 0);
            else if (part == 1) dk[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, d0, dk[c], 0, 0, 0);
            else if (part == 2) dv[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p1, dv[c], 0, 0, 0);
            else dk[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, d1, dk[c], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        } else {
          // Operands come from LDS a fixed number of matrix instructions ahead of their use (a
          // read issued right in front of the instruction that needs it costs the wave a whole
          // LDS round trip per instruction); scheduling barriers keep that distance.
          constexpr int PF = 2, PFS = 2;
          f32x16 sacc, pacc;
#pragma unroll
          for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
          if constexpr (PFS > 0) {
            bf16x8 qa[PFS + 1], da[PFS + 1], va[PFS + 1];       // Q, dO and V fragments of contraction step s in slot s % (PFS + 1)
#pragma unroll
            for (int s = 0; s < PFS; ++s) {
              qa[s] = L::nat(qs, lr, s, hb); da[s] = L::nat(dos, lr, s, hb); va[s] = LV::nat(vblk, 32 * wave + lr, s, hb);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              if (s + PFS < NS) {
                const int n = (s + PFS) % (PFS + 1);
                qa[n] = L::nat(qs, lr, s + PFS, hb); da[n] = L::nat(dos, lr, s + PFS, hb); va[n] = LV::nat(vblk, 32 * wave + lr, s + PFS, hb);
              }
              sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s % (PFS + 1)], kf[s], sacc, 0, 0, 0);
              pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da[s % (PFS + 1)], va[s % (PFS + 1)], pacc, 0, 0, 0);
              __builtin_amdgcn_sched_barrier(0);
            }
          } else {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::nat(qs, lr, s, hb), kf[s], sacc, 0, 0, 0);
              pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L::nat(dos, lr, s, hb), LV::nat(vblk, 32 * wave + lr, s, hb), pacc, 0, 0, 0);
            }
          }
          // the first transposed fragments of the products below are on their way while the
          // probabilities are formed.  Product w of 4 * NC: column block w / 4; w % 4 = 0: dV, keys
          // half 0; 1: dK, half 0; 2: dV, half 1; 3: dK, half 1 (each accumulator takes half 0 first,
          // and no instruction follows one that writes the same accumulator)
          auto tr_operand = [&](int w) -> bf16x8 {
            const int c = w >> 2, part = w & 3;
            return L::tr((part & 1) ? qs : dos, c, 16 * (part >> 1));
          };
          bf16x8 ta[PF + 1];
#pragma unroll
          for (int w = 0; w < PF; ++w) ta[w] = tr_operand(w);
          __builtin_amdgcn_sched_barrier(0);
          // only blocks that touch the diagonal or the end of the sequence need the mask: a
          // masked score becomes -inf, so its recomputed probability is exactly 0
          if ((ib + 32 > N) || (j0w + 32 > N) || (causal && j0w + 31 > ib)) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int gi = ib + acc_row(r, hb);
              if ((gi >= N) || (j >= N) || (causal && j > gi)) sacc[r] = -INFINITY;
            }
          }
          // registers 4g .. 4g+3 of a lane hold query rows 8g + 4*hb + {0..3}: their statistics
          // are four consecutive floats, one 16-byte LDS read each
          float pv[16], ds[16];
          const float4* sl4 = reinterpret_cast<const float4*>(sl + 4 * hb);
          const float4* sd4 = reinterpret_cast<const float4*>(sd + 4 * hb);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 l4 = sl4[2 * g], d4 = sd4[2 * g];
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int r = 4 * g + e;
              const float p = fast_exp2(fmaf(sacc[r], scale_log2, -lv[e] * kLog2e));
              pv[r] = p;
              ds[r] = p * (pacc[r] - dv4[e]);
            }
          }
          const bf16x8 p0 = pack8(pv), p1 = pack8(pv + 8), d0 = pack8(ds), d1 = pack8(ds + 8);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int w = 0; w < 4 * NC; ++w) {
            if (w + PF < 4 * NC) ta[(w + PF) % (PF + 1)] = tr_operand(w + PF);
            const int c = w >> 2, part = w & 3;
            const bf16x8 a = ta[w % (PF + 1)];
            if (part == 0) dv[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p0, dv[c], 0, 0, 0);
            else if (part == 1) dk[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, d0, dk[c], 0, 0, 0);
            else if (part == 2) dv[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p1, dv[c], 0, 0, 0);
            else dk[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, d1, dk[c], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      ib += RS;
      if (--ib_left == 0) { ib_left = ntq; ib = q_begin; }
      wait_requests<(PD - 1) * NREQ>();
      __syncthreads();
    }
    if (j < N) {
      bf16* out = dqkv + ((int64_t)b * N + j) * rs + kvh * D;
      // dK rows first, then dV rows: the eight 16-byte pieces that make up a 128-byte line
      // leave in consecutive instructions and meet in the L2 before the line is written out
      // (interleaved with the other tensor's stores, lines went out half-filled: 1.28x the bytes)
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 vk;
#pragma unroll
          for (int e = 0; e < 4; ++e) vk[e] = (bf16)(dk[c][4 * g + e] * scale);
          *reinterpret_cast<bf16x4*>(out + ko + 32 * c + 8 * g + 4 * hb) = vk;
        }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 vv;
#pragma unroll
          for (int e = 0; e < 4; ++e) vv[e] = (bf16)dv[c][4 * g + e];
          *reinterpret_cast<bf16x4*>(out + vo + 32 * c + 8 * g + 4 * hb) = vv;
        }
    }
    item = tq_next(tq, qc, entry, &mail);
  }
  tq_done(tq);
}

// Workgroup shape.  The kernels are written for NW waves and a ring of stages; measured on
// the 8 x 1024 x 16 x 128 causal problem, 8 waves with four stages (one workgroup per CU,
// three tiles in flight) was no faster than 4 waves with two stages (two workgroups per CU;
// measured again for dK/dV at 16 x 2048 x 32 x 128 and 8 x 4096 x 32 x 128: 6 - 20 % slower):
// the loop is bound by the softmax arithmetic sharing the VALU port with MFMA issue, not by
// load latency.  Only the 4-wave shape is instantiated.
template <typename K>
mosaic_status launch_queued(K kern, std::once_flag& once, hipError_t& once_rc, size_t smem, hipStream_t s, int quota,
                            int wg_per_cu, int64_t heads, int tiles, int causal, TileQueueArgs* tq, int* grid, int* hb) {
  std::call_once(once, [&] {
    once_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  });
  MOSAIC_HIP(once_rc);
  // heads per block: about two rounds of an XCD's workgroups under a causal mask, else one head
  // The queue pays once every workgroup draws several items (tiles of unequal cost under a
  // causal mask, ragged last tiles, and heads that stay together on an XCD: measured 5-10 %
  // on the audio encoder's full attention at 32 and 64 CUs, 25-40 % on causal rows of 4096);
  // with up to three rounds static rounds do as well without the claims.
  const int64_t resident = (int64_t)tile_queue_sure_cus(quota) * wg_per_cu;
  const bool prefer_queue = heads * tiles > 3 * resident;
  const int per_xcd = (int)((resident + 7) / 8);
  *hb = causal ? (int)std::min<int64_t>(std::max<int64_t>(1, (2 * per_xcd + tiles - 1) / tiles), std::max<int64_t>(1, heads / 8)) : 1;
  MOSAIC_TRY(tile_queue_plan(s, quota, wg_per_cu, heads * tiles, *hb * tiles, prefer_queue, tq, grid));
  if (tq->mode == TQ_ROUNDS) *hb = 1;
  return MOSAIC_OK;
}

template <int D, int NW>
mosaic_status fwd_t(hipStream_t s, int quota, int B, int N, int H, int Hkv, int causal, const bf16* qkv, bf16* O, float* lse) {
  const int qtiles = (int)ceil_div(N, 32 * NW);
  // resident workgroups per CU: two by registers at head size 128; at 64 the forward and dQ
  // kernels need ~150 registers, so three fit (measured: forward 151 -> 130 us at B8 N1500 H20)
  constexpr size_t smem = (size_t)Ring<NW>::NST * 2 * LdsTile<64, D, NW>::BYTES;
  static std::once_flag once;
  static hipError_t once_rc = hipSuccess;
  TileQueueArgs tq;
  int grid, hb;
  // head size 128: the skewed pipeline, two workgroups per CU by registers; head size 64: the
  // tile-at-a-time kernel, three per CU
  constexpr bool PIPE = D == 128;
  auto kern = [] { if constexpr (PIPE) return attn_fwd_mfma<D, NW>; else return attn_fwd_tile_mfma<D, NW>; }();
  MOSAIC_TRY(launch_queued(kern, once, once_rc, smem, s, quota, (!PIPE && NW == 4) ? 3 : 8 / NW,
                           (int64_t)B * H, qtiles, causal, &tq, &grid, &hb));
  kern<<<grid, 64 * NW, smem, s>>>(qkv, O, lse, B, N, H, Hkv, causal, kLog2e / sqrtf((float)D), qtiles, hb, tq);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

template <int D, int NW>
mosaic_status bwd_t(hipStream_t s, int quota, int B, int N, int H, int Hkv, int causal, const bf16* qkv, const bf16* O,
                    const float* lse, const bf16* dO, bf16* dqkv, float* delta) {
  const int tiles = (int)ceil_div(N, 32 * NW);
  const float scale = 1.0f / sqrtf((float)D);
  {
    // dQ first: it also writes the per-row delta that the dK/dV kernel reads
    constexpr size_t smem = (size_t)Ring<NW>::NST * 2 * LdsTile<64, D, NW>::BYTES;
    static std::once_flag once;
    static hipError_t once_rc = hipSuccess;
    TileQueueArgs tq;
    int grid, hb;
    MOSAIC_TRY(launch_queued(attn_bwd_dq_mfma<D, NW>, once, once_rc, smem, s, quota, (D == 64 && NW == 4) ? 3 : 8 / NW,
                             (int64_t)B * H, tiles, causal, &tq, &grid, &hb));   // residency as in the forward kernel
    attn_bwd_dq_mfma<D, NW><<<grid, 64 * NW, smem, s>>>(qkv, O, dO, lse, delta, dqkv, B, N, H, Hkv, causal, scale, tiles, hb, tq);
    MOSAIC_LAUNCH_CHECK();
  }
  {
    constexpr size_t smem = (size_t)Ring<NW>::NST * 2 * LdsTile<32, D, NW>::BYTES + LdsTile<32 * NW, D, NW>::BYTES +
                            (size_t)Ring<NW>::NST * 2 * 64 * sizeof(float);
    static std::once_flag once;
    static hipError_t once_rc = hipSuccess;
    TileQueueArgs tq;
    int grid, hb;
    MOSAIC_TRY(launch_queued(attn_bwd_dkv_mfma<D, NW>, once, once_rc, smem, s, quota, 8 / NW, (int64_t)B * Hkv, tiles, causal, &tq, &grid, &hb));
    attn_bwd_dkv_mfma<D, NW><<<grid, 64 * NW, smem, s>>>(qkv, dO, lse, delta, dqkv, B, N, H, Hkv, causal, scale, tiles, hb, tq);
    MOSAIC_LAUNCH_CHECK();
  }
  return MOSAIC_OK;
}

}  // namespace

bool attention_mfma_supported(int dtype, int d) { return dtype == MOSAIC_BF16 && (d == 64 || d == 128); }

mosaic_status launch_attention_fwd_mfma(hipStream_t s, int quota, int B, int N, int H, int Hkv, int d, int causal,
                                        const void* qkv, void* O, float* lse) {
  if (d == 64) return fwd_t<64, 4>(s, quota, B, N, H, Hkv, causal, (const bf16*)qkv, (bf16*)O, lse);
  return fwd_t<128, 4>(s, quota, B, N, H, Hkv, causal, (const bf16*)qkv, (bf16*)O, lse);
}

mosaic_status launch_attention_bwd_mfma(hipStream_t s, int quota, int B, int N, int H, int Hkv, int d, int causal,
                                        const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv,
                                        float* delta) {
  if (d == 64) return bwd_t<64, 4>(s, quota, B, N, H, Hkv, causal, (const bf16*)qkv, (const bf16*)O, lse, (const bf16*)dO, (bf16*)dqkv, delta);
  return bwd_t<128, 4>(s, quota, B, N, H, Hkv, causal, (const bf16*)qkv, (const bf16*)O, lse, (const bf16*)dO, (bf16*)dqkv, delta);
}
