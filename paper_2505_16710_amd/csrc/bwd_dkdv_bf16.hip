// dK/dV of one chunk, bf16 matrix cores, accumulated into the persistent fp32 KV-gradient
// buffers (Alg. 1 second loop; Alg. 2 with per-chunk weights):
//   gV[c] += w * sum_{heads of the group} P^T dO      gK[c] += w * s * sum_{heads} dS^T Q
//
// Column-parallel: one workgroup is the only writer of 128 cache rows of one (batch, KV head),
// so the read-modify-write of gK/gV needs no atomics and the result is deterministic.
//
// The workgroup has 8 wavefronts: 4 column blocks of 32 cache rows x 2 roles.
//   role A ("probabilities"): keeps K^T fragments and the dV accumulator; computes
//          S = Q K^T, P = exp(s S - LSE) (causal mask applied), hands P (bf16) to its partner
//          through LDS and accumulates dV += P^T dO;
//   role B ("score gradient"): keeps V^T fragments and the dK accumulator; computes
//          dP = dO V^T, dS = P * (dP - delta) and accumulates dK += dS^T Q.
// Each of the four products is computed exactly once, and a wavefront holds one 32x128 fp32
// accumulator plus one operand fragment set instead of two of each, which is what lets two
// wavefronts share a SIMD.  Role A runs one row tile ahead of role B, so the P hand-over
// costs no extra barrier: one barrier per 64-row stage.
//
// The two roles are two instantiations of one body (template parameter ROLE) behind a wavefront-uniform branch at
// the top of the kernel, not two arms of a branch inside a common loop: each role then has a loop, accumulators and
// a register allocation of its own (224 instead of 256 registers, no execution-mask juggling; 7 % faster).
//
// Q, dO, -LSE / s and -delta of one stage of query rows stream through a three-deep ring of swizzled LDS
// slots, laid out region by region (Q tiles, dO tiles, row statistics, P buffers; one of each per slot)
// (A reads Q of stage i+1 while B reads Q and dO of stage i and stage i+2 is landing);
// Q and dO are copied global -> LDS directly (no staging registers), issued two stages ahead (after the first
// MFMA chain of an iteration, so that the matrix pipe starts right behind the barrier).
// S and dP are computed in the "row = query" orientation, so P and dS sit in the C layout
// with lane = cache row and feed the second products as A operands; dO and Q for those
// products come through the LDS transpose read.  P is written to LDS once (bf16, in operand
// order) for role B; role A keeps its own copy in registers for the dV product of the next iteration.
// Inside an iteration every wavefront runs four MFMA chains; the LDS operands of a chain are requested while
// the chain before it runs (across the barrier too), and the exponentials / dS products of a row block are
// written between the MFMAs of a later chain.
//
// Column tiles are enumerated from a by-value segment table (runs of cache rows that share
// one non-zero weight); SpaCO's unselected chunks simply have no tiles.
//
// A workgroup occupies a whole CU, so a launch runs in rounds of 256 column tiles and a last round with few
// tiles costs as much as a full one.  When the last round would hold at most 128 tiles, the last column tiles
// of every (batch, KV head) are therefore divided among 2 or 4 workgroups by query head: each writes its
// fp32 sums to the workspace and dkdv_tail_merge_kernel adds them to gK/gV in head order (still one writer
// per element and a fixed summation order, so results stay reproducible).
//
// The same kernel serves the transposed order of the backward pass (seco_chunk_attn_bwd_gather): there the column
// run is one chunk and the query rows are that chunk's and every later one's, p.C of them from p.q_start on, with
// -delta and -LSE read from arrays kept for the whole sequence (stat_stride, stat_off).  With ROWS the rows come as
// runs with one weight each (Alg. 2 in that order): rows outside the runs are never read, and a run's weight
// enters as log2 w added to -LSE, i.e. as a factor on P and through it on dV and dS alike.
#include "mfma_tiles.h"
#include "seco_internal.h"

#ifndef SECO_DKDV_RB
#define SECO_DKDV_RB 2
#endif

namespace seco {
namespace {

constexpr int kPBytes = 2048;   // one 32x32 bf16 P tile
constexpr int kStages = 3;

// NCB: 32-row column blocks per workgroup (2 wavefronts each); RB: 32-row query blocks per stage
template <int NCB, int RB>
struct DkdvCfg {
  static constexpr int kThreads = NCB * 128;
  static constexpr int kBQ = 32 * RB;                                   // query rows per stage
  static constexpr int kTileBytes = kBQ * kRowBytes;
  // LDS layout, region by region: the Q tiles of the kStages slots, their dO tiles, their row statistics (-LSE / s
  // and -delta, kBQ floats each), and one P buffer per slot, column block and row block.  A per-lane operand
  // offset carries the region it is used with (role A reads rows of Q and transposed blocks of dO, role B the
  // reverse), so that a slot's tile base is one scalar for both tiles.
  static constexpr int kDoRegion = kStages * kTileBytes;
  static constexpr int kStatRegion = 2 * kStages * kTileBytes;
  static constexpr int kStatBytes = 2 * kBQ * 4;
  static constexpr int kPRegion = kStatRegion + kStages * kStatBytes;
  static constexpr int kSmemBytes = kPRegion + kStages * NCB * RB * kPBytes;
  static constexpr int kCols = NCB * 32;                                // cache rows per workgroup
};

// The last n_tiles column tiles of every (batch, KV head) are each divided among hs workgroups by query head;
// their sums go to part[split tile][head share][dV, dK][cache row of the tile][128] instead of gK/gV.
struct TailSplit {
  int n_tiles;
  int hs;
  float* part;
};

// (RB is fixed to 2 by the hand-pipelined main loop.)
// ROWS: the query rows are taken from a table of runs (rows relative to p.q_start, each run with one weight whose
// log2 is added to -LSE, i.e. its probabilities are scaled by the weight) instead of being all p.C rows with weight 1.
// ROLE: 0 = role A, 1 = role B.  The body of a wavefront is instantiated once per role, so that a role's accumulators
// and working set are the variables of a loop of its own: with both roles as the two arms of a branch inside one
// loop, unrolled over the ring slots, the register allocator could not keep the working set in registers.
template <int NCB, int RB, bool ROWS, int ROLE>
__device__ __forceinline__ void dkdv_bf16_body(const AttnParams& p, const SegTable& seg, const TailSplit& ts,
                                               const RowRuns& rr, int total_items, lds_char* smem) {
  using Cfg = DkdvCfg<NCB, RB>;
  constexpr int BQ = Cfg::kBQ, kTileBytes = Cfg::kTileBytes;
  constexpr int kDoRegion = Cfg::kDoRegion, kStatRegion = Cfg::kStatRegion, kStatBytes = Cfg::kStatBytes;
  constexpr int NW = 2 * NCB;                 // wavefronts
  constexpr int kCopies = (BQ / 4) / NW;      // 4-row direct copies of Q (and of dO) per wavefront and stage
  static_assert((BQ / 4) % NW == 0, "stage rows must split evenly over the wavefronts");
  lds_char* pbuf = smem + Cfg::kPRegion;

  const int item = xcd_item(blockIdx.x, total_items);
  if (item < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  constexpr int role = ROLE;
  const int cb = wave % NCB;
  // item -> (batch, kv head, column tile, share of the query heads); the divided tiles come last in a unit
  const int n_ctiles = seg.tile_begin[seg.n];
  const int n_whole = n_ctiles - ts.n_tiles;
  const int per_unit = n_whole + ts.n_tiles * ts.hs;
  const int unit = item / per_unit, in_unit = item % per_unit;
  const bool divided = in_unit >= n_whole;
  const int tile = divided ? n_whole + (in_unit - n_whole) / ts.hs : in_unit;
  const int share = divided ? (in_unit - n_whole) % ts.hs : 0;
  const int n_heads = divided ? p.G / ts.hs : p.G;   // query heads of the group handled here, from head0 on
  const int head0 = share * n_heads;
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  int si = 0;
  while (si + 1 < seg.n && tile >= seg.tile_begin[si + 1]) ++si;
  const int c0 = seg.col_begin[si] + (tile - seg.tile_begin[si]) * Cfg::kCols;
  const int c_end = min(c0 + Cfg::kCols, seg.col_end[si]);
  const float weight = seg.weight[si];

  const int kv_len = p.q_start + p.C;
  const int n0 = c0 + cb * 32;     // first cache row of this wavefront
  const int col = n0 + l32;        // this lane's cache row in the score tile
  // role A holds K^T fragments, role B holds V^T fragments
  const __bf16* fptr = static_cast<const __bf16*>(role == 0 ? p.k : p.v) + b * p.kvs[0] + kvh * p.kvs[1] +
                       (int64_t)min(col, kv_len - 1) * p.kvs[2];
  bf16x8 frag[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) frag[t] = *reinterpret_cast<const bf16x8*>(fptr + 16 * t + 8 * g);
  // Role A starts its MFMA chains from -LSE / s instead of zero, so that a chain delivers q.k - LSE / s and
  // P = exp2(c * that) with c = s * log2(e): one multiply per score, in fp32.  (Folding c into the K^T fragments
  // would save that multiply but round K a second time, to bf16: with scores far from zero, as with the outlier
  // components of trained models, P = exp(S - LSE) hangs on the low-order bits of S, and the extra rounding showed
  // as errors of several per cent in gV and gK.)  Role B starts its chains from -delta.
  const float c2 = p.scale * kLog2e;

  // query-row stages that see at least one cache row of this workgroup; iteration = (head of the group, stage)
  const int rt0 = max(0, c0 - p.q_start) / BQ;
  struct Pos { int hg, r0, ri; };   // head within the group, first chunk-local row of the stage, run of rows
  // first stage of a head, and the number of stages per head
  int first_ri = 0, first_r0 = rt0 * BQ, n_rt;
  if constexpr (ROWS) {
    while (first_ri + 1 < rr.n && rr.end[first_ri] <= first_r0) ++first_ri;
    first_r0 = max(first_r0, rr.begin[first_ri]);
    n_rt = (rr.end[first_ri] - first_r0 + BQ - 1) / BQ;
    for (int i = first_ri + 1; i < rr.n; ++i) n_rt += (rr.end[i] - rr.begin[i] + BQ - 1) / BQ;
    n_rt = max(n_rt, 0);
  } else {
    n_rt = (p.C + BQ - 1) / BQ - rt0;
  }
  const int n_iter = n_rt * n_heads;
  // rows [x.r0, row_limit(x)) of a stage exist; the others are masked
  auto row_limit = [&](Pos x) { return ROWS ? rr.end[x.ri] : p.C; };
  auto advance = [&](Pos x) {
    x.r0 += BQ;
    if constexpr (ROWS) {
      if (x.r0 >= rr.end[x.ri]) {
        if (++x.ri == rr.n) { x.ri = first_ri; x.r0 = first_r0; x.hg += 1; }
        else x.r0 = rr.begin[x.ri];
      }
    } else {
      if (x.r0 >= p.C) { x.r0 = first_r0; x.hg += 1; }
    }
    return x;
  };

  const __bf16* qbase = static_cast<const __bf16*>(p.q) + b * p.qs[0] + (int64_t)kvh * p.G * p.qs[1];
  const __bf16* dobase = static_cast<const __bf16*>(p.d_o) + b * p.os[0] + (int64_t)kvh * p.G * p.os[1];
  const int64_t stat_base = ((int64_t)b * p.Hq + (int64_t)kvh * p.G) * p.stat_stride + p.stat_off;
  // asynchronous global -> LDS copy of the Q and dO tiles of one stage (4 rows per wavefront and copy).  A stage
  // that lies entirely inside the chunk is copied from scalar base addresses with constant per-lane offsets (no
  // vector arithmetic); the last, ragged one uses clamped per-lane addresses.
  uint32_t q_lane_off[kCopies], do_lane_off[kCopies];
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    q_lane_off[i] = dma_lane_offset(4 * (wave + NW * i), p.qs[2] * 2, lane);
    do_lane_off[i] = dma_lane_offset(4 * (wave + NW * i), p.os[2] * 2, lane);
  }
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + wave * 4 * kRowBytes);
  // Global addresses of a stage's first row (Q, dO, and the row statistic this wavefront copies).  They are carried
  // along with the stage two ahead and advanced by one stage's worth per iteration: computing them from (head, row)
  // costs a dozen 64-bit scalar multiplies per iteration and wavefront.
  struct Src { const __bf16* q; const __bf16* d_o; const float* stat; };
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto src_of = [&](Pos x) {
    Src r;
    r.q = qbase + x.hg * p.qs[1] + (int64_t)x.r0 * p.qs[2];
    r.d_o = dobase + x.hg * p.os[1] + (int64_t)x.r0 * p.os[2];
    r.stat = (wave_u == 0 ? p.nlse2 : p.delta) + stat_base + (int64_t)x.hg * p.stat_stride + x.r0;
    return r;
  };
  auto copy_stage = [&](Pos x, int slot, const Src& src) {
    if (x.r0 + BQ <= row_limit(x)) {
      const __bf16* q_src = src.q;
      const __bf16* do_src = src.d_o;
#pragma unroll
      for (int i = 0; i < kCopies; ++i) {
        const uint32_t dst = lds_wave + slot * kTileBytes + i * (4 * NW * kRowBytes);
        dma16_sbase(q_src, q_lane_off[i], dst);
        dma16_sbase(do_src, do_lane_off[i], dst + kDoRegion);
      }
    } else {
      lds_char* qt = smem + slot * kTileBytes;
#pragma unroll
      for (int i = 0; i < kCopies; ++i) {
        const int r = 4 * (wave + NW * i);
        const int src_row = min(x.r0 + r + (lane >> 4), p.C - 1);
        dma4rows(qt, r, qbase + x.hg * p.qs[1] + (int64_t)src_row * p.qs[2], lane);
        dma4rows(qt + kDoRegion, r, dobase + x.hg * p.os[1] + (int64_t)src_row * p.os[2], lane);
      }
    }
  };
  // -LSE / s and -delta of the stage's rows, as the dQ kernel left them in the workspace: one
  // asynchronous 64-lane copy each (wavefronts 0 and 1), straight into the stage's slot.  The last, ragged stage
  // of a head goes through registers instead: rows past the chunk get -LSE = -inf so that their probabilities vanish.
  static_assert(BQ == 64, "one 64-lane copy per row statistic");
  const uint32_t lds_stat = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + kStatRegion + (wave & 1) * BQ * 4);
  auto copy_stat = [&](Pos x, int slot, const Src& src) {
    if (x.r0 + BQ <= row_limit(x)) {
      if (wave_u < 2) {
        const uint64_t a = (uint64_t)(uintptr_t)src.stat;
        // (wavefront-uniform by construction; the halves go through readfirstlane so that the compiler keeps them
        // in scalar registers; each half is widened from an unsigned 32-bit value)
        const uint64_t src = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(a >> 32)) << 32) |
                             (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)a);
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1"
                     :
                     : "v"(lane * 4), "s"(src), "s"(lds_stat + slot * kStatBytes)
                     : "memory", "m0");
      }
    } else if (wave_u < 2) {             // (wavefront-uniform control flow only: the copies above need scalar addresses)
      const int row = x.r0 + lane;
      const float v = (wave_u == 0 ? p.nlse2 : p.delta)[stat_base + (int64_t)x.hg * p.stat_stride + min(row, p.C - 1)];
      const float stat = wave_u == 0 && row >= row_limit(x) ? -INFINITY : v;
      *reinterpret_cast<SECO_LDS float*>(smem + kStatRegion + slot * kStatBytes + (wave_u * BQ + lane) * 4) = stat;
    }
  };

  // lane-dependent parts of the LDS operand addresses (constant for the whole kernel)
  int r_off[8];
  TrOff t_off[4];
  // role A reads rows of Q and transposed blocks of dO, role B rows of dO and transposed blocks of Q: the region of
  // the tile an offset is used with is part of the offset
  const int r_region = role == 0 ? 0 : kDoRegion, t_region = role == 0 ? kDoRegion : 0;
#pragma unroll
  for (int t = 0; t < 8; ++t) r_off[t] = row8_lane_off(l32, 2 * t + g) + r_region;
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    t_off[db] = tr8_lane_off(db, lane);
    t_off[db].lo += t_region;
    t_off[db].hi += t_region;
  }

  f32x16 acc[4];   // role A: dV, role B: dK  (32 cache rows x 128)
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  // P of the stage held in slot `slot`, row block rb, this wavefront's column block: p_lane is the lane-dependent
  // part of the address (the lane's 16 bytes of the wavefront's block), the rest a constant per slot and row block
  int p_lane = cb * RB * kPBytes + lane * 16;
  auto pslot = [&](int slot, int rb) { return pbuf + (slot * NCB * RB + rb) * kPBytes + p_lane; };

  // zero the probabilities of a 32x32 block (first query position qpos0) that lie above the diagonal
  // (register r of a score tile holds query row 8 (r / 4) + 4 g + r % 4 of the block: the lane-dependent part of the
  // comparison is one value, the rest compile-time constants, so that nothing per-lane has to be kept for it)
  auto mask_above_diagonal = [&](f32x16& s, int qpos0) {
    if (n0 + 31 > qpos0) {
      const int ahead = col - qpos0 - 4 * g;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (ahead > 8 * (r >> 2) + (r & 3)) s[r] = 0.f;
    }
  };

  // role A: S = Q K^T for row block rb of the stage in `slot`, P = exp2(c2 * (S - LSE / s)) with the causal mask;
  // P goes to pbuf as two operand halves (lane-contiguous 16-byte words)
  auto scores = [&](int slot, int r0, int rb, float lw) {   // lw: log2 of the rows' weight, divided by c2
    lds_char* qt = smem + slot * kTileBytes;
    SECO_LDS float* lse_s = reinterpret_cast<SECO_LDS float*>(smem + kStatRegion + slot * kStatBytes) + 32 * rb;
    bf16x8 a[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) a[t] = lds_row8(qt, 32 * rb + l32, 2 * t + g);
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = lse_s[8 * (r >> 2) + 4 * g + (r & 3)];
    if constexpr (ROWS) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] += lw;
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) s = mfma(a[t], frag[t], s);
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = fast_exp2(s[r] * c2);
    mask_above_diagonal(s, p.q_start + r0 + 32 * rb);
    lds_char* pb = pslot(slot, rb);
    *reinterpret_cast<SECO_LDS bf16x8*>(pb) = pack8(s, 0);
    *reinterpret_cast<SECO_LDS bf16x8*>(pb + 1024) = pack8(s, 1);
  };

  Pos cur{head0, first_r0, first_ri};
  Pos nxt = advance(cur);
  {
    const Src s0 = src_of(cur), s1 = src_of(nxt);
    copy_stage(cur, 0, s0);
    copy_stat(cur, 0, s0);
    if (n_iter > 1) {
      copy_stage(nxt, 1, s1);
      copy_stat(nxt, 1, s1);
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) settle(frag[t]);
  dma_wait_all();
  __syncthreads();
  if constexpr (role == 0) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) scores(0, cur.r0, rb, ROWS ? rr.log2w[cur.ri] / c2 : 0.f);
  }
  __syncthreads();
  Pos nxt2 = advance(nxt);
  Src src2 = src_of(nxt2);
  // (all rows, no runs) one stage on: BQ rows further, or, behind a head's last stage, back to the first stage's row
  // of the next head
  const int64_t q_step = (int64_t)BQ * p.qs[2], do_step = (int64_t)BQ * p.os[2];
  const int64_t back_rows = (int64_t)(n_rt - 1) * BQ;
  const int64_t q_wrap = p.qs[1] - back_rows * p.qs[2], do_wrap = p.os[1] - back_rows * p.os[2];
  const int64_t stat_wrap = p.stat_stride - back_rows;

  // One operand buffer x[8] rotates through the four MFMA chains of an iteration: while a chain consumes x[t], the
  // operand of the next chain is requested into the same register ("comes in behind").  The last chain of an
  // iteration requests the operands of the first chain of the next one, which read a stage that has already
  // landed, so that no wavefront starts an iteration by waiting for LDS.  Role A also carries the probabilities of
  // the stage it is about to use for dV (pa0, pa1: its own P blocks, as operands) in registers.
  bf16x8 x[8];
  bf16x8 pa0[2], pa1[2];
  auto p_half = [&](lds_char* pb, int t) { return *reinterpret_cast<SECO_LDS bf16x8*>(pb + 1024 * t); };
  if constexpr (role == 0) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      pa0[t] = p_half(pslot(0, 0), t);
      pa1[t] = p_half(pslot(0, 1), t);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = lds_tr8_at(smem, t_off[i & 3], 16 * (i >> 2));
  } else {
#pragma unroll
    for (int t = 0; t < 8; ++t) x[t] = lds_row8_at(smem + r_off[t], 0);
  }

  int slot = 0;   // it % kStages
  for (int it = 0; it < n_iter; ++it) {
    const int slot1 = slot + 1 == kStages ? 0 : slot + 1;
    const int slot2 = slot1 + 1 == kStages ? 0 : slot1 + 1;
    // The copies of stage it + 2 are issued after the first MFMA chain of the iteration, not at its top: right
    // after the barrier every wavefront has the operands of its first chain in registers, and the matrix pipe
    // should start on them at once instead of waiting behind sixteen copy instructions and their address
    // arithmetic (3 % on the kernel; issued later still, the copy has too little time to land before the
    // wait at the end of the iteration).
    auto issue_copies = [&]() {
      if (it + 2 < n_iter) {
        copy_stage(nxt2, slot2, src2);
        copy_stat(nxt2, slot2, src2);
      }
    };
    // tiles of the stage in `slot` and of the next stage; whether an access goes to the Q or to the dO tile of the
    // slot is decided by the region that its per-lane offset (r_off, t_off) carries
    lds_char* t0 = smem + slot * kTileBytes;
    lds_char* t1 = smem + slot1 * kTileBytes;
    // Row blocks above the diagonal are not skipped: their probabilities are masked to zero and contribute nothing
    // (only the first stages of a diagonal column tile are affected).  In both roles the vector work on a row block
    // (exponentials; dS = P * (dP - delta)) is written between the MFMAs of a later chain, two values per MFMA, so
    // that a wavefront keeps the matrix pipe fed while its own vector instructions issue.
    if constexpr (role == 0) {
      // stage `it`: dV += P^T dO (P from the previous iteration); stage `it + 1`: P = exp2(Q K^T c - LSE)
      SECO_LDS float* lse_s = reinterpret_cast<SECO_LDS float*>(smem + kStatRegion + slot1 * kStatBytes);
      // dV of row block 0; Q rows of row block 0 of the next stage come in behind
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc[i & 3] = mfma(pa0[i >> 2], x[i], acc[i & 3]);
        x[i] = lds_row8_at(t1 + r_off[i], 0);
      }
      issue_copies();
      f32x16 s0, s1;
#pragma unroll
      for (int r = 0; r < 16; ++r) s0[r] = lse_s[8 * (r >> 2) + 4 * g + (r & 3)];
#pragma unroll
      for (int r = 0; r < 16; ++r) s1[r] = lse_s[32 + 8 * (r >> 2) + 4 * g + (r & 3)];
      if constexpr (ROWS) {                   // probabilities of the next stage's rows carry their run's weight
        const float lw = rr.log2w[nxt.ri] / c2;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s0[r] += lw;
          s1[r] += lw;
        }
      }
      // log2 P of row block 0 (chain started from -LSE); Q rows of row block 1 come in behind
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        s0 = mfma(x[t], frag[t], s0);
        x[t] = lds_row8_at(t1 + r_off[t], 32);
      }
      // log2 P of row block 1, with the exponentials of row block 0; dO^T of row block 1 (stage `it`) comes in behind
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        s1 = mfma(x[t], frag[t], s1);
        x[t] = lds_tr8_at(t0, t_off[t & 3], 32 + 16 * (t >> 2));
        s0[2 * t] = fast_exp2(s0[2 * t] * c2);
        s0[2 * t + 1] = fast_exp2(s0[2 * t + 1] * c2);
      }
      mask_above_diagonal(s0, p.q_start + nxt.r0);
      const bf16x8 pn0[2] = {pack8(s0, 0), pack8(s0, 1)};
      lds_char* pw0 = pslot(slot1, 0);
      *reinterpret_cast<SECO_LDS bf16x8*>(pw0) = pn0[0];
      *reinterpret_cast<SECO_LDS bf16x8*>(pw0 + 1024) = pn0[1];
      // dV of row block 1, with the exponentials of row block 1 of the next stage; dO^T of row block 0 of the next
      // stage comes in behind (for the first chain of the next iteration)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc[i & 3] = mfma(pa1[i >> 2], x[i], acc[i & 3]);
        x[i] = lds_tr8_at(t1, t_off[i & 3], 16 * (i >> 2));
        s1[2 * i] = fast_exp2(s1[2 * i] * c2);
        s1[2 * i + 1] = fast_exp2(s1[2 * i + 1] * c2);
      }
      mask_above_diagonal(s1, p.q_start + nxt.r0 + 32);
      pa0[0] = pn0[0];
      pa0[1] = pn0[1];
      pa1[0] = pack8(s1, 0);
      pa1[1] = pack8(s1, 1);
      lds_char* pw1 = pslot(slot1, 1);
      *reinterpret_cast<SECO_LDS bf16x8*>(pw1) = pa1[0];
      *reinterpret_cast<SECO_LDS bf16x8*>(pw1 + 1024) = pa1[1];
    } else {
      // stage `it`: dS = P * (dO V^T - delta), dK += dS^T Q
      SECO_LDS float* delta_s = reinterpret_cast<SECO_LDS float*>(smem + kStatRegion + slot * kStatBytes) + BQ;
      lds_char* pb0 = pslot(slot, 0);
      const bf16x8 ph0[2] = {p_half(pb0, 0), p_half(pb0, 1)};
      lds_char* pb1 = pslot(slot, 1);
      const bf16x8 ph1[2] = {p_half(pb1, 0), p_half(pb1, 1)};
      f32x16 d0, d1;
#pragma unroll
      for (int r = 0; r < 16; ++r) d0[r] = delta_s[8 * (r >> 2) + 4 * g + (r & 3)];
#pragma unroll
      for (int r = 0; r < 16; ++r) d1[r] = delta_s[32 + 8 * (r >> 2) + 4 * g + (r & 3)];
      // dP - delta of row block 0 (chain started from -delta); dO rows of row block 1 come in behind
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        d0 = mfma(x[t], frag[t], d0);
        x[t] = lds_row8_at(t0 + r_off[t], 32);
      }
      issue_copies();
      // dP - delta of row block 1, with dS of row block 0; Q^T of row block 0 comes in behind
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        d1 = mfma(x[t], frag[t], d1);
        x[t] = lds_tr8_at(t0, t_off[t & 3], 16 * (t >> 2));
        d0[2 * t] *= (float)ph0[t >> 2][(2 * t) & 7];
        d0[2 * t + 1] *= (float)ph0[t >> 2][(2 * t + 1) & 7];
      }
      const bf16x8 ds0[2] = {pack8(d0, 0), pack8(d0, 1)};
      // dK of row block 0, with dS of row block 1; Q^T of row block 1 comes in behind
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc[i & 3] = mfma(ds0[i >> 2], x[i], acc[i & 3]);
        x[i] = lds_tr8_at(t0, t_off[i & 3], 32 + 16 * (i >> 2));
        d1[2 * i] *= (float)ph1[i >> 2][(2 * i) & 7];
        d1[2 * i + 1] *= (float)ph1[i >> 2][(2 * i + 1) & 7];
      }
      const bf16x8 ds1[2] = {pack8(d1, 0), pack8(d1, 1)};
      // dK of row block 1; dO rows of row block 0 of the next stage come in behind (for the next iteration)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc[i & 3] = mfma(ds1[i >> 2], x[i], acc[i & 3]);
        x[i] = lds_row8_at(t1 + r_off[i], 0);
      }
    }
    dma_wait_all();
    __syncthreads();
    cur = nxt;
    nxt = nxt2;
    {
      const Pos adv = advance(nxt2);
      if constexpr (ROWS) {
        src2 = src_of(adv);
      } else {
        const bool wrap = adv.hg != nxt2.hg;
        src2.q += wrap ? q_wrap : q_step;
        src2.d_o += wrap ? do_wrap : do_step;
        src2.stat += wrap ? stat_wrap : (int64_t)BQ;
      }
      nxt2 = adv;
    }
    slot = slot1;
  }

  // The lane-dependent indices of the epilogue are derived again from the thread index (through an empty asm, so
  // that the compiler does not keep the ones computed before the loop alive across it: the loop uses every register).
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int l32_e = tid_e & 31, g_e = (tid_e >> 5) & 1, n0_e = c0 + ((tid_e >> 6) % NCB) * 32;
  if (divided) {
    // a share of the heads: plain stores of the unweighted sums, all 32 rows (the merge drops rows past the tile's end)
    float* pb = ts.part + ((((int64_t)unit * ts.n_tiles + (tile - n_whole)) * ts.hs + share) * 2 + role) *
                              (int64_t)(Cfg::kCols * 128) + (cb * 32) * 128 + l32_e;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float* pr = pb + (8 * (r >> 2) + 4 * g_e + (r & 3)) * 128;
#pragma unroll
      for (int db = 0; db < 4; ++db) pr[32 * db] = acc[db][r];
    }
    return;
  }
  // exclusive read-modify-write of this workgroup's gK/gV rows: role A adds dV, role B adds s * dK
  float* gbase = (role == 0 ? p.gv : p.gk) + b * p.gs[0] + kvh * p.gs[1];
  const float wf = role == 0 ? weight : weight * p.scale;
  // All 64 old values are requested before the first one is used (rows past the tile's end read a clamped
  // address and are not written back): one memory round trip instead of one per group of rows.
  float old[16][4];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int kvrow = min(n0_e + 8 * (r >> 2) + 4 * g_e + (r & 3), c_end - 1);
    const float* gr = gbase + (int64_t)kvrow * p.gs[2] + l32_e;
#pragma unroll
    for (int db = 0; db < 4; ++db) old[r][db] = gr[32 * db];
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int kvrow = n0_e + 8 * (r >> 2) + 4 * g_e + (r & 3);
    if (kvrow < c_end) {
      float* gr = gbase + (int64_t)kvrow * p.gs[2] + l32_e;
#pragma unroll
      for (int db = 0; db < 4; ++db) gr[32 * db] = old[r][db] + wf * acc[db][r];
    }
  }
}

template <int NCB, int RB, bool ROWS>
__global__ __launch_bounds__(NCB * 128, 2) void dkdv_bf16_kernel(AttnParams p, SegTable seg, TailSplit ts,
                                                                  RowRuns rr, int total_items) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];   // Cfg::kSmemBytes (can exceed the 64 KiB static limit)
  lds_char* smem = (lds_char*)smem_raw;
  // wavefronts 0 .. NCB-1: role A, the others role B (wavefront-uniform: a scalar branch)
  const int role_u = __builtin_amdgcn_readfirstlane((int)threadIdx.x / (64 * NCB));
  if (role_u == 0)
    dkdv_bf16_body<NCB, RB, ROWS, 0>(p, seg, ts, rr, total_items, smem);
  else
    dkdv_bf16_body<NCB, RB, ROWS, 1>(p, seg, ts, rr, total_items, smem);
}

// gK/gV of the divided column tiles: g += w * (sum of the head shares, in head order).  One thread per four
// consecutive elements of a (tile, dV or dK) pair.
template <int COLS>
__global__ __launch_bounds__(256) void dkdv_tail_merge_kernel(AttnParams p, SegTable seg, TailSplit ts, int n_units) {
  constexpr int kQuads = COLS * 128 / 4;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int quad = (int)(gid % kQuads);
  const int64_t pair = gid / kQuads;
  const int role = (int)(pair & 1);
  const int64_t st = pair >> 1;                       // divided tile, counted over all units
  if (st >= (int64_t)n_units * ts.n_tiles) return;
  const int unit = (int)(st / ts.n_tiles);
  const int n_ctiles = seg.tile_begin[seg.n];
  const int tile = n_ctiles - ts.n_tiles + (int)(st % ts.n_tiles);
  int si = 0;
  while (si + 1 < seg.n && tile >= seg.tile_begin[si + 1]) ++si;
  const int row = seg.col_begin[si] + (tile - seg.tile_begin[si]) * COLS + quad / 32;
  if (row >= seg.col_end[si]) return;
  const float wf = role == 0 ? seg.weight[si] : seg.weight[si] * p.scale;
  const float* src = ts.part + (st * ts.hs * 2 + role) * (int64_t)(COLS * 128) + (int64_t)quad * 4;
  float4 sum = *reinterpret_cast<const float4*>(src);
  for (int h = 1; h < ts.hs; ++h) {
    const float4 x = *reinterpret_cast<const float4*>(src + (int64_t)h * 2 * COLS * 128);
    sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
  }
  const int kvh = unit % p.Hkv, b = unit / p.Hkv;
  float* g = (role == 0 ? p.gv : p.gk) + b * p.gs[0] + kvh * p.gs[1] + (int64_t)row * p.gs[2] + (quad % 32) * 4;
  float4 old = *reinterpret_cast<float4*>(g);
  old.x += wf * sum.x; old.y += wf * sum.y; old.z += wf * sum.z; old.w += wf * sum.w;
  *reinterpret_cast<float4*>(g) = old;
}

}  // namespace

template <int NCB, int RB, bool ROWS>
int launch_cfg(const AttnParams& p, const SegTable& seg, const RowRuns& rr, hipStream_t s) {
  using Cfg = DkdvCfg<NCB, RB>;
  const int n_units = p.Hkv * p.B, n_ctiles = seg.tile_begin[seg.n];
  TailSplit ts{0, 1, p.tail_part};
  int n_rows = p.C;
  if (ROWS) {
    n_rows = 0;
    for (int i = 0; i < rr.n; ++i) n_rows += rr.end[i] - rr.begin[i];
  }
  const TailPlan tp = tail_plan(n_units, n_ctiles, p.G, n_rows);
  if (p.tail_part && tp.hs > 1) {
    ts.n_tiles = tp.n_tiles;
    ts.hs = tp.hs;
  }
  const int total = n_units * (n_ctiles - ts.n_tiles + ts.n_tiles * ts.hs);
  auto kern = dkdv_bf16_kernel<NCB, RB, ROWS>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          Cfg::kSmemBytes) != hipSuccess)
    return SECO_ERR_LAUNCH;
  {
    ProfScope prof(kKernelDkdv, s);   // the merge of the divided tiles counts as part of the dK/dV pass
    hipLaunchKernelGGL(kern, dim3(xcd_grid(total)), dim3(Cfg::kThreads), Cfg::kSmemBytes, s, p, seg, ts, rr, total);
    if (ts.n_tiles > 0) {
      const int64_t threads = (int64_t)n_units * ts.n_tiles * 2 * (Cfg::kCols * 128 / 4);
      hipLaunchKernelGGL(dkdv_tail_merge_kernel<Cfg::kCols>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, p,
                         seg, ts, n_units);
    }
  }
  return launch_status();
}

int launch_dkdv_bf16(const AttnParams& p, const SegTable& seg, hipStream_t s) {
  if (seg.tile_begin[seg.n] == 0) return SECO_OK;
  RowRuns none;
  none.n = 0;
  return launch_cfg<kColTileBf16 / 32, SECO_DKDV_RB, false>(p, seg, none, s);
}

int launch_dkdv_rows_bf16(const AttnParams& p, const SegTable& seg, const RowRuns& rr, hipStream_t s) {
  if (seg.tile_begin[seg.n] == 0 || rr.n == 0) return SECO_OK;
  return launch_cfg<kColTileBf16 / 32, SECO_DKDV_RB, true>(p, seg, rr, s);
}

}  // namespace seco
