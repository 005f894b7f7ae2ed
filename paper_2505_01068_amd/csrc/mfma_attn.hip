// Flash-style IM attention on the CDNA4 matrix cores: bf16 operands, fp32
// accumulation, head dimension 64 (forward also head dimensions 8 / 16 in its
// sub-head mode).
//
// All three kernels compute "transposed" products so that every per-row
// quantity of the softmax lives on the lane that owns the row:
//   forward / dQ : lane <-> query row.  S^T = K Q^T  (rows = keys, cols = queries);
//                  O^T = V^T P^T and dQ^T = K^T dS^T take P^T / dS^T straight from
//                  the accumulator registers (see perm32 in mfma_common.hpp).
//   dK / dV      : lane <-> key row.    S = Q K^T (rows = queries), dP = dO V^T;
//                  dV^T = dO^T P and dK^T = Q^T dS take P / dS from registers.
// K/V (or Q/dO) tiles of 64 rows go through a ring of LDS stages, row-major
// (swizzled, filled by asynchronous global->LDS copies); products
// that need the tile transposed (V^T, K^T, Q^T, dO^T as the MFMA "A" operand)
// read it with the gfx950 LDS transpose read (ds_read_b64_tr_b16), so no
// transposed copy of any tensor exists in HBM.
//
// Conventions between the kernels: the Q rows arrive multiplied by scale * log2(e) (the QKV projection's
// epilogue does it before its one rounding to bf16), so Q K^T is the score in the exponent domain of
// exp2 and no kernel multiplies scores; the per-row statistic saved by the forward is the NEGATED
// log2-sum-exp (-inf for a row without any valid key), which the backward kernels add to the score --
// every kernel by starting its score accumulator from it (the forward from its running reference),
// as the dP accumulators start from -delta: the MFMA chains end as S - lse and dP - delta and the
// softmax needs no add per element (dK/dV in sub-head mode still adds them per element).
//
// Only live (query segment, key segment) blocks of the Interlaced Mask are
// visited (Sec. 6 "Decomposition"); a row with several live segments carries
// one running max / sum across all of them (Sec. "Information Disorder").
#include <algorithm>
#include <type_traits>
#include "mfma_common.hpp"
#include "mfma_path.hpp"

namespace imattn {

constexpr int KT = 64;  // keys (or query rows) per staged tile

// Workgroup -> (tile, head, batch element).  As with xcd_block_index every XCD owns a contiguous
// range of (batch element, head) pairs, but inside that range the workgroups are ordered by segment
// first (the tile order lists the segments by decreasing work per tile), then pair, then tile.  A
// workgroup of a long live range runs several times longer than one of a short range; started pair
// by pair, the long workgroups of the last pairs begin late and the XCD drains with most of its CUs
// idle.  Started first, they leave the short ones to fill the tail.  The plain order is kept when
// the pairs do not divide evenly over the 8 XCDs.
__device__ __forceinline__ void xcd_tile_index(const int* prefix, int nord, bool tile_first, int& tile, int& h, int& b) {
  const unsigned gx = gridDim.x, gy = gridDim.y, npair = gy * gridDim.z;
  if (npair & 7u) {
    xcd_block_index(tile, h, b);
    return;
  }
  const unsigned lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  const unsigned xcd = lin & 7u, idx = lin >> 3, per = npair >> 3;  // pairs per XCD
  int k = 0;
  while (k + 1 < nord && idx >= per * (unsigned)prefix[k + 1]) ++k;
  const unsigned nt = (unsigned)(prefix[k + 1] - prefix[k]), j = idx - per * (unsigned)prefix[k];
  unsigned pl, t, hh, bb;
  if (tile_first) udivmod(j, per, t, pl);  // packed rows: see segment_major_index
  else udivmod(j, nt, pl, t);
  udivmod(xcd * per + pl, gy, bb, hh);
  tile = prefix[k] + (int)t;
  h = (int)hh;
  b = (int)bb;
}

// key-validity bit mask of one 64-key tile (bit k <=> key k0+k is a valid key)
__device__ __forceinline__ unsigned long long tile_key_mask(const uint8_t* key_pad_row, int k0, int klen, int lane) {
  const int k = k0 + lane;
  bool ok = k < klen;
  if (ok && key_pad_row) ok = key_pad_row[k] == 0;
  return __ballot(ok);
}

// Streamed operands (K and V tiles in the forward and dQ kernels, Q and dO tiles in the dK/dV
// kernel) go from global memory straight into a ring of RING_NST LDS stages with asynchronous
// global->LDS copies (no staging registers, no LDS store instructions): stage t+2 is requested
// while stage t is consumed, with one workgroup barrier per stage.  Each lane fetches the 16-byte
// chunk that belongs at ITS position of the swizzled tile (see sw_f), so the copy produces the
// conflict-free layout directly.  The tiles of all live segments form one sequence, so the ring
// does not drain between segments.
constexpr int RING_NST = 3;
constexpr int RING_STAGE = 2 * KT * SW_LD;  // bf16 elements per stage: two 64 x 64 tiles

// Cursor over the 64-row tiles of the live segments, ascending segment order; segments whose
// length (as given by len_of) is <= 0 are skipped.  len <= 0 <=> exhausted.  All scalar.
struct TileCursor {
  unsigned rest;  // live segments not started yet
  int seg, r0, len;
};
template <class LenFn>
__device__ __forceinline__ void cursor_next_seg(TileCursor& c, LenFn len_of) {
  c.r0 = 0;
  c.len = 0;
  while (c.rest && c.len <= 0) {
    c.seg = __builtin_ctz(c.rest);
    c.rest &= c.rest - 1;
    c.len = len_of(c.seg);
  }
}
template <class LenFn>
__device__ __forceinline__ void cursor_step(TileCursor& c, LenFn len_of) {
  c.r0 += KT;
  if (c.r0 >= c.len) cursor_next_seg(c, len_of);
}

// Per-lane constants of the ring copies: the two tile rows whose chunk positions this lane fills
// and the byte offset of the logical chunk inside a row of head h.
struct RingLane {
  int trow0, trow1;
  unsigned col0, col1;
};
// NW = waves per workgroup: with 4 waves a lane fills chunk positions in two tile rows (trow0, trow0 + 32) of
// each streamed matrix, with 8 waves in one row (trow1 / col1 unused).
template <int NW = 4>
__device__ __forceinline__ RingLane ring_lane(int wave, int lane, int h) {
  RingLane r;
  r.trow0 = wave * 8 + (lane >> 3);
  r.trow1 = NW == 4 ? r.trow0 + 32 : r.trow0;
  r.col0 = (unsigned)(h * 64 + (((lane & 7) ^ sw_f(r.trow0)) << 3)) * 2u;
  r.col1 = (unsigned)(h * 64 + (((lane & 7) ^ sw_f(r.trow1)) << 3)) * 2u;
  return r;
}
// Scalar state of the ring copies inside the current segment: byte pointers to the first row of the
// next tile of the two streamed matrices, and the rows the segment has from there on (> 0).  Kept in
// scalar registers and advanced by one tile per request, so a request costs a handful of scalar adds.
struct RingFeed {
  const char* a;
  const char* b;
  int rows;
};
// per-lane byte offsets of this lane's four chunks in a tile that lies wholly inside the segment
struct RingLaneOff { unsigned a0, b0, a1, b1; };
__device__ __forceinline__ RingLaneOff ring_lane_off(const RingLane& rl, unsigned pitch_a, unsigned pitch_b) {
  return {__umul24((unsigned)rl.trow0, pitch_a) + rl.col0, __umul24((unsigned)rl.trow0, pitch_b) + rl.col0,
          __umul24((unsigned)rl.trow1, pitch_a) + rl.col1, __umul24((unsigned)rl.trow1, pitch_b) + rl.col1};
}
// Request the next 64-row tile pair of the segment into LDS stage `stage` (4 copies per wave with 4 waves, 2
// with 8; row pitches in bytes) and advance the feed.  Only the last tile of a segment can be ragged; its
// missing rows repeat the segment's last row.
template <int NW = 4>
__device__ __forceinline__ void ring_feed_issue(const RingLane& rl, const RingLaneOff& lo, RingFeed& f, unsigned pitch_a,
                                                unsigned pitch_b, int wave, bf16_t* stage) {
  if (f.rows >= KT) {
    dma16_off(f.a, lo.a0, stage + wave * 512);
    dma16_off(f.b, lo.b0, stage + KT * SW_LD + wave * 512);
    if (NW == 4) {
      dma16_off(f.a, lo.a1, stage + (4 + wave) * 512);
      dma16_off(f.b, lo.b1, stage + KT * SW_LD + (4 + wave) * 512);
    }
  } else {
    const unsigned r0c = (unsigned)min(rl.trow0, f.rows - 1), r1c = (unsigned)min(rl.trow1, f.rows - 1);
    dma16_off(f.a, __umul24(r0c, pitch_a) + rl.col0, stage + wave * 512);
    dma16_off(f.b, __umul24(r0c, pitch_b) + rl.col0, stage + KT * SW_LD + wave * 512);
    if (NW == 4) {
      dma16_off(f.a, __umul24(r1c, pitch_a) + rl.col1, stage + (4 + wave) * 512);
      dma16_off(f.b, __umul24(r1c, pitch_b) + rl.col1, stage + KT * SW_LD + (4 + wave) * 512);
    }
  }
  f.a += (size_t)KT * pitch_a;
  f.b += (size_t)KT * pitch_b;
  f.rows -= KT;
}
// wait until at most `later` (0 or 1) stages of copies (4 per wave with 4 waves, 2 with 8) requested after the
// wanted one are outstanding, then meet the other waves: the wanted stage is visible to all, and every wave
// has finished reading the stage consumed before it.
template <int NW = 4>
__device__ __forceinline__ void ring_wait(int later) {
  if (later > 0) {
    if (NW == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __builtin_amdgcn_s_barrier();
}

// ------------------------------------------------------------------------------------------
// Forward.  Workgroup = 4 waves; each wave owns QB blocks of 32 query rows.
//
// DH = 64: one head = one 64-column group of the activation rows.
// DH = 8 or 16 ("sub-head" mode, d % 64 == 0): a head is a slice of a 64-column group.  The K/V
// tiles of the whole group are streamed as before; S^T needs only the one 16-deep k-step that
// holds the head's columns (for DH = 8 the Q operand of the other lane half is zero), and
// O^T only the one 32-row block of V^T that holds them.  Per 64-key tile that is 2 + 4 MFMAs per
// query block instead of 8 + 8, and the softmax stays on 32 x 32 accumulator tiles -- about a
// quarter of the VALU instructions of the row-per-lane kernel at these head sizes.
// PAIR: two problems of the same shape in one launch (two encoders side by side; see Geo::pair_B): grid z = 2 B.
template <int QB, int DH, int NST, int WGS, int NW, bool PAIR, bool HEADW = false>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(WGS * NW / 4, WGS * NW / 4))) void mfma_fwd_kernel(Geo g, const bf16_t* __restrict__ QKV, long ld,
                                                       const int32_t* __restrict__ valid_len,
                                                       const uint8_t* __restrict__ key_pad, bf16_t* __restrict__ O,
                                                       long ldo, float* __restrict__ lse2) {
  __shared__ __attribute__((aligned(1024))) bf16_t sT[NST * RING_STAGE];  // per stage: K tile, V tile
  const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: branches on it are wave-uniform
  int tile, h, b;
  xcd_tile_index(g.q_tile_prefix, g.q_nord, g.cu != nullptr, tile, h, b);
  // HEADW (sub-head mode): the NW waves of a workgroup are NW heads of one 64-column group over the SAME 32 QB query
  // rows (grid.y counts groups of NW heads) -- the K/V stream is shared as before, but a tile is 64 rows instead of
  // 256, which at segment lengths like 50 / 500 / 375 leaves 4 % of the rows of the tiles empty instead of 28 %.
  if (HEADW) h = h * NW + wave;
  const bool second = PAIR && b >= g.pair_B;
  const int bm = second ? b - g.pair_B : b;   // batch element of the masks (valid_len, key_pad)
  constexpr int WG_ROWS = HEADW ? 32 * QB : 32 * NW * QB;
  int qs, q0;
  // HALF: the launch may give the query segment with the longest key range tiles of half the height (one query
  // block per wave instead of two), see launch_mfma_fwd; such a workgroup runs the loop below for one block.
  constexpr bool HALF = HEADW && !PAIR && QB == 2;
  bool half_tile = false;
  if (HALF) {
    int k = 0;
    while (k + 1 < g.q_nord && tile >= g.q_tile_prefix[k + 1]) ++k;
    qs = g.q_order[k];
    half_tile = (g.q_half >> k) & 1u;
    q0 = (tile - g.q_tile_prefix[k]) * (half_tile ? WG_ROWS / 2 : WG_ROWS);
  } else {
    decode_tile(second ? g.q_order2 : g.q_order, second ? g.q_tile_prefix2 : g.q_tile_prefix, second ? g.q_nord2 : g.q_nord,
                WG_ROWS, tile, qs, q0);
  }
  const unsigned live = second ? g.q_live2[qs] : g.q_live[qs];   // live key segments of the tile's query segment
  const int qlen = useg_rows(g, b, qs);
  if (q0 >= qlen) return;  // packed rows: this batch element's segment ends before the tile
  const int d = g.d;

  constexpr int NS = DH == 64 ? 4 : 1;    // k-steps of S^T
  constexpr int NDB = DH == 64 ? 2 : 1;   // 32-row blocks of O^T
  const int cg = (h * DH) >> 6;           // 64-column group of this head
  const int wo = (h * DH) & 63;           // first column of the head inside the group
  const int s0 = DH == 64 ? 0 : wo >> 4;  // k-step and O^T block that hold the head (sub-head mode)
  const int db0 = DH == 64 ? 0 : wo >> 5;

  // Q operand (B of S^T = K Q^T): lane holds query row lo of each block, 8 consecutive dh per k-step
  bf16x8 qreg[QB][NS];
  int qrow[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    qrow[qb] = q0 + ((HEADW ? 0 : wave * QB) + qb) * 32 + lo;
    if (HALF && half_tile && qb > 0) qrow[qb] = qlen;   // the next tile's rows: not computed, not stored
    const int rc = min(qrow[qb], qlen - 1);
    const bf16_t* p = QKV + (useg_row0(g, b, qs) + rc) * ld + cg * 64 + hi * 8;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      u32x4 v = *(const u32x4*)(p + (s0 + s) * 16);
      if (DH == 8 && hi != ((wo >> 3) & 1)) v = u32x4{0u, 0u, 0u, 0u};  // the other head of this k-step
      qreg[qb][s] = as_bf16x8(v);
    }
  }

  f32x16 oacc[NDB][QB], nm[QB];
  float m[QB], l[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m[qb] = IM_NEG_INF;
    l[qb] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) nm[qb][r] = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
  }

  const int prow = perm32(lo);
  constexpr float tau = 8.f;  // scores are exponents of 2 (Q carries scale * log2(e))
  // The compiler does not see the asynchronous copies in its vmcnt bookkeeping: consuming the Q
  // registers here makes it wait for their (ordinary) loads now, not inside the ring loop.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int s = 0; s < NS; ++s) asm volatile("" :: "v"(qreg[qb][s]));

  // key tiles of the live key segments; a segment contributes its first min(length, valid length) keys
  auto klen_of = [&](int j) {
    int n = useg_rows(g, b, j);
    if (valid_len) n = min(n, max(0, valid_len[bm * g.n_seg + j]));
    return n;
  };
  const RingLane rl = ring_lane<NW>(wave, lane, cg);
  const unsigned ldb = (unsigned)ld * 2u;
  TileCursor ic = {live, 0, 0, 0}, cc = ic;
  cursor_next_seg(ic, klen_of);
  cursor_next_seg(cc, klen_of);
  int islot = 0, cslot = 0, inflight = 0;
  const RingLaneOff rlo = ring_lane_off(rl, ldb, ldb);
  RingFeed feed = {nullptr, nullptr, 0};
  // K and V rows of segment ic.seg; rows past the valid length but inside the segment are fetched and masked
  auto seg_begin = [&]() {
    feed.a = (const char*)(QKV + useg_row0(g, b, ic.seg) * ld + d);
    feed.b = feed.a + (size_t)d * 2;
    feed.rows = useg_rows(g, b, ic.seg);
  };
  if (ic.len > 0) seg_begin();
  auto issue = [&]() {
    ring_feed_issue<NW>(rl, rlo, feed, ldb, ldb, wave, sT + islot * RING_STAGE);
    islot = (islot + 1 == NST) ? 0 : islot + 1;
    ic.r0 += KT;
    if (ic.r0 >= ic.len) {
      cursor_next_seg(ic, klen_of);
      if (ic.len > 0) seg_begin();
    }
  };
  // NST - 1 stages are requested ahead: the slot refilled in an iteration is the one consumed in the one before
  if (ic.len > 0) { issue(); ++inflight; }
  if (NST > 2 && ic.len > 0) { issue(); ++inflight; }
  // The ring loop, for NQB of the wave's QB query blocks (NQB < QB: a tile of half the height).
  auto ring_loop = [&](auto nqb_tag) {
    constexpr int NQB = decltype(nqb_tag)::value;
    while (cc.len > 0) {
      ring_wait<NW>(inflight - 1);
      if (ic.len > 0) issue(); else --inflight;
      const bf16_t* sK = sT + cslot * RING_STAGE;
      const bf16_t* sV = sK + KT * SW_LD;
      cslot = (cslot + 1 == NST) ? 0 : cslot + 1;
      const int k0 = cc.r0, klen = cc.len;
      const uint8_t* kp_row = key_pad ? key_pad + useg_row0(g, bm, cc.seg) : nullptr;
      cursor_step(cc, klen_of);
      const bool need_mask = (k0 + KT > klen) || (kp_row != nullptr);  // tail tile or key_pad present (wave-uniform)
      unsigned long long km = ~0ull;
      if (need_mask) km = tile_key_mask(kp_row, k0, klen, lane) >> (8 * hi);
      // The tile is processed as two blocks of 32 keys, each S^T -> softmax -> O^T, so that only one block of
      // scores and of probabilities is live at a time.
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        // ---- S^T = K Q^T ----
        // The accumulator chain starts from -m (nm: the running reference of the lane's query row in all 16
        // registers), so the scores leave the matrix cores already relative to it.
        f32x16 sacc[QB];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const bf16x8 a = lds_frag_sw(sK, kb * 32, prow, 2 * (s0 + s) + hi);
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) sacc[qb] = mfma32(a, qreg[qb][s], s == 0 ? nm[qb] : sacc[qb]);
        }
        if (need_mask) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            // register r of block kb on this lane half is key kb*32 + 16*(r/8) + 8*hi + r%8
            const bool ok = (km >> (kb * 32 + 16 * (r >> 3) + (r & 7))) & 1ull;
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) sacc[qb][r] = ok ? sacc[qb][r] : IM_NEG_INF;
          }
        }
        // ---- online softmax, one running (reference, sum) per query row ----
        bf16x8 pb[QB][2];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          // P^T operands of the block from its scores; returns the lane's part of the row sum, taken over the
          // bf16-rounded probabilities (the values that multiply V) with two-element dot products against (1, 1)
          auto exponentiate = [&]() {
            float p[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) p[r] = fast_exp2(sacc[qb][r]);
            pb[qb][0] = pack8(p);
            pb[qb][1] = pack8(p + 8);
            return sum_bf16x8(pb[qb][1], sum_bf16x8(pb[qb][0], 0.f));
          };
          // Almost every block: every row of the wave has a reference already and the scores are exponentiated
          // as they left the matrix cores -- no maximum is taken at all.  fp32 and bf16 share their exponent
          // range, so probabilities far above 1 lose nothing; only a row without a reference yet, or a row sum
          // beyond 2^24 (or inf / NaN), sends the block through the rescaling branch, which recomputes it.
          float rs = exponentiate();
          if (__builtin_expect(__any(m[qb] == IM_NEG_INF || !(rs <= 16777216.f)), 0)) {
            asm volatile("" ::: "memory");  // a real branch: nothing of it is to be executed speculatively
            float mx = sacc[qb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[qb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // block maximum relative to m (the raw maximum while m = -inf)
            // The reference moves when a row has none yet, or when the block maximum exceeds it by more than
            // 2^8 in the exponent domain: accumulator rescale, shifting the block's scores to the new reference
            // and rebuilding nm.
            const bool first = m[qb] == IM_NEG_INF;
            const bool upd = first ? mx > IM_NEG_INF : mx > tau;
            const float shift = upd ? mx : 0.f;
            const float alpha = first ? 0.f : fast_exp2(-shift);
            l[qb] *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
              for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= alpha;
            if (upd) m[qb] = first ? mx : m[qb] + mx;
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[qb][r] -= shift;
            const float nmv = (m[qb] == IM_NEG_INF) ? 0.f : -m[qb];
#pragma unroll
            for (int r = 0; r < 16; ++r) nm[qb][r] = nmv;
            rs = exponentiate();
          }
          l[qb] += rs;
        }
        // ---- O^T += V^T P^T over the 32 keys of the block ----
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const bf16x8 a = lds_frag_tr_sw(sV, kb * 32 + half * 16, (db0 + db) * 32, lane);
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) oacc[db][qb] = mfma32(a, pb[qb][half], oacc[db][qb]);
          }
      }
    }
  };
  if (HALF && half_tile) ring_loop(std::integral_constant<int, 1>{});
  else ring_loop(std::integral_constant<int, QB>{});

  // ---- epilogue: normalise, write O rows, O^T columns and the log-sum-exp ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float lt = l[qb] + __shfl_xor(l[qb], 32, 64);
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const int row = qrow[qb];
    if (row >= qlen) continue;
    const long t = useg_row0(g, b, qs) + row;
    if (hi == 0 && lse2) lse2[useg_stat0(g, b, h, qs) + row] = lt > 0.f ? -(m[qb] + log2f(lt)) : IM_NEG_INF;  // negated
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int dh0 = (db0 + db) * 32 + 8 * i + 4 * hi;  // column inside the 64-column group
        if (DH < 64 && (dh0 < wo || dh0 >= wo + DH)) continue;
        float v[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) v[jj] = oacc[db][qb][4 * i + jj] * inv;
        const u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *(u32x2*)(O + t * ldo + cg * 64 + dh0) = pk;
      }
  }
}

// ------------------------------------------------------------------------------------------
// dQ (and delta = rowsum(dO * O)).  Same ownership as the forward: lane <-> query row.
// The two constant accumulator seeds (negated lse, -delta: 32 registers) put the kernel at 194 registers
// and two workgroups per CU; with them the softmax is exp2, one multiply and the bf16 pack per score, and
// that was measured faster than three workgroups per CU with two more vector instructions per score.
template <int QB, int DH, int NST, int WGS, bool SEED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WGS, WGS))) void mfma_dq_kernel(Geo g, const bf16_t* __restrict__ QKV, long ld,
                                                      const bf16_t* __restrict__ O,
                                                      const bf16_t* __restrict__ dO, long ldo,
                                                      const float* __restrict__ lse2,
                                                      const int32_t* __restrict__ valid_len,
                                                      const uint8_t* __restrict__ key_pad, float* __restrict__ delta,
                                                      bf16_t* __restrict__ dQKV, long ldg) {
  __shared__ __attribute__((aligned(1024))) bf16_t sT[NST * RING_STAGE];  // per stage: K tile, V tile
  const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: branches on it are wave-uniform
  int tile, h, b;
  xcd_tile_index(g.q_tile_prefix, g.q_nord, g.cu != nullptr, tile, h, b);
  constexpr int WG_ROWS = 128 * QB;
  int qs, q0;
  decode_tile(g.q_order, g.q_tile_prefix, g.q_nord, WG_ROWS, tile, qs, q0);
  const int qlen = useg_rows(g, b, qs);
  if (q0 >= qlen) return;  // packed rows: this batch element's segment ends before the tile
  const int d = g.d;

  // sub-head mode (DH = 8 / 16) as in the forward: one k-step for S^T and dP^T, one 32-row block of dQ^T
  constexpr int NS = DH == 64 ? 4 : 1;
  constexpr int NDB = DH == 64 ? 2 : 1;
  const int cg = (h * DH) >> 6, wo = (h * DH) & 63;
  const int s0 = DH == 64 ? 0 : wo >> 4, db0 = DH == 64 ? 0 : wo >> 5;
  const bool other_half = DH == 8 && hi != ((wo >> 3) & 1);  // this lane half holds another head's columns

  bf16x8 qreg[QB][NS], greg[QB][NS];
  int qrow[QB];
  float ls[QB], dl[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    qrow[qb] = q0 + (wave * QB + qb) * 32 + lo;
    const int rc = min(qrow[qb], qlen - 1);
    const long t = useg_row0(g, b, qs) + rc;
    const bf16_t* p = QKV + t * ld + cg * 64 + hi * 8;
    const bf16_t* pg = dO + t * ldo + cg * 64 + hi * 8;
    const bf16_t* po = O + t * ldo + cg * 64 + hi * 8;
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      u32x4 qv = *(const u32x4*)(p + (s0 + s) * 16);
      u32x4 gv = *(const u32x4*)(pg + (s0 + s) * 16);
      const u32x4 ov = *(const u32x4*)(po + (s0 + s) * 16);
      if (other_half) { qv = u32x4{0u, 0u, 0u, 0u}; gv = qv; }
      qreg[qb][s] = as_bf16x8(qv);
      greg[qb][s] = as_bf16x8(gv);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = fmaf(__uint_as_float(gv[e] << 16), __uint_as_float(ov[e] << 16), acc);
        acc = fmaf(__uint_as_float(gv[e] & 0xffff0000u), __uint_as_float(ov[e] & 0xffff0000u), acc);
      }
    }
    acc += __shfl_xor(acc, 32, 64);
    dl[qb] = acc;
    const long li = useg_stat0(g, b, h, qs) + rc;
    const float lv = lse2[li];
    ls[qb] = lv;  // negated log2-sum-exp; -inf for a row without valid keys: every probability is exactly zero
    if (hi == 0 && qrow[qb] < qlen) delta[li] = DH == 64 ? -acc : acc;  // see the dK/dV kernel
  }

  f32x16 dqacc[NDB][QB], nlb[QB], ndb[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dqacc[db][qb][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) { nlb[qb][r] = SEED ? ls[qb] : 0.f; ndb[qb][r] = SEED ? -dl[qb] : 0.f; }
  }

  const int prow = perm32(lo);
  // The compiler does not see the asynchronous copies in its vmcnt bookkeeping: consuming the
  // loaded registers here makes it wait for their (ordinary) loads now, not inside the ring loop.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
    for (int s = 0; s < NS; ++s) asm volatile("" :: "v"(qreg[qb][s]), "v"(greg[qb][s]));
    asm volatile("" :: "v"(ls[qb]), "v"(dl[qb]));
  }

  auto klen_of = [&](int j) {
    int n = useg_rows(g, b, j);
    if (valid_len) n = min(n, max(0, valid_len[b * g.n_seg + j]));
    return n;
  };
  const RingLane rl = ring_lane(wave, lane, cg);
  const unsigned ldb = (unsigned)ld * 2u;
  TileCursor ic = {g.q_live[qs], 0, 0, 0}, cc = ic;
  cursor_next_seg(ic, klen_of);
  cursor_next_seg(cc, klen_of);
  int islot = 0, cslot = 0, inflight = 0;
  const RingLaneOff rlo = ring_lane_off(rl, ldb, ldb);
  RingFeed feed = {nullptr, nullptr, 0};
  // K and V rows of segment ic.seg; rows past the valid length but inside the segment are fetched and masked
  auto seg_begin = [&]() {
    feed.a = (const char*)(QKV + useg_row0(g, b, ic.seg) * ld + d);
    feed.b = feed.a + (size_t)d * 2;
    feed.rows = useg_rows(g, b, ic.seg);
  };
  if (ic.len > 0) seg_begin();
  auto issue = [&]() {
    ring_feed_issue(rl, rlo, feed, ldb, ldb, wave, sT + islot * RING_STAGE);
    islot = (islot + 1 == NST) ? 0 : islot + 1;
    ic.r0 += KT;
    if (ic.r0 >= ic.len) {
      cursor_next_seg(ic, klen_of);
      if (ic.len > 0) seg_begin();
    }
  };
  if (ic.len > 0) { issue(); ++inflight; }
  if (NST > 2 && ic.len > 0) { issue(); ++inflight; }
  while (cc.len > 0) {
    ring_wait(inflight - 1);
    if (ic.len > 0) issue(); else --inflight;
    const bf16_t* sK = sT + cslot * RING_STAGE;
    const bf16_t* sV = sK + KT * SW_LD;
    cslot = (cslot + 1 == NST) ? 0 : cslot + 1;
    const int k0 = cc.r0, klen = cc.len;
    const uint8_t* kp_row = key_pad ? key_pad + useg_row0(g, b, cc.seg) : nullptr;
    cursor_step(cc, klen_of);
    {
      const bool need_mask = (k0 + KT > klen) || (kp_row != nullptr);
      unsigned long long km = ~0ull;
      if (need_mask) km = tile_key_mask(kp_row, k0, klen, lane) >> (8 * hi);
      // two blocks of 32 keys, each S^T, dP^T -> dS^T -> dQ^T, so that one block of dS^T is live at a time
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        bf16x8 dsb[QB][2];
        // The chains start from the row's negated lse resp. -delta (nlb, ndb: the lane's value in all 16
        // registers), so they end as S^T - lse and dP^T - delta.
        f32x16 sacc[QB], pacc[QB];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const bf16x8 ak = lds_frag_sw(sK, kb * 32, prow, 2 * (s0 + s) + hi);
          const bf16x8 av = lds_frag_sw(sV, kb * 32, prow, 2 * (s0 + s) + hi);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            sacc[qb] = mfma32(ak, qreg[qb][s], s == 0 ? nlb[qb] : sacc[qb]);   // S^T  = K Q^T
            pacc[qb] = mfma32(av, greg[qb][s], s == 0 ? ndb[qb] : pacc[qb]);   // dP^T = V dO^T
          }
        }
        if (need_mask) {  // wave-uniform: tail tile or key_pad present
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              sacc[qb][r] = ((km >> (kb * 32 + 16 * (r >> 3) + (r & 7))) & 1ull) ? sacc[qb][r] : IM_NEG_INF;
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          float ds[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = fast_exp2(SEED ? sacc[qb][r] : sacc[qb][r] + ls[qb]);
            ds[r] = p * (SEED ? pacc[qb][r] : pacc[qb][r] - dl[qb]);
          }
          dsb[qb][0] = pack8(ds);
          dsb[qb][1] = pack8(ds + 8);
        }
        // dQ^T += K^T dS^T over the 32 keys of the block
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const bf16x8 a = lds_frag_tr_sw(sK, kb * 32 + half * 16, (db0 + db) * 32, lane);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) dqacc[db][qb] = mfma32(a, dsb[qb][half], dqacc[db][qb]);
          }
      }
    }
  }

#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = qrow[qb];
    if (row >= qlen) continue;
    const long t = useg_row0(g, b, qs) + row;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int dh0 = (db0 + db) * 32 + 8 * i + 4 * hi;  // column inside the 64-column group
        if (DH < 64 && (dh0 < wo || dh0 >= wo + DH)) continue;
        float v[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) v[jj] = dqacc[db][qb][4 * i + jj] * g.scale;
        const u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *(u32x2*)(dQKV + t * ldg + cg * 64 + dh0) = pk;
      }
  }
}

// ------------------------------------------------------------------------------------------
// dK, dV.  Each wave owns KB blocks of 32 key rows (lane <-> key row) and streams
// the query rows of every query segment that reads this key segment.  A key tile
// has exactly one producer, so the result is deterministic without atomics.
//
// Ring stage = Q tile, dO tile (see RING_STAGE) plus the 64 lse and 64 delta values of the rows.
// At head dim 64 the delta buffer holds -delta (the dQ kernel writes it so): the dP accumulator
// starts from it, so the MFMA chain ends as dP - delta and no separate subtraction is needed.
__device__ const float k_neg_inf = -__builtin_inff();

template <int KB, int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void mfma_dkv_kernel(Geo g, const bf16_t* __restrict__ QKV, long ld,
                                                       const bf16_t* __restrict__ dO, long ldo,
                                                       const float* __restrict__ lse2, const float* __restrict__ delta,
                                                       const int32_t* __restrict__ valid_len,
                                                       const uint8_t* __restrict__ key_pad, bf16_t* __restrict__ dQKV,
                                                       long ldg) {
  __shared__ __attribute__((aligned(1024))) bf16_t sT[RING_NST * RING_STAGE];
  __shared__ __attribute__((aligned(256))) float sLD[RING_NST * 2 * KT];  // per stage: lse[64], delta[64]
  const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: branches on it are wave-uniform
  int tile, h, b;
  xcd_tile_index(g.k_tile_prefix, g.k_nord, g.cu != nullptr, tile, h, b);
  constexpr int WG_ROWS = 128 * KB;
  int ks, k0;
  decode_tile(g.k_order, g.k_tile_prefix, g.k_nord, WG_ROWS, tile, ks, k0);
  const int klen_seg = useg_rows(g, b, ks);
  if (k0 >= klen_seg) return;  // packed rows: this batch element's segment ends before the tile
  const int d = g.d;

  // sub-head mode (DH = 8 / 16): one k-step for S and dP, one 32-row block of dV^T and dK^T
  constexpr int NS = DH == 64 ? 4 : 1;
  constexpr int NDB = DH == 64 ? 2 : 1;
  const int cg = (h * DH) >> 6, wo = (h * DH) & 63;
  const int s0 = DH == 64 ? 0 : wo >> 4, db0 = DH == 64 ? 0 : wo >> 5;
  const bool other_half = DH == 8 && hi != ((wo >> 3) & 1);  // this lane half holds another head's columns

  auto qlen_of = [&](int i) { return useg_rows(g, b, i); };
  const RingLane rl = ring_lane(wave, lane, cg);
  const unsigned ldb = (unsigned)ld * 2u, ldob = (unsigned)ldo * 2u;  // row pitches in bytes
  TileCursor ic = {g.k_live[ks], 0, 0, 0}, cc = ic;
  cursor_next_seg(ic, qlen_of);
  cursor_next_seg(cc, qlen_of);
  int islot = 0, cslot = 0, inflight = 0;
  const RingLaneOff rlo = ring_lane_off(rl, ldb, ldob);
  RingFeed feed = {nullptr, nullptr, 0};
  const float* feed_l = nullptr;  // lse and delta of the next tile's first row
  const float* feed_d = nullptr;
  auto seg_begin = [&]() {  // Q and dO rows, lse and delta of segment ic.seg
    const long row0 = useg_row0(g, b, ic.seg);
    const long lb = useg_stat0(g, b, h, ic.seg);
    feed.a = (const char*)(QKV + row0 * ld);
    feed.b = (const char*)(dO + row0 * ldo);
    feed.rows = ic.len;
    feed_l = lse2 + lb;
    feed_d = delta + lb;
  };
  if (ic.len > 0) seg_begin();
  auto issue = [&]() {
    // negated lse (wave 0) and delta (wave 1), one float per lane.  Rows past the segment read -inf
    // as negated lse, so their probabilities are exactly zero.
    if (wave < 2) {
      float* dst = sLD + islot * 2 * KT + wave * KT;
      if (feed.rows >= KT) {
        dma4_off(wave == 0 ? feed_l : feed_d, (unsigned)lane * 4u, dst);
      } else {
        const float* src = (wave == 0) ? (lane < feed.rows ? feed_l + lane : &k_neg_inf) : feed_d + min(lane, feed.rows - 1);
        dma4(src, dst);
      }
    }
    feed_l += KT;
    feed_d += KT;
    ring_feed_issue(rl, rlo, feed, ldb, ldob, wave, sT + islot * RING_STAGE);
    islot = (islot + 1 == RING_NST) ? 0 : islot + 1;
    ic.r0 += KT;
    if (ic.r0 >= ic.len) {
      cursor_next_seg(ic, qlen_of);
      if (ic.len > 0) seg_begin();
    }
  };

  bf16x8 kreg[KB][NS], vreg[KB][NS];
  int krow[KB];
  bool kvalid[KB];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    krow[kb] = k0 + (wave * KB + kb) * 32 + lo;
    const int rc = min(krow[kb], klen_seg - 1);
    const long t = useg_row0(g, b, ks) + rc;
    const bf16_t* p = QKV + t * ld + d + cg * 64 + hi * 8;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      u32x4 kv = *(const u32x4*)(p + (s0 + s) * 16), vv = *(const u32x4*)(p + d + (s0 + s) * 16);
      if (other_half) { kv = u32x4{0u, 0u, 0u, 0u}; vv = kv; }
      kreg[kb][s] = as_bf16x8(kv);
      vreg[kb][s] = as_bf16x8(vv);
    }
    bool ok = krow[kb] < klen_seg;
    if (ok && valid_len) ok = krow[kb] < valid_len[b * g.n_seg + ks];
    if (ok && key_pad) ok = key_pad[t] == 0;
    kvalid[kb] = ok;
  }

  f32x16 dkacc[NDB][KB], dvacc[NDB][KB];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) { dkacc[db][kb][r] = 0.f; dvacc[db][kb][r] = 0.f; }

  // The compiler does not see the asynchronous copies in its vmcnt bookkeeping.  Consuming the
  // K / V registers here makes it wait for their (ordinary) loads now, before the ring starts,
  // instead of draining the ring with a vmcnt(0) at their first use inside the loop.
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int s = 0; s < NS; ++s) asm volatile("" :: "v"(kreg[kb][s]), "v"(vreg[kb][s]));

  if (ic.len > 0) { issue(); ++inflight; }
  if (ic.len > 0) { issue(); ++inflight; }

  const int prow = perm32(lo);
  while (cc.len > 0) {
    // Copies complete in issue order.  The wanted stage is complete once at most the copies of the
    // stage requested after it (4 tile chunks, plus 1 on the waves that fetch lse / delta) are
    // outstanding.
    if (inflight > 1) {
      if (wave < 2) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();  // stage visible to all waves; everyone is done with the one before
    if (ic.len > 0) issue(); else --inflight;  // refills the slot of the stage consumed before
    const bf16_t* sQ = sT + cslot * RING_STAGE;
    const bf16_t* sG = sQ + KT * SW_LD;
    const float* sL = sLD + cslot * 2 * KT;
    const float* sD = sL + KT;
    cslot = (cslot + 1 == RING_NST) ? 0 : cslot + 1;
    cursor_step(cc, qlen_of);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      // negated lse / delta of the query rows of the block: register r of an accumulator holds row
      // (r / 8) * 16 + hi * 8 + r % 8.  At head dim 64 both go straight into the accumulators (the delta buffer
      // holds -delta): the MFMA chains then end as S - lse and dP - delta, and neither needs a vector
      // instruction per element.  In sub-head mode they are fetched four rows at a time where they are used.
      auto rows4 = [&](const float* base, int r4) {   // values of registers 4 r4 .. 4 r4 + 3
        return *(const float4*)&base[qb * 32 + (r4 >> 1) * 16 + hi * 8 + (r4 & 1) * 4];
      };
      bf16x8 pb[KB][2], dsb[KB][2];
      f32x16 sacc[KB], pacc[KB];
      float D[16], NL[16];
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const float4 d4 = rows4(sD, r4);
        D[4 * r4] = d4.x; D[4 * r4 + 1] = d4.y; D[4 * r4 + 2] = d4.z; D[4 * r4 + 3] = d4.w;
        if (DH == 64) {
          const float4 l4 = rows4(sL, r4);
          NL[4 * r4] = l4.x; NL[4 * r4 + 1] = l4.y; NL[4 * r4 + 2] = l4.z; NL[4 * r4 + 3] = l4.w;
        }
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[kb][r] = DH == 64 ? NL[r] : 0.f; pacc[kb][r] = DH == 64 ? D[r] : 0.f; }
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const bf16x8 aq = lds_frag_sw(sQ, qb * 32, prow, 2 * (s0 + s) + hi);
        const bf16x8 ag = lds_frag_sw(sG, qb * 32, prow, 2 * (s0 + s) + hi);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          sacc[kb] = mfma32(aq, kreg[kb][s], sacc[kb]);   // S  = Q K^T
          pacc[kb] = mfma32(ag, vreg[kb][s], pacc[kb]);   // dP = dO V^T
        }
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        float p[16], ds[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          float L[4] = {0.f, 0.f, 0.f, 0.f};
          if (DH != 64) {
            const float4 l4 = rows4(sL, r4);
            L[0] = l4.x; L[1] = l4.y; L[2] = l4.z; L[3] = l4.w;
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int r = 4 * r4 + u;
            p[r] = DH == 64 ? fast_exp2(sacc[kb][r]) : fast_exp2(sacc[kb][r] + L[u]);
            ds[r] = DH == 64 ? p[r] * pacc[kb][r] : p[r] * (pacc[kb][r] - D[r]);
          }
        }
        pb[kb][0] = pack8(p); pb[kb][1] = pack8(p + 8);
        dsb[kb][0] = pack8(ds); dsb[kb][1] = pack8(ds + 8);
      }
      // dV^T += dO^T P ; dK^T += Q^T dS   (contraction over the 32 query rows of this block)
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const bf16x8 agt = lds_frag_tr_sw(sG, qb * 32 + half * 16, (db0 + db) * 32, lane);
          const bf16x8 aqt = lds_frag_tr_sw(sQ, qb * 32 + half * 16, (db0 + db) * 32, lane);
#pragma unroll
          for (int kb = 0; kb < KB; ++kb) {
            dvacc[db][kb] = mfma32(agt, pb[kb][half], dvacc[db][kb]);
            dkacc[db][kb] = mfma32(aqt, dsb[kb][half], dkacc[db][kb]);
          }
        }
    }
  }

#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    const int row = krow[kb];
    if (row >= klen_seg) continue;
    const long t = useg_row0(g, b, ks) + row;
    // dK = scale dS^T Q, and the staged Q rows are scale log2(e) Q: the accumulator needs a factor ln 2
    const float zk = kvalid[kb] ? 0.69314718055994530942f : 0.f, zv = kvalid[kb] ? 1.f : 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int dh0 = (db0 + db) * 32 + 8 * i + 4 * hi;  // column inside the 64-column group
        if (DH < 64 && (dh0 < wo || dh0 >= wo + DH)) continue;
        const u32x2 pk = {pack_bf16(dkacc[db][kb][4 * i] * zk, dkacc[db][kb][4 * i + 1] * zk),
                          pack_bf16(dkacc[db][kb][4 * i + 2] * zk, dkacc[db][kb][4 * i + 3] * zk)};
        const u32x2 pv = {pack_bf16(dvacc[db][kb][4 * i] * zv, dvacc[db][kb][4 * i + 1] * zv),
                          pack_bf16(dvacc[db][kb][4 * i + 2] * zv, dvacc[db][kb][4 * i + 3] * zv)};
        *(u32x2*)(dQKV + t * ldg + d + cg * 64 + dh0) = pk;
        *(u32x2*)(dQKV + t * ldg + 2 * d + cg * 64 + dh0) = pv;
      }
  }
}

// ---- host launchers ----
// Launch shapes, each chosen by measurement at B = 8, segments 512 / 2048 / 2048, d = 512, 8 heads:
//   forward, head dim 64: 1 query block per wave, 4 waves, a 2-stage ring and 128 registers, so that four
//     workgroups (16 waves) share a CU -- 10 % faster than 3 stages at three workgroups; 8-wave workgroups
//     (256 query rows) were slower;
//   forward, sub-head mode: 2 query blocks per wave (half the K/V tile traffic per score), 3 stages, 3 workgroups;
//   dQ, head dim 64: 3 stages, 3 workgroups per CU, accumulators seeded with -lse and -delta (unseeded: 7 % slower;
//     4 workgroups need spills);
//   dQ, sub-head mode: 3 workgroups per CU as well (114 registers; 27 against 33 us with two at B = 32, 50 / 500 / 375
//     rows, 8 heads of 8);
//   dK/dV: 1 key block per wave, 3 workgroups per CU at head dim 64, 2 in sub-head mode (3 measured the same).
constexpr int FWD_QB = 1, FWD_QB_SUB = 2, DQ_QB = 1, DKV_KB = 1;
constexpr int FWD_NST = 2, FWD_WGS = 4, FWD_NW = 4;   // ring stages, workgroups per CU, waves per workgroup (head dim 64)
constexpr int FWD_SUB_NST = 3, FWD_SUB_WGS = 3;       // the same in sub-head mode (4 waves)
constexpr int DQ_NST = 3, DQ_WGS = 3;                 // dQ at head dim 64
// sub-head mode with a multiple of 4 heads: four heads of a 64-column group per workgroup, 64-row tiles
static bool fwd_headw(int dh, int H) { return dh != 64 && H % 4 == 0; }
int mfma_fwd_tile_rows(int dh, int H) { return dh == 64 ? 32 * FWD_NW * FWD_QB : fwd_headw(dh, H) ? 32 * FWD_QB_SUB : 128 * FWD_QB_SUB; }
int mfma_dq_tile_rows() { return 128 * DQ_QB; }
int mfma_dkv_tile_rows() { return 128 * DKV_KB; }

// Sub-head forward with four heads per workgroup, padded rows.  The workgroups of the query segment with the longest
// key range finish last; when they are few (at most a quarter of the workgroup slots -- segments 50 / 500 / 375 under
// the forward inter-modal mask: the one tile of the 50 text rows reads 500 keys, the eight tiles of the vision rows
// 375) and clearly the longest, their tiles become 32 rows tall: twice the workgroups, one query block per wave,
// a shorter tail of the launch (measured: -3 % at that shape).  A half-height workgroup does more work per score (the
// K/V fragments are read per block), so a launch whose long workgroups are many -- it is bound by the CUs'
// instruction issue, not by its last workgroup -- keeps the full tiles (halving them there measured +3 %).
static int device_cus() {
  static int cus = 0;   // compute units of the device (the first device that launches; one GPU per process)
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
    else cus = 256;
  }
  return cus;
}
static void fwd_half_tiles(Geo& g) {
  g.q_half = 0;
  if (g.cu || g.q_nord < 2) return;
  const int rows = 32 * FWD_QB_SUB;
  const long units = (long)g.B * (g.H / 4), slots = (long)FWD_SUB_WGS * device_cus();
  long len[IM_MAX_SEG], tiles[IM_MAX_SEG];
  int longest = 0;
  for (int k = 0; k < g.q_nord; ++k) {
    const int sgm = g.q_order[k];
    len[k] = 0;
    for (int j = 0; j < g.n_seg; ++j)
      if ((g.q_live[sgm] >> j) & 1u) len[k] += (g.seg_len[j] + KT - 1) / KT;
    tiles[k] = (g.seg_len[sgm] + rows - 1) / rows;
    if (len[k] > len[longest]) longest = k;
  }
  long second = 0;
  for (int k = 0; k < g.q_nord; ++k)
    if (k != longest && len[k] > second) second = len[k];
  if (4 * len[longest] < 5 * second || 4 * tiles[longest] * units > slots) return;
  const long half_tiles = (g.seg_len[g.q_order[longest]] + rows / 2 - 1) / (rows / 2);
  g.q_half = 1u << longest;
  for (int k = 0; k < g.q_nord; ++k)
    g.q_tile_prefix[k + 1] = g.q_tile_prefix[k] + (int)(k == longest ? half_tiles : tiles[k]);
}

void launch_mfma_fwd(const Geo& g_in, const bf16_t* qkv, long ld, const int32_t* valid_len, const uint8_t* key_pad,
                     bf16_t* o, long ldo, float* lse2, hipStream_t st) {
  Geo g = g_in;
  g.q_half = 0;
  if (fwd_headw(g.dh, g.H)) fwd_half_tiles(g);
  // query segments with no live block: output 0, lse -inf
  for (int s = 0; s < g.n_seg; ++s) {
    if (g.q_live[s]) continue;
    launch_zero_seg_rows(g, s, 1, o, ldo, 0, g.d, st);
    if (lse2) launch_fill_seg_stat(g, s, lse2, -__builtin_inff(), st);
  }
  const int nt = g.q_tile_prefix[g.q_nord];
  if (nt == 0) return;
  ProfScope ps(PF_ATTN_FWD, st);
  const dim3 grid(nt, g.H, g.B), gridw(nt, g.H / 4, g.B);
  const bool hw = fwd_headw(g.dh, g.H);
  if (g.dh == 64) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB, 64, FWD_NST, FWD_WGS, FWD_NW, false>), grid, dim3(64 * FWD_NW), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else if (g.dh == 16 && hw) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 16, FWD_SUB_NST, FWD_SUB_WGS, 4, false, true>), gridw, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else if (hw) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 8, FWD_SUB_NST, FWD_SUB_WGS, 4, false, true>), gridw, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else if (g.dh == 16) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 16, FWD_SUB_NST, FWD_SUB_WGS, 4, false>), grid, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 8, FWD_SUB_NST, FWD_SUB_WGS, 4, false>), grid, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
}

// Forward of two problems of the same shape (masks g0 / g1) in one launch; their rows follow each other in
// qkv, o and lse2 (2 B batch elements).  Sub-head mode and padded rows only; both masks must give every query
// segment a live block (same tile count), which the caller checks with mfma_fwd_pair_ok.
bool mfma_fwd_pair_ok(const Geo& g0, const Geo& g1) {
  if (g0.dh == 64 || g0.cu || g1.cu || g0.q_tile_prefix[g0.q_nord] != g1.q_tile_prefix[g1.q_nord]) return false;
  for (int s = 0; s < g0.n_seg; ++s)
    if (!g0.q_live[s] || !g1.q_live[s]) return false;
  return 2L * g0.B <= 65535;
}
void launch_mfma_fwd_pair(const Geo& g0, const Geo& g1, const bf16_t* qkv, long ld, const int32_t* valid_len,
                          const uint8_t* key_pad, bf16_t* o, long ldo, float* lse2, hipStream_t st) {
  Geo g = g0;
  g.pair_B = g0.B;
  g.q_nord2 = g1.q_nord;
  for (int i = 0; i < IM_MAX_SEG; ++i) { g.q_live2[i] = g1.q_live[i]; g.q_order2[i] = g1.q_order[i]; }
  for (int i = 0; i <= IM_MAX_SEG; ++i) g.q_tile_prefix2[i] = g1.q_tile_prefix[i];
  ProfScope ps(PF_ATTN_FWD, st);
  const dim3 grid(g.q_tile_prefix[g.q_nord], g.H, 2 * g.B), gridw(g.q_tile_prefix[g.q_nord], g.H / 4, 2 * g.B);
  const bool hw = fwd_headw(g.dh, g.H);
  if (g.dh == 16 && hw) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 16, FWD_SUB_NST, FWD_SUB_WGS, 4, true, true>), gridw, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else if (hw) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 8, FWD_SUB_NST, FWD_SUB_WGS, 4, true, true>), gridw, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else if (g.dh == 16) hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 16, FWD_SUB_NST, FWD_SUB_WGS, 4, true>), grid, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
  else hipLaunchKernelGGL((mfma_fwd_kernel<FWD_QB_SUB, 8, FWD_SUB_NST, FWD_SUB_WGS, 4, true>), grid, dim3(256), 0, st, g, qkv, ld, valid_len, key_pad, o, ldo, lse2);
}

void launch_mfma_bwd(const Geo& g, const bf16_t* qkv, long ld, const bf16_t* o, const bf16_t* d_o, long ldo,
                     const float* lse2, const int32_t* valid_len, const uint8_t* key_pad, float* delta, bf16_t* dqkv,
                     long ldg, hipStream_t st) {
  for (int s = 0; s < g.n_seg; ++s) {
    if (!g.q_live[s])
      launch_zero_seg_rows(g, s, 1, dqkv, ldg, 0, g.d, st);
    if (!g.k_live[s])
      launch_zero_seg_rows(g, s, 1, dqkv, ldg, g.d, 2 * g.d, st);
  }
  const int nq = g.q_tile_prefix[g.q_nord], nk = g.k_tile_prefix[g.k_nord];
  if (nq == 0) return;
  { ProfScope ps(PF_ATTN_DQ, st);
    const dim3 grid(nq, g.H, g.B);
    if (g.dh == 64) hipLaunchKernelGGL((mfma_dq_kernel<DQ_QB, 64, DQ_NST, DQ_WGS, true>), grid, dim3(256), 0, st, g, qkv, ld, o, d_o, ldo, lse2, valid_len, key_pad, delta, dqkv, ldg);
    else if (g.dh == 16) hipLaunchKernelGGL((mfma_dq_kernel<DQ_QB, 16, 3, 3, true>), grid, dim3(256), 0, st, g, qkv, ld, o, d_o, ldo, lse2, valid_len, key_pad, delta, dqkv, ldg);
    else hipLaunchKernelGGL((mfma_dq_kernel<DQ_QB, 8, 3, 3, true>), grid, dim3(256), 0, st, g, qkv, ld, o, d_o, ldo, lse2, valid_len, key_pad, delta, dqkv, ldg); }
  { ProfScope ps(PF_ATTN_DKV, st);
    const dim3 grid(nk, g.H, g.B);
    if (g.dh == 64) hipLaunchKernelGGL((mfma_dkv_kernel<DKV_KB, 64>), grid, dim3(256), 0, st, g, qkv, ld, d_o, ldo, lse2, delta, valid_len, key_pad, dqkv, ldg);
    else if (g.dh == 16) hipLaunchKernelGGL((mfma_dkv_kernel<DKV_KB, 16>), grid, dim3(256), 0, st, g, qkv, ld, d_o, ldo, lse2, delta, valid_len, key_pad, dqkv, ldg);
    else hipLaunchKernelGGL((mfma_dkv_kernel<DKV_KB, 8>), grid, dim3(256), 0, st, g, qkv, ld, d_o, ldo, lse2, delta, valid_len, key_pad, dqkv, ldg); }
}

}  // namespace imattn
