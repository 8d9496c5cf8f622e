// bf16 MFMA kernel for every blocked-softmax pass of spatio-temporal Monarch attention on gfx950,
// with one wave per SIMD and two 32-query tiles per wave: the R-update of a fitting sweep
// (Eq. R + Eq. alpha_L/c_L: logits, alpha_L = R K and c_L), the R-update of the last sweep (the
// same plus y = R V of App. A, from ONE evaluation of the logits and of the softmax) and the
// first-frame recomputation (Sec. 3.3).  All three are Alg. 1 with the running max / sum /
// entropy of App. B.
//
// One workgroup = 4 waves = 256 query rows; a wave owns 64 query rows (two tiles of 32) for the
// whole key loop and the full register file of its SIMD (512 registers), which is what lets one
// wave hold both accumulator sets (R K and R V: 2 x 2 x 4 tiles of 16 registers) beside its
// queries and logits.  Keys (and values) stream through LDS in 64-row tiles, four slots per
// tensor, loaded two tiles ahead.  Both contractions use v_mfma_f32_32x32x16_bf16:
//
//   S^T = K Q^T     A = K rows read from LDS (ds_read_b128), B = Q^T held in registers.  One A
//                   operand serves both query tiles: half the LDS bytes per MFMA of a
//                   one-tile wave.  In the result lane (q, g) holds the logits of query q for
//                   16 of the 32 keys, so max, sum and entropy are per-lane scalars and need
//                   one exchange with lane^32 for the max only.
//   O^T += X^T P^T  A = X^T (X = K for alpha_L, X = V for y) fetched from the same row-major
//                   LDS tile with the LDS transpose read (ds_read_b64_tr_b16), again shared by
//                   both query tiles; B = P^T, the S^T accumulator converted to bf16 in place.
//
// The 16-byte chunk c of key row r is stored at chunk c ^ swz(r) (RowGeo in common.h) so that
// both the row-wise b128 reads and the transpose reads spread over all banks.
#include "../../include/vmonarch.h"
#include <type_traits>

#include "common.h"
#include "flash_device.h"

namespace vm {

namespace {

constexpr int W2 = 4;             // waves per workgroup, one per SIMD
constexpr int Q2 = 2;             // 32-query tiles per wave
constexpr int BQ2 = 32 * Q2 * W2;  // query rows per workgroup
// A reference max moves only when a row maximum outgrew it by 2^32.  The probabilities are formed in fp32 and
// rounded to bf16, which has fp32's exponent range, and the sums are fp32, so a stale reference costs the
// outputs no precision until 2^t nears overflow.  c_L needs one precaution: h = sum p t and l = sum p must
// weigh every key alike, or their mismatch (about 1e-3 relative when l holds the bf16-rounded p and h the
// unrounded ones) is multiplied by the mean of t, which a stale reference lets grow to 32; so h is summed with
// the ROUNDED p here.  Moving a reference is expensive in this kernel (the accumulators sit in accumulation
// registers and pass through ordinary ones to be rescaled), and in the last sweep's update, where c_R
// sharpens some rows tenfold, a margin of 2^8 would move one in most steps.
constexpr float RESCALE_TH2 = 32.0f;
// Where a moving reference is put: this far (log2 units) above the row maximum that moved it, the first one
// included.  Any reference gives the same results (the sums and the accumulators carry the common factor
// 2^-reference, and fp32 / bf16 have exponent range to spare: the largest probability of a row is then 2^-64, keys
// more than 2^-62 below the row maximum flush to zero); a high one makes later moves rare, which matters where
// attention is sharp (logits many times their usual spread: row maxima then jump by more than 2^32 from tile to tile).
constexpr float HEADROOM2 = 64.0f;

__device__ __forceinline__ uint32_t avg_bf16x2(uint32_t a, uint32_t b) {
  const float lo = 0.5f * (__uint_as_float(a << 16) + __uint_as_float(b << 16));
  const float hi = 0.5f * (__uint_as_float(a & 0xffff0000u) + __uint_as_float(b & 0xffff0000u));
  return pack_bf16(lo, hi);
}
__device__ __forceinline__ uint4 avg_bf16x8(uint4 a, uint4 b) {
  return make_uint4(avg_bf16x2(a.x, b.x), avg_bf16x2(a.y, b.y), avg_bf16x2(a.z, b.z), avg_bf16x2(a.w, b.w));
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Nothing moves across this line in the instruction schedule.
#define F2_FENCE() __builtin_amdgcn_sched_barrier(0)
// The hardware does not interlock an MFMA's result against plain vector instructions: passes + 3 = 11 issue
// slots must lie between the issue of this 8-pass MFMA and the first instruction that reads (or
// overwrites) what it writes.  The MFMAs of this kernel are inline assembly, which the compiler's hazard
// handling cannot see, so wherever vector code follows an MFMA closely this wait is written out.
#define F2_MFMA_RESULT_WAIT() asm volatile("s_nop 7\n\ts_nop 3" ::: "memory")

template <int D, bool OUT_K, bool OUT_V, int ENT, bool SPLIT>
__global__ void __launch_bounds__(64 * W2) flash2_kernel(FlashParams P) {
  using G = RowGeo<D>;
  constexpr int ROW_BYTES = G::ROW_BYTES;
  constexpr int TILE_BYTES = BK * ROW_BYTES;  // 16 KB (d = 128) or 8 KB (d = 64)
  constexpr int KS = G::KS;                   // k-steps of S^T = K Q^T
  constexpr int CT = G::CT;                   // 32-channel tiles of an output row
  constexpr int CH = G::CH;                   // 16-byte chunks per row
  constexpr int RPI = G::RPI;                 // rows filled by one 64-lane global -> LDS load
  constexpr int V_OFF = NSLOT * TILE_BYTES;   // the V slots follow the K slots
  constexpr int NX = (OUT_K ? 1 : 0) + (OUT_V ? 1 : 0);  // accumulator sets: [R K][R V]
  constexpr int XV = OUT_K ? 1 : 0;                       // index of the R V set
  static_assert(OUT_K || OUT_V, "at least one product");
  static_assert(Q2 == 2, "the schedule below is written for two query tiles");
  auto swz = [](int row) { return G::swz(row); };
  extern __shared__ __attribute__((aligned(16))) char smem[];  // [K|V][NSLOT][64 rows][2 D bytes]

  // XCD-aware placement: hardware deals workgroups to the 8 XCDs round-robin, so give each
  // XCD one contiguous range of work items; the query blocks of one (head, frame) then share
  // that XCD's L2 copy of the frame's K and V.
  const int bid = blockIdx.x;
  const int wid = (bid & 7) * P.blocks_per_xcd + (bid >> 3);
  if (wid >= P.total_blocks) return;
  const int per_problem = P.nqb * P.nsplit;
  const int prob = wid / per_problem;
  const int rem = wid - prob * per_problem;
  // the query blocks of one key range are neighbours: they stream the same K and V tiles at
  // the same time and share them through the XCD's L2
  const int split = rem / P.nqb;
  const int qb = rem - split * P.nqb;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int ql = lane & 31;
  const int g = lane >> 5;

  const int kbeg = split * P.keys_per_split;
  const int kend = min(P.nk, kbeg + P.keys_per_split);
  const int nkeys = kend - kbeg;
  const int ntiles = (nkeys + BK - 1) / BK;
  const int last_left = nkeys - (ntiles - 1) * BK;  // 1..64 keys in the last tile
  // The key loop can visit the tiles in rotated order, tile (i + first) mod ntiles at loop position i: any order
  // gives the same sums, and with queries and keys from the same rows (the R-update) the query block's own
  // tiles hold, for video tokens, the largest logits of its rows, so the references settle at once.  The
  // launcher decides (P.own_tile_first); the rotation costs the blocks of a frame their common L2 lines.
  const int first_tile = P.own_tile_first ? min(qb * (BQ2 / BK), ntiles - 1) : 0;
  auto tile_at = [&](int i) __attribute__((always_inline)) -> int {
    const int t = i + first_tile;
    return t >= ntiles ? t - ntiles : t;
  };

  const long long qrow0 = (long long)prob * P.q_rows_per_problem;
  const char* kbase = reinterpret_cast<const char*>(P.k + ((long long)prob * P.k_rows_per_problem + kbeg) * D);
  const char* vbase = OUT_V ? reinterpret_cast<const char*>(P.v + ((long long)prob * P.k_rows_per_problem + kbeg) * D) : nullptr;

  // ---- global -> LDS staging (global_load_lds_dwordx4) --------------------------------------
  // One wave instruction fills 64 consecutive 16-byte slots (RPI key rows); slot = key * CH +
  // physical chunk.  Wave w issues the instructions for key rows RPI (W2 r + w) .. + RPI - 1
  // (r = 0 .. NR - 1); each lane fetches the logical chunk that belongs in its slot: its byte offset
  // inside a tile is a per-lane constant (goff[r]), the tile's address a wave-uniform base.
  // Rows past the end of the key range are clamped to the last valid row: finite data whose
  // logits are pushed far down again before they are exponentiated (and which cannot change a row
  // maximum, being copies).
  // The loads are inline assembly on purpose: issued through the builtin, the compiler treats
  // them as LDS writes that any later LDS read may alias and waits for them (vmcnt(0)) in front of
  // the next LDS read, a few instructions after they were issued.  The loop below waits for them
  // itself, before the barrier that publishes a tile.  Loads the compiler does not know about
  // only make its own vmcnt waits longer, never shorter: the counter retires in order.
  constexpr int NR = BK / (RPI * W2);
  static_assert(BK % (RPI * W2) == 0, "every wave issues the same number of loads per tile");
  static_assert((RPI * W2) % 16 == 0, "the rows of one lane share a swizzle");
  const int st_key = RPI * wave + lane / CH;  // + RPI W2 r
  const int st_lc = (lane % CH) ^ swz(st_key);
  unsigned goff[NR];
#pragma unroll
  for (int r = 0; r < NR; ++r) goff[r] = (unsigned)((RPI * W2 * r + st_key) * ROW_BYTES + st_lc * 16);
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)smem;
  auto issue_tile = [&](int i) __attribute__((always_inline)) {  // loop position i: slot i & 3, tile tile_at(i)
    const int t = tile_at(i);
    const unsigned kb = lds_base + (i & (NSLOT - 1)) * TILE_BYTES;
    const char* ksrc = kbase + (long long)t * TILE_BYTES;
    const char* vsrc = OUT_V ? vbase + (long long)t * TILE_BYTES : nullptr;
    const bool ragged = t == ntiles - 1 && last_left < BK;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      unsigned off = goff[r];
      if (ragged) off = (unsigned)(min(RPI * W2 * r + st_key, last_left - 1) * ROW_BYTES + st_lc * 16);
      // wave-uniform LDS byte address in M0; lane lands at + 16 * lane
      const unsigned dst = __builtin_amdgcn_readfirstlane(kb + (RPI * W2 * r + RPI * wave) * ROW_BYTES);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(ksrc), "s"(dst) : "memory", "m0");
      if (OUT_V) {
        const unsigned vdst = dst + V_OFF;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(vsrc), "s"(vdst) : "memory", "m0");
      }
    }
  };
  // the first two tiles go out before anything else so that they travel while Q is fetched
  if (ntiles > 0) issue_tile(0);
  if (ntiles > 1) issue_tile(1);
  // Step 0 has no predecessor and multiplies P^T = 0 with slot 3 of K (and of V): clear those
  // slots, LDS may hold NaN patterns from whoever used it last (0 * NaN would poison the
  // accumulators).
  {
    const uint4 z = {0u, 0u, 0u, 0u};
    static_assert(TILE_BYTES % (16 * 64 * W2) == 0, "the clear covers the slot exactly");
#pragma unroll
    for (int r = 0; r < TILE_BYTES / (16 * 64 * W2); ++r) {
      if (OUT_K) *reinterpret_cast<uint4*>(smem + 3 * TILE_BYTES + (r * 64 * W2 + tid) * 16) = z;
      if (OUT_V) *reinterpret_cast<uint4*>(smem + V_OFF + 3 * TILE_BYTES + (r * 64 * W2 + tid) * 16) = z;
    }
  }

  // ---- queries: B operand of S^T = K Q^T, kept in registers -------------------------------
  bf16x8 qreg[Q2][KS];
  float sc[Q2];
#pragma unroll
  for (int qt = 0; qt < Q2; ++qt) {
    const int r = qb * BQ2 + wave * (32 * Q2) + qt * 32 + ql;
    const int row = r < P.nq ? r : P.nq - 1;
    const bf16_t* qp = P.q + (qrow0 + row) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[qt][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    float c = P.cR ? P.cR[qrow0 + row] : 1.0f;
    c = fmaxf(c, P.cr_min);
    sc[qt] = P.row_scale * LOG2E / c;
  }

  // LDS read addresses, one register each, everything else of an address is an instruction immediate.
  // Row reads (A of S^T): key row = 32 st + ql, logical chunk 2 ks + g.
  unsigned a_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) a_off[ks] = lds_base + ql * ROW_BYTES + (((2 * ks + g) ^ swz(ql)) << 4);
  // Transpose reads (A of O^T += X^T P^T): 16-lane group u = lane / 16 -> g = u / 2, channel
  // half u & 1; lane r' of the group supplies key (r' / 4) and channels 4 (r' & 3) .. + 3.  The V slots
  // lie beyond the reach of the 16-bit offset field, hence a second set of registers for them.
  unsigned t_off[NX][CT][2];
  {
    const int rp = lane & 15;
    const int chh = (lane >> 4) & 1;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int key = 8 * hh + 4 * g + (rp >> 2);  // + 32 st + 16 c added as an immediate
        const int lc = 4 * ct + 2 * chh + ((rp >> 1) & 1);
        const unsigned o = lds_base + key * ROW_BYTES + ((lc ^ swz(key)) << 4) + ((rp & 1) << 3);
        if (OUT_K) t_off[0][ct][hh] = o;
        if (OUT_V) t_off[XV][ct][hh] = o + V_OFF;
      }
  }
  // keep the compiler from re-deriving these from one another inside the loop
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(a_off[ks]));
#pragma unroll
  for (int x = 0; x < NX; ++x)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) asm volatile("" : "+v"(t_off[x][ct][0]), "+v"(t_off[x][ct][1]));
  typedef __attribute__((address_space(3))) const bf16x8* lds_b128_ptr;
  typedef __attribute__((address_space(3))) bf16x4* lds_b64_ptr;
  auto rd_row = [&](unsigned addr) __attribute__((always_inline)) -> bf16x8 { return *(lds_b128_ptr)(unsigned long long)addr; };
  auto rd_tr = [&](unsigned addr) __attribute__((always_inline)) -> bf16x4 {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(unsigned long long)addr);
  };

  // ---- accumulators and statistics ---------------------------------------------------------
  // The products accumulate in accumulation registers (constraint "a" below): with the two query tiles,
  // the logits and the queries in the 256 ordinary registers, 2 x 2 x CT tiles of 16 live there.
  f32x16 oacc[NX][Q2][CT];
#pragma unroll
  for (int x = 0; x < NX; ++x)
#pragma unroll
    for (int qt = 0; qt < Q2; ++qt)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[x][qt][ct][r] = 0.f;
  float msc[Q2], ltil[Q2], hsum[Q2];
#pragma unroll
  for (int qt = 0; qt < Q2; ++qt) {
    msc[qt] = NEG_BIG;
    ltil[qt] = 0.f;
    hsum[qt] = 0.f;
  }

  // ---- the MFMAs, as inline assembly ---------------------------------------------------------
  // With more than 256 registers per wave the compiler gives every MFMA it selects itself an
  // accumulation-register result, which plain vector instructions cannot read; here the logits must land in
  // ordinary registers (the softmax consumes them element by element) and the products in accumulation
  // registers.  Consecutive MFMAs that accumulate into exactly the registers the previous one wrote need
  // no wait; a vector instruction that reads a result does (F2_MFMA_RESULT_WAIT, or enough MFMAs issued in
  // between: each one waits for the pipe, 8 passes).
  auto mfma_first = [&](f32x16& acc, const bf16x8& a, const bf16x8& b) __attribute__((always_inline)) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
  };
  auto mfma_v = [&](f32x16& acc, const bf16x8& a, const bf16x8& b) __attribute__((always_inline)) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
  };
  auto mfma_a = [&](f32x16& acc, const bf16x8& a, const bf16x8& b) __attribute__((always_inline)) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
  };

  // ---- one step = one 32-key sub-tile, as a fixed sequence of groups ------------------------
  // Software pipeline over sub-tiles n = 0, 1, ...  Step n carries, in the one wave,
  //   matrix:  S^T of sub-tile n+1 (both query tiles), then O^T += X^T P^T of sub-tile n-1;
  //   vector:  p = 2^t, running sums and bf16 P^T of sub-tile n, then the row maxima of sub-tile
  //            n+1 (which decide whether the references move at step n+1).
  // A group is the two MFMAs (query tile 0, query tile 1) that share one A operand from LDS: KS groups of
  // logits, then 2 CT NX groups of products in the order (16-key half c, channel tile ct, product x).  The
  // operand of group i + PF is requested while group i runs (a ring of four operand registers; NG is a
  // multiple of four, so ring positions repeat from step to step and the requests run on across steps,
  // tiles and barriers).  The vector work is cut into pieces that are dealt to the MFMA slots so that no
  // slot carries more than an MFMA's worth of it when there is enough matrix work to hide it.
  constexpr int NPV = 2 * CT * NX;
  constexpr int NG = KS + NPV;
  constexpr int NSL = 2 * NG;  // MFMA slots per step
  constexpr int PF = 2;        // groups between an operand's request and its use
  static_assert(NG % 4 == 0, "ring positions repeat from step to step");
  bf16x8 ring[4];
  // request the A operand of group `gi` of a step whose logits come from byte offset s_off (slot and
  // sub-tile of the K tile) and whose products read byte offset pv_off (slot and sub-tile, K and V alike)
  auto request = [&](auto gc, int s_off, int pv_off) __attribute__((always_inline)) {
    constexpr int GI = decltype(gc)::value;
    if constexpr (GI < KS) {
      ring[GI & 3] = rd_row(a_off[GI] + s_off);
    } else {
      constexpr int h = GI - KS;
      constexpr int c = h / (CT * NX);
      constexpr int ct = (h % (CT * NX)) / NX;
      constexpr int x = h % NX;
      const bf16x4 lo = rd_tr(t_off[x][ct][0] + pv_off + c * 16 * ROW_BYTES);
      const bf16x4 hi = rd_tr(t_off[x][ct][1] + pv_off + c * 16 * ROW_BYTES);
      ring[GI & 3] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  auto issue = [&](auto gc, auto qc, f32x16 (&snext)[Q2], bf16x8 (&pbprev)[Q2][2]) __attribute__((always_inline)) {
    constexpr int GI = decltype(gc)::value;
    constexpr int qt = decltype(qc)::value;
    if constexpr (GI == 0) {
      mfma_first(snext[qt], ring[GI & 3], qreg[qt][GI]);
    } else if constexpr (GI < KS) {
      mfma_v(snext[qt], ring[GI & 3], qreg[qt][GI]);
    } else {
      constexpr int h = GI - KS;
      constexpr int c = h / (CT * NX);
      constexpr int ct = (h % (CT * NX)) / NX;
      constexpr int x = h % NX;
      mfma_a(oacc[x][qt][ct], ring[GI & 3], pbprev[qt][c]);
    }
  };

  // vector pieces
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 ones2;
  ones2[0] = (__bf16)1.0f;
  ones2[1] = (__bf16)1.0f;
  // Two scores of one query tile: t = s sc - m, p = 2^t, bf16 pair, l += rounded p, h += rounded p t.  The three
  // stages of a pair (scale, exponent, the rest) are dependent instructions; each stage goes to an MFMA slot of its
  // own (the stages that share a slot then belong to different pairs and issue back to back), so that a single
  // wave does not sit out the latency of its own chain.
  float tq[2][2], pq[2][2];  // in flight between the stages, by parity of the pair
  auto score_scale = [&](auto kc, f32x16 (&scur)[Q2]) __attribute__((always_inline)) {
    constexpr int K = decltype(kc)::value;  // 0 .. 15
    constexpr int qt = K & 1;
    constexpr int j = K >> 1;
    tq[K & 1][0] = __builtin_fmaf(scur[qt][2 * j], sc[qt], -msc[qt]);
    tq[K & 1][1] = __builtin_fmaf(scur[qt][2 * j + 1], sc[qt], -msc[qt]);
  };
  auto score_exp = [&](auto kc) __attribute__((always_inline)) {
    constexpr int K = decltype(kc)::value;
    pq[K & 1][0] = __builtin_amdgcn_exp2f(tq[K & 1][0]);
    pq[K & 1][1] = __builtin_amdgcn_exp2f(tq[K & 1][1]);
  };
  auto score_sums = [&](auto kc, bf16x8 (&pbcur)[Q2][2]) __attribute__((always_inline)) {
    constexpr int K = decltype(kc)::value;
    constexpr int qt = K & 1;
    constexpr int j = K >> 1;
    bf16x2 pr;
    pr[0] = (__bf16)pq[K & 1][0];  // round to nearest even; the pair is one v_cvt_pk_bf16_f32
    pr[1] = (__bf16)pq[K & 1][1];
    ltil[qt] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, ltil[qt], false);
    if (ENT == 1) {
      // h with the same rounded weights that l and the products carry
      uint32_t w;
      __builtin_memcpy(&w, &pr, 4);
      hsum[qt] = __builtin_fmaf(__uint_as_float(w << 16), tq[K & 1][0], hsum[qt]);
      hsum[qt] = __builtin_fmaf(__uint_as_float(w & 0xffff0000u), tq[K & 1][1], hsum[qt]);
    }
    pbcur[qt][j >> 2][2 * (j & 3)] = pr[0];
    pbcur[qt][j >> 2][2 * (j & 3) + 1] = pr[1];
    asm volatile("" : "+v"(ltil[qt]));
    if (ENT == 1) asm volatile("" : "+v"(hsum[qt]));
  };
  float mpend[Q2];     // references that take effect at the start of the next step
  bool moved = false;  // wave-uniform: some reference moves at the start of the next step
  float cand[Q2];
  auto row_max = [&](auto qc, f32x16 (&snext)[Q2]) __attribute__((always_inline)) {
    constexpr int qt = decltype(qc)::value;
    cand[qt] = subtile_max(snext[qt]) * sc[qt];
    asm volatile("" : "+v"(cand[qt]));
  };
  auto decide = [&]() __attribute__((always_inline)) {
    const bool grow = (cand[0] > msc[0] + RESCALE_TH2) || (cand[1] > msc[1] + RESCALE_TH2);
    moved = __any(grow);
#pragma unroll
    for (int qt = 0; qt < Q2; ++qt) {
      // a reference that moves goes HEADROOM2 above the row's maximum: the next move then needs a maximum
      // 2^(HEADROOM2 + RESCALE_TH2) times the present one
      mpend[qt] = moved ? fmaxf(msc[qt], cand[qt] + HEADROOM2) : msc[qt];
      asm volatile("" : "+v"(mpend[qt]));
    }
  };
  // which MFMA slot carries which vector piece
  constexpr int SLOT_MAX0 = 2 * KS + 2;                      // two MFMAs after the last logit MFMA: its result is ready
  constexpr int SLOT_MAX1 = 2 * KS + 4 < NSL ? 2 * KS + 4 : NSL - 1;
  constexpr int SLOT_DECIDE = NSL - 1;
  static_assert(SLOT_MAX0 < NSL && SLOT_MAX1 >= SLOT_MAX0 && SLOT_DECIDE >= SLOT_MAX1, "the maxima follow the logits inside the step");

  // S_OFF / PV_OFF: byte offsets (slot and sub-tile) this step's logits and products read;
  // NS_OFF / NPV_OFF: the same for the step that follows (its first operands are requested here).
  auto step = [&](auto s_c, auto pv_c, auto ns_c, auto npv_c, f32x16 (&scur)[Q2], f32x16 (&snext)[Q2], bf16x8 (&pbprev)[Q2][2],
                  bf16x8 (&pbcur)[Q2][2], int keys_left) __attribute__((always_inline)) {
    constexpr int S_OFF = decltype(s_c)::value, PV_OFF = decltype(pv_c)::value;
    constexpr int NS_OFF = decltype(ns_c)::value, NPV_OFF = decltype(npv_c)::value;
    if (keys_left < 32) {
      // ragged end of the key range: rows keys_left .. 31 of this sub-tile are copies of the
      // last valid row; push their logits far down so that they get probability zero
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float off = (8 * (r >> 2) + 4 * g + (r & 3)) >= keys_left ? -1.0e9f : 0.f;
#pragma unroll
        for (int qt = 0; qt < Q2; ++qt) scur[qt][r] += off;
      }
    }
    const bool moved_now = moved;
    float alpha[Q2];
    if (moved_now) {
      // a reference moves (rare: only when a row maximum outgrew it by 2^RESCALE_TH): the running sums now
      // (App. B: h <- a h + a log(a) l), the accumulators at the end of the step, after the products of
      // sub-tile n-1, which were formed against the old reference
#pragma unroll
      for (int qt = 0; qt < Q2; ++qt) {
        const float dl = msc[qt] - mpend[qt];  // log2 of the rescale factor, <= 0
        alpha[qt] = __builtin_amdgcn_exp2f(dl);
        if (ENT == 1) hsum[qt] = alpha[qt] * (hsum[qt] + dl * ltil[qt]);
        ltil[qt] *= alpha[qt];
        msc[qt] = mpend[qt];
      }
    }
    F2_FENCE();
    static_for<0, NG>([&](auto gc) {
      constexpr int GI = decltype(gc)::value;
      // request the operand of group GI + PF (of the next step beyond the end of this one)
      if constexpr (GI + PF < NG) {
        request(std::integral_constant<int, GI + PF>{}, S_OFF, PV_OFF);
      } else {
        request(std::integral_constant<int, GI + PF - NG>{}, NS_OFF, NPV_OFF);
      }
      static_for<0, 2>([&](auto qc) {
        constexpr int SL = 2 * GI + decltype(qc)::value;
        issue(gc, qc, snext, pbprev);
        // score pairs dealt evenly over the slots: pair k starts in slot floor(k NSL / 16), its exponents follow one
        // slot later and its sums two slots later (both clamped to the step's last slot).  Pairs in ascending
        // order, stages in their own order: a pair's stages that meet in one slot stay in sequence, and the sums
        // of pair k come before pair k + 2 reuses its buffers (it starts at least two slots after pair k).
        static_for<0, 16>([&](auto kc) {
          constexpr int K = decltype(kc)::value;
          constexpr int S0 = (K * NSL) / 16;
          constexpr int S1 = S0 + 1 < NSL ? S0 + 1 : NSL - 1;
          constexpr int S2 = S0 + 2 < NSL ? S0 + 2 : NSL - 1;
          if constexpr (S0 == SL) score_scale(kc, scur);
          if constexpr (S1 == SL) score_exp(kc);
          if constexpr (S2 == SL) score_sums(kc, pbcur);
        });
        if constexpr (SL == SLOT_MAX0) row_max(std::integral_constant<int, 0>{}, snext);
        if constexpr (SL == SLOT_MAX1) row_max(std::integral_constant<int, 1>{}, snext);
        if constexpr (SL == SLOT_DECIDE) decide();
        F2_FENCE();
      });
    });
#pragma unroll
    for (int qt = 0; qt < Q2; ++qt) asm volatile("" : "+v"(pbcur[qt][0]), "+v"(pbcur[qt][1]));
    if (moved_now) {
      F2_MFMA_RESULT_WAIT();  // the last products above are still in the pipe
      F2_FENCE();
#pragma unroll
      for (int x = 0; x < NX; ++x)
#pragma unroll
        for (int qt = 0; qt < Q2; ++qt)
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) {
            // one tile at a time (the empty statements tie the tile's copies out of and back into the
            // accumulation registers to this place, so they do not pile up beside the loop's registers)
            asm volatile("" : "+a"(oacc[x][qt][ct]));
            scale_acc(oacc[x][qt][ct], alpha[qt]);
            asm volatile("" : "+a"(oacc[x][qt][ct]));
            F2_FENCE();
          }
      asm volatile("s_nop 1" ::: "memory");
    }
  };
  if (ntiles > 0) {
    // Four LDS slots, tile t in slot t & 3: during tile t the products of the last sub-tile of
    // tile t-1 are still outstanding, tile t+1 is resident (its first sub-tile is needed one
    // step ahead) and tile t+2 is in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    f32x16 sA[Q2], sB[Q2];
    bf16x8 pbA[Q2][2], pbB[Q2][2];
    {
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int qt = 0; qt < Q2; ++qt)
#pragma unroll
        for (int c = 0; c < 2; ++c) pbB[qt][c] = zero;  // step 0 has no predecessor: it adds P^T = 0
    }
    // A wave whose 64 query rows all lie past the end of the problem (the tail of the last query
    // block) only helps to load the tiles.
    const bool active = qb * BQ2 + wave * (32 * Q2) < P.nq;
    if (active) {
      // logits and row maxima of sub-tile 0, plain form
      static_for<0, KS>([&](auto kc) {
        constexpr int ks = decltype(kc)::value;
        const bf16x8 a = rd_row(a_off[ks]);
        if constexpr (ks == 0) {
          mfma_first(sA[0], a, qreg[0][ks]);
          mfma_first(sA[1], a, qreg[1][ks]);
        } else {
          mfma_v(sA[0], a, qreg[0][ks]);
          mfma_v(sA[1], a, qreg[1][ks]);
        }
      });
      F2_MFMA_RESULT_WAIT();
      F2_FENCE();
      row_max(std::integral_constant<int, 0>{}, sA);
      row_max(std::integral_constant<int, 1>{}, sA);
      decide();
      // operands of the first groups of the first step (sub-tile 1 of slot 0; products against slot 3)
      static_for<0, PF>([&](auto gc) { request(gc, 32 * ROW_BYTES, 3 * TILE_BYTES + 32 * ROW_BYTES); });
    }
    // Four tiles per trip so that every LDS slot offset is an instruction immediate.
    auto tile_iteration = [&](auto slot_c, int t) __attribute__((always_inline)) {
      constexpr int SLOT = decltype(slot_c)::value;
      if (t > 0) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // tile t+1 has landed for everyone; everyone is done with tile t-2
      }
      if (t + 2 < ntiles) issue_tile(t + 2);
      constexpr int kp = ((SLOT + 3) & 3) * TILE_BYTES;  // tile t-1
      constexpr int kt = SLOT * TILE_BYTES;
      constexpr int kn = ((SLOT + 1) & 3) * TILE_BYTES;
      constexpr int HALF = 32 * ROW_BYTES;  // second sub-tile of a tile
      const int left0 = tile_at(t) == ntiles - 1 ? last_left : 64;
      if (active) {
        // logits of (t, 1), products of (t-1, 1) [at t = 0: P^T = 0 against the cleared slot 3], softmax of (t, 0);
        // the step after it: logits of (t+1, 0), products of (t, 0)
        step(std::integral_constant<int, kt + HALF>{}, std::integral_constant<int, kp + HALF>{},
             std::integral_constant<int, kn>{}, std::integral_constant<int, kt>{}, sA, sB, pbB, pbA, left0);
        // logits of (t+1, 0), products of (t, 0), softmax of (t, 1); then logits of (t+1, 1), products of (t, 1)
        step(std::integral_constant<int, kn>{}, std::integral_constant<int, kt>{},
             std::integral_constant<int, kn + HALF>{}, std::integral_constant<int, kt + HALF>{}, sB, sA, pbA, pbB, left0 - 32);
      }
    };
    for (int t0_ = 0; t0_ < ntiles; t0_ += 4) {
      tile_iteration(std::integral_constant<int, 0>{}, t0_);
      if (t0_ + 1 < ntiles) tile_iteration(std::integral_constant<int, 1>{}, t0_ + 1);
      if (t0_ + 2 < ntiles) tile_iteration(std::integral_constant<int, 2>{}, t0_ + 2);
      if (t0_ + 3 < ntiles) tile_iteration(std::integral_constant<int, 3>{}, t0_ + 3);
    }
    if (active) {
      // drain: the products of the last sub-tile, (ntiles-1, 1), plain form
      const int pv_off = ((ntiles - 1) & 3) * TILE_BYTES + 32 * ROW_BYTES;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int x = 0; x < NX; ++x) {
            const bf16x4 lo = rd_tr(t_off[x][ct][0] + pv_off + c * 16 * ROW_BYTES);
            const bf16x4 hi = rd_tr(t_off[x][ct][1] + pv_off + c * 16 * ROW_BYTES);
            const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            mfma_a(oacc[x][0][ct], a, pbB[0][c]);
            mfma_a(oacc[x][1][ct], a, pbB[1][c]);
          }
    }
  }
  F2_MFMA_RESULT_WAIT();  // the accumulators are read by plain vector code from here on
#pragma unroll
  for (int x = 0; x < NX; ++x)
#pragma unroll
    for (int qt = 0; qt < Q2; ++qt)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) asm volatile("" : "+a"(oacc[x][qt][ct]));  // ... and not before this line
  F2_FENCE();
  // ---- epilogue ------------------------------------------------------------------------------
  // Normalised rows are staged in LDS (each wave owns the 64 rows it computed, swizzled like the
  // key tiles; the R K rows over the K slots, the R V rows over the V slots) and leave as whole
  // rows, 16 bytes per lane.  Lane-dependent values are derived again from the thread index,
  // behind an opaque copy, so that none of the epilogue's address arithmetic stays live across
  // the key loop.
  __syncthreads();  // every wave is done with the key/value tiles
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int lane_e = tid_e & 63;
  const int ql_e = lane_e & 31;
  const int g_e = lane_e >> 5;
  const int row_first = qb * BQ2 + wave * (32 * Q2);
  constexpr int STAGE_BYTES = 32 * Q2 * ROW_BYTES;  // per wave and product: W2 of them fill the NSLOT slots exactly
  static_assert(W2 * STAGE_BYTES <= NSLOT * TILE_BYTES, "staged rows fit the slots of their tensor");
#pragma unroll
  for (int qt = 0; qt < Q2; ++qt) {
    const int qr = row_first + qt * 32 + ql_e;
    const bool qvalid = qr < P.nq;
    const long long row = qrow0 + (qvalid ? qr : P.nq - 1);
    const float lt = ltil[qt] + __shfl_xor(ltil[qt], 32);
    const float inv = lt > 0.f ? 1.0f / lt : 0.f;
    if (!SPLIT) {
      if (P.lse != nullptr && qvalid && g_e == 0) P.lse[row] = LN2 * (msc[qt] + __log2f(lt));
      if (ENT == 1) {
        // App. B: H = log S - L / S; here in base-2 units, c_L = -H
        const float h = hsum[qt] + __shfl_xor(hsum[qt], 32);
        const float H2 = __log2f(lt) - h * inv;
        if (qvalid && g_e == 0) P.cl[row] = -LN2 * H2;
      }
      if (ENT == 2 && OUT_K) {
        // sum_l R_l z_l = scale * aR . (sum_l R_l K_l): c_L = scale * (aR . alpha_L) - logsumexp
        float dot = 0.f;
        const bf16_t* qp = P.q + row * D;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint2 w = *reinterpret_cast<const uint2*>(qp + 32 * ct + 8 * c + 4 * g_e);
            dot += __uint_as_float(w.x << 16) * oacc[0][qt][ct][4 * c + 0];
            dot += __uint_as_float(w.x & 0xffff0000u) * oacc[0][qt][ct][4 * c + 1];
            dot += __uint_as_float(w.y << 16) * oacc[0][qt][ct][4 * c + 2];
            dot += __uint_as_float(w.y & 0xffff0000u) * oacc[0][qt][ct][4 * c + 3];
          }
        dot += __shfl_xor(dot, 32);
        const float mean_t = dot * inv * sc[qt];  // sum_l R_l (s_l sc), log2 units
        const float lse2 = msc[qt] + __log2f(lt);
        if (qvalid && g_e == 0) P.cl[row] = LN2 * (mean_t - lse2);
      }
      // lane (q, g) holds channels 32 ct + 8 c + 4 g .. + 3 of query q: 8-byte pieces
#pragma unroll
      for (int x = 0; x < NX; ++x) {
        char* stage = smem + (x == XV && OUT_V ? V_OFF : 0) + wave * STAGE_BYTES;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            uint2 w;
            w.x = pack_bf16(oacc[x][qt][ct][4 * c + 0] * inv, oacc[x][qt][ct][4 * c + 1] * inv);
            w.y = pack_bf16(oacc[x][qt][ct][4 * c + 2] * inv, oacc[x][qt][ct][4 * c + 3] * inv);
            *reinterpret_cast<uint2*>(stage + (32 * qt + ql_e) * ROW_BYTES + (((4 * ct + c) ^ swz(ql_e)) << 4) + 8 * g_e) = w;
          }
      }
    } else {
      // partial result of this key range: normalised output and log2-sum-exp
      if (qvalid) {
        const long long nprob = P.total_blocks / (P.nqb * P.nsplit);
        const long long prow = ((long long)split * nprob + prob) * P.nq + qr;
        if (g_e == 0) P.part_lse[prow] = lt > 0.f ? msc[qt] + __log2f(lt) : NEG_BIG;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int ch = 32 * ct + 8 * c + 4 * g_e;
            const float4 w = {oacc[NX - 1][qt][ct][4 * c + 0] * inv, oacc[NX - 1][qt][ct][4 * c + 1] * inv,
                              oacc[NX - 1][qt][ct][4 * c + 2] * inv, oacc[NX - 1][qt][ct][4 * c + 3] * inv};
            *reinterpret_cast<float4*>(P.part_o + prow * D + ch) = w;
          }
      }
    }
  }
  if (!SPLIT) {
    // the staged rows are private to the wave: no barrier, only the LDS writes above must land
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int x = 0; x < NX; ++x) {
      const char* stage = smem + (x == XV && OUT_V ? V_OFF : 0) + wave * STAGE_BYTES;
      bf16_t* dst = (x == XV && OUT_V) ? P.outv : P.outk;
#pragma unroll
      for (int ps = 0; ps < 32 * Q2 / RPI; ++ps) {
        const int lr = ps * RPI + lane_e / CH;  // row within the wave's block
        const int pc = lane_e % CH;
        const int lc = pc ^ swz(lr);
        if (row_first + lr < P.nq) {
          uint4 w = *reinterpret_cast<const uint4*>(stage + lr * ROW_BYTES + pc * 16);
          uint4* gp = reinterpret_cast<uint4*>(dst + (qrow0 + row_first + lr) * D + lc * 8);
          if (P.blend) w = avg_bf16x8(w, *gp);
          *gp = w;
        }
      }
    }
  }
}

template <int D, bool OUT_K, bool OUT_V, int ENT, bool SPLIT>
hipError_t launch_flash2(const FlashParams& P, hipStream_t st) {
  // four K slots always (the logits need them), four V slots when values are multiplied: 128 KB at d = 128
  constexpr int LDS_BYTES = (OUT_V ? 2 : 1) * NSLOT * BK * D * 2;
  auto kern = flash2_kernel<D, OUT_K, OUT_V, ENT, SPLIT>;
  static bool configured = false;  // the attribute is per function, set once per process
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(P.blocks_per_xcd * 8), dim3(64 * W2), LDS_BYTES, st, P);
  return hipGetLastError();
}

#undef F2_FENCE
#undef F2_MFMA_RESULT_WAIT

}  // namespace

int flash2_query_block() { return BQ2; }

// Exact attention of a contiguous run of nrows query rows per head over all keys (Sec. 3.3) on this kernel, the keys
// cut into `ns` ranges of keys_per_split (a multiple of the tile) whose partial results go to part_o / part_lse
// for the merge (ns == 1: straight to out / lse).  Same 256-row query blocks and partial-result layout as the
// one-tile kernel's pass.
hipError_t launch_first_frame_flash2(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, float* lse,
                                     float* part_o, float* part_lse, const Dims& dm, int nrows, int ns,
                                     int keys_per_split, hipStream_t st) {
  FlashParams P = {};
  P.q = q; P.k = k; P.v = v; P.outv = out; P.lse = lse; P.part_o = part_o; P.part_lse = part_lse;
  P.q_rows_per_problem = dm.N; P.k_rows_per_problem = dm.N;
  P.nq = nrows;
  P.nk = (int)dm.N;
  P.nqb = (nrows + BQ2 - 1) / BQ2;
  P.nsplit = ns;
  P.keys_per_split = keys_per_split;
  const long long total = (long long)dm.BH * P.nqb * ns;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = 1.0f / sqrtf((float)dm.d);
  P.cr_min = 0.f;
  const bool split = ns > 1;
  if (dm.d == 128) return split ? launch_flash2<128, false, true, 0, true>(P, st) : launch_flash2<128, false, true, 0, false>(P, st);
  return split ? launch_flash2<64, false, true, 0, true>(P, st) : launch_flash2<64, false, true, 0, false>(P, st);
}

// One R-update on the one-wave-per-SIMD kernel: alpha_L, c_L (and lse if not null), plus y when v is given.
hipError_t launch_r_update_flash2(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL,
                                  float* cL, bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min,
                                  int entropy_mode, hipStream_t st) {
  if (!(dm.d == 128 || dm.d == 64) || (v == nullptr) != (y == nullptr)) return hipErrorInvalidValue;
  FlashParams P = {};
  P.q = aR; P.cR = cR; P.k = k; P.v = v; P.outk = aL; P.outv = y; P.cl = cL; P.lse = lse;
  P.q_rows_per_problem = dm.b; P.k_rows_per_problem = dm.b;
  P.nq = dm.b; P.nk = dm.b;
  P.nqb = (dm.b + BQ2 - 1) / BQ2;
  P.nsplit = 1;
  P.keys_per_split = ((dm.b + BK - 1) / BK) * BK;
  const long long total = (long long)dm.BH * dm.T * P.nqb;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = row_scale; P.cr_min = cr_min;
  // 0: every query block of a frame walks the key tiles in the same order, so that the blocks resident on one XCD ask
  // for the same tile at about the same time and all but the first request hit its L2 (starting each block at its own
  // tile instead measured 1.9x the algorithmic HBM reads at the same speed)
  P.own_tile_first = 0;
  const bool ident = entropy_mode == VMONARCH_ENTROPY_IDENTITY;
  const bool d128 = dm.d == 128;
  if (v != nullptr) {
    if (ident) return d128 ? launch_flash2<128, true, true, 2, false>(P, st) : launch_flash2<64, true, true, 2, false>(P, st);
    return d128 ? launch_flash2<128, true, true, 1, false>(P, st) : launch_flash2<64, true, true, 1, false>(P, st);
  }
  if (ident) return d128 ? launch_flash2<128, true, false, 2, false>(P, st) : launch_flash2<64, true, false, 2, false>(P, st);
  return d128 ? launch_flash2<128, true, false, 1, false>(P, st) : launch_flash2<64, true, false, 1, false>(P, st);
}

}  // namespace vm
