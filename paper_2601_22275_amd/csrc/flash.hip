// bf16 MFMA kernels for the blocked-softmax passes of spatio-temporal Monarch attention on
// gfx950: the R-update (Eq. R + Eq. alpha_L/c_L, computed as Alg. 1 with the running
// max / sum / entropy of App. B) and the first-frame recomputation (Sec. 3.3).
//
// One workgroup = 8 waves = 256 query rows; each wave owns 32 query rows for the whole key
// loop.  Keys (and values) stream through LDS in 64-row tiles, four slots per tensor, loaded
// two tiles ahead.  Both contractions use v_mfma_f32_32x32x16_bf16:
//
//   S^T = K Q^T     A = K rows read from LDS (ds_read_b128), B = Q^T held in registers.
//                   In the result lane (q, g) holds the logits of query q for 16 of the 32
//                   keys, so the row statistics (max, sum, entropy) are per-lane scalars
//                   and need one exchange with lane^32 for the max only.
//   O^T += X^T P^T  A = X^T (X = K for alpha_L, X = V for y) fetched from the same
//                   row-major LDS tile with the LDS transpose read (ds_read_b64_tr_b16),
//                   B = P^T, which is the S^T accumulator converted to bf16 in place:
//                   eight consecutive accumulator registers are exactly one B operand.
//
// The kernels are instantiated for d = 128 and d = 64.  The 16-byte chunk c of key row r is
// stored at chunk c ^ swz(r) (RowGeo in common.h) so that both the row-wise b128 reads and
// the transpose reads spread over all banks.
#include "../../include/vmonarch.h"
#include <type_traits>

#include "common.h"
#include "flash_device.h"

namespace vm {

namespace {

// element-wise (a + b) / 2 of eight bf16 values, in float, rounded once
__device__ __forceinline__ uint32_t average_bf16x2(uint32_t a, uint32_t b);
__device__ __forceinline__ uint4 average_bf16x8(uint4 a, uint4 b);

template <int D, bool OUT_K, bool OUT_V, int ENT, bool SPLIT, int BIAS = 0>
__global__ void __launch_bounds__(64 * NW) flash_kernel(FlashParams P) {
  using G = RowGeo<D>;
  constexpr int ROW_BYTES = G::ROW_BYTES;
  constexpr int TILE_BYTES = BK * ROW_BYTES;  // 16 KB (d = 128) or 8 KB (d = 64)
  constexpr int KS = G::KS;                   // k-steps of S^T = K Q^T
  constexpr int CT = G::CT;                   // 32-channel tiles of an output row
  constexpr int CH = G::CH;                   // 16-byte chunks per row
  constexpr int RPI = G::RPI;                 // rows filled by one 64-lane global -> LDS load
  auto swz = [](int row) { return G::swz(row); };
  extern __shared__ __attribute__((aligned(16))) char smem[];  // [K|V][NSLOT][64 rows][2 D bytes] [key biases]
  static_assert(BIAS == 0 || (!SPLIT && ENT == 0), "the biased modes are whole-range passes without entropy");

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
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ql = lane & 31;
  const int g = lane >> 5;

  const int kbeg = split * P.keys_per_split;
  const int kend = min(P.nk, kbeg + P.keys_per_split);
  const int nkeys = kend - kbeg;
  const int ntiles = (nkeys + BK - 1) / BK;

  const long long rs = P.row_stride ? P.row_stride : 1;  // distance between consecutive rows of a problem
  const int inner = P.inner ? P.inner : 1;
  const int p_out = prob / inner, p_in = prob - p_out * inner;
  const long long qrow0 = (long long)p_out * P.q_rows_per_problem + (long long)p_in * P.inner_rows;
  const long long krow0 = (long long)p_out * P.k_rows_per_problem + (long long)p_in * P.inner_rows;
  const bf16_t* kbase = P.k + (krow0 + kbeg * rs) * D;
  const bf16_t* vbase = OUT_V ? P.v + (krow0 + kbeg * rs) * D : nullptr;

  // ---- LDS addressing ----------------------------------------------------------------
  // staging: global -> LDS directly (global_load_lds_dwordx4).  One wave instruction fills 64
  // consecutive 16-byte slots (RPI key rows); slot = key * CH + physical chunk.  Wave w issues
  // the instructions for key rows RPI (NW r + w) .. + RPI - 1 (r = 0 .. BK / (RPI NW) - 1);
  // each lane fetches the logical chunk that belongs in its slot.  Rows past the end of the key range are
  // clamped to the last valid row: finite data whose logits are pushed to -1e9 again before
  // they are exponentiated (and which cannot change a row maximum, being copies).
  static_assert(BK % (RPI * NW) == 0, "every wave issues the same number of loads per tile");
  const int st_key = RPI * wave + lane / CH;  // + RPI NW r
  const int st_lc = (lane % CH) ^ swz(st_key);
  // LDS: NSLOT K tiles at [0, NSLOT * 16 KB), then NSLOT V tiles; tile t lives in slot t & 3.
  // The global -> LDS loads are written as inline assembly on purpose.  Issued through the
  // builtin, the compiler tracks them as LDS writes that any later LDS read may alias and puts
  // s_waitcnt vmcnt(0) in front of the next transpose read, a few instructions after the
  // load was issued: the prefetch of tile t+2 then stalls every tile for a full memory
  // latency.  The loop below waits for them itself (s_waitcnt vmcnt(0) before the barrier that
  // publishes a tile).  Loads the compiler does not know about only make its own vmcnt waits
  // longer, never shorter, because the counter retires in order.
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)smem;
  auto issue_tile = [&](int t) {
    const unsigned kb = lds_base + (t & (NSLOT - 1)) * TILE_BYTES;
#pragma unroll
    for (int r = 0; r < BK / (RPI * NW); ++r) {
      int key = min(t * BK + RPI * NW * r + st_key, nkeys - 1);
      const bf16_t* src = kbase + (long long)key * rs * D + st_lc * 8;
      // wave-uniform LDS byte address in M0; lane lands at + 16 * lane
      const unsigned dst = __builtin_amdgcn_readfirstlane(kb + (RPI * NW * r + RPI * wave) * ROW_BYTES);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(dst) : "memory", "m0");
      if (OUT_V) {
        const bf16_t* vsrc = vbase + (long long)key * rs * D + st_lc * 8;
        const unsigned vdst = dst + NSLOT * TILE_BYTES;
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(vsrc), "s"(vdst) : "memory", "m0");
      }
    }
  };
  // the first two tiles go out before anything else so that they travel while Q is fetched
  if (ntiles > 0) issue_tile(0);
  if (ntiles > 1) issue_tile(1);
  // Step 0 has no predecessor and multiplies P^T = 0 with slot 3 of X: clear that slot, LDS
  // may hold NaN patterns from whoever used it last (0 * NaN would poison the accumulators).
  {
    char* x3 = smem + (OUT_K ? 0 : NSLOT * TILE_BYTES) + 3 * TILE_BYTES;
    const uint4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int r = 0; r < TILE_BYTES / (16 * 64 * NW); ++r) *reinterpret_cast<uint4*>(x3 + (r * 64 * NW + tid) * 16) = z;
    static_assert(TILE_BYTES % (16 * 64 * NW) == 0, "the clear covers the slot exactly");
  }
  // Biased modes: the additive term of every key of the problem, gathered once into LDS behind the tile slots
  // (the launcher sizes the allocation: (ntiles + 1) * 64 floats; keys past the end get 0 and are masked anyway).
  float* kb_lds = reinterpret_cast<float*>(smem + 2 * NSLOT * TILE_BYTES);
  if (BIAS != 0) {
    for (int l = tid; l < (ntiles + 1) * BK; l += 64 * NW)
      kb_lds[l] = l < nkeys ? P.kb_scale * P.kbias[krow0 + (long long)(kbeg + l) * rs] : 0.f;
  }

  // ---- queries: B operand of S^T = K Q^T, kept in registers -------------------------
  bf16x8 qreg[QT][KS];
  float sc[QT];
  int qrow[QT];   // row within the problem's list of query rows
  int grow[QT];   // the row of the problem it stands for (the same unless a row list is given)
  bool qvalid[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    int r = qb * BQ + wave * (32 * QT) + qt * 32 + ql;
    qvalid[qt] = r < P.nq;
    qrow[qt] = qvalid[qt] ? r : P.nq - 1;
    grow[qt] = qrow[qt];
    if (P.q_index != nullptr) {
      // a listed row; an entry that does not name a row of the head is skipped (read as row 0, never stored)
      const int gi = P.q_index[qrow[qt]];
      const bool inside = gi >= 0 && gi < P.q_index_limit;
      qvalid[qt] = qvalid[qt] && inside;
      grow[qt] = inside ? gi : 0;
    }
    const bf16_t* qp = P.q + (qrow0 + grow[qt] * rs) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[qt][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    float c = P.cR ? P.cR[qrow0 + grow[qt] * rs] : 1.0f;
    c = fmaxf(c, P.cr_min);
    sc[qt] = P.row_scale * LOG2E / c;
  }

  // row reads (A of S^T): key row = 32 st + ql, logical chunk 2 ks + g
  int a_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) a_off[ks] = ql * ROW_BYTES + (((2 * ks + g) ^ swz(ql)) << 4);
  // transpose reads (A of O^T += X^T P^T): 16-lane group u = lane / 16 -> g = u / 2, channel
  // half u & 1; lane r' of the group supplies key (r' / 4) and channels 4 (r' & 3) .. + 3.
  // For X = V the offsets point into the V slots.
  int t_off[CT][2];
  {
    const int rp = lane & 15;
    const int chh = (lane >> 4) & 1;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        int key = 8 * hh + 4 * g + (rp >> 2);  // + 32 st + 16 c' added as an immediate
        int lc = 4 * ct + 2 * chh + ((rp >> 1) & 1);
        t_off[ct][hh] = key * ROW_BYTES + ((lc ^ swz(key)) << 4) + ((rp & 1) << 3) + (OUT_K ? 0 : NSLOT * TILE_BYTES);
      }
  }

  // ---- accumulators and statistics -------------------------------------------------------
  static_assert(OUT_K != OUT_V, "one accumulator set per pass (see launch_r_update_flash)");
  f32x16 oacc[QT][CT];  // O^T tiles: [query tile][32-channel tile]
#pragma unroll
  for (int qt = 0; qt < QT; ++qt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qt][ct][r] = 0.f;
  float msc[QT], ltil[QT], hsum[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    msc[qt] = NEG_BIG;
    ltil[qt] = 0.f;
    hsum[qt] = 0.f;
    // BIAS == 2: the reference of a row is given and never moves (every exponent is <= 0 by construction)
    if (BIAS == 2) msc[qt] = P.qb_scale * P.qbias[qrow0 + grow[qt] * rs];
  }
  float inv_sc[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) inv_sc[qt] = BIAS != 0 ? 1.0f / sc[qt] : 0.f;
  // Biased modes: logits of sub-tile `sub` (keys 32 sub .. 32 sub + 31) get their keys' terms, expressed in units of the
  // raw product (divided by the row's scale) so that everything downstream treats them like any other logit.
  auto add_key_bias = [&](f32x16 (&sacc)[QT], int sub) {
    if (BIAS == 0) return;
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) {
      const float4 kb = *reinterpret_cast<const float4*>(kb_lds + 32 * sub + 8 * c4 + 4 * g);
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        sacc[qt][4 * c4 + 0] = __builtin_fmaf(kb.x, inv_sc[qt], sacc[qt][4 * c4 + 0]);
        sacc[qt][4 * c4 + 1] = __builtin_fmaf(kb.y, inv_sc[qt], sacc[qt][4 * c4 + 1]);
        sacc[qt][4 * c4 + 2] = __builtin_fmaf(kb.z, inv_sc[qt], sacc[qt][4 * c4 + 2]);
        sacc[qt][4 * c4 + 3] = __builtin_fmaf(kb.w, inv_sc[qt], sacc[qt][4 * c4 + 3]);
      }
    }
  };

  // Software pipeline over 32-key sub-tiles n = 0, 1, ...  Step n carries two independent
  // instruction streams:
  //   matrix:  S^T of sub-tile n+1, then O^T += X^T P^T of sub-tile n-1 (P^T from step n-1);
  //   vector:  p = 2^t, running sums and bf16 P^T of sub-tile n, then the row maxima of
  //            sub-tile n+1 (which decide whether the references move at step n+1).
  // A reference move (rare: only when a row maximum outgrew its reference by 2^RESCALE_TH)
  // rescales the scalar statistics at the top of the step, before they are added to, and the
  // accumulators at the bottom, after the products of sub-tile n-1 (computed against the old
  // reference) have been issued and before those of sub-tile n are.
  // Every step is the same code: the step after the last sub-tile's predecessor forms the
  // logits of a sub-tile that does not exist (from whatever its LDS slot holds) and nobody
  // reads them; a ragged last tile only adds one uniform branch at the top of its two steps.
  auto logits = [&](const char* ktile, int st, f32x16 (&sacc)[QT]) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[qt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 a = lds_read_b128(ktile + st * 32 * ROW_BYTES + a_off[ks]);
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
        sacc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qt][ks], sacc[qt], 0, 0, 0);
    }
  };
  // O^T += X^T P^T for sub-tile `st` of the tile whose K slot is `ktile`
  auto accumulate = [&](const char* ktile, int st, bf16x8 (&pb)[QT][2]) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int koff = (st * 32 + c * 16) * ROW_BYTES;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        bf16x4 lo = lds_read_tr(ktile + koff + t_off[ct][0]);
        bf16x4 hi = lds_read_tr(ktile + koff + t_off[ct][1]);
        bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          oacc[qt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qt][c], oacc[qt][ct], 0, 0, 0);
      }
    }
  };
  float mpend[QT];     // references that take effect at the start of the next step
  bool moved = false;  // wave-uniform: some reference moves at the start of the next step
  auto look_ahead = [&](f32x16 (&snext)[QT]) {
    if (BIAS == 2) {
      moved = false;
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) mpend[qt] = msc[qt];
      return;
    }
    bool grow = false;
    float cand[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      cand[qt] = subtile_max(snext[qt]) * sc[qt];
      grow = grow || (cand[qt] > msc[qt] + RESCALE_TH);
    }
    moved = __any(grow);
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) mpend[qt] = moved ? fmaxf(msc[qt], cand[qt]) : msc[qt];
  };
  auto step = [&](f32x16 (&scur)[QT], f32x16 (&snext)[QT], bf16x8 (&pbprev)[QT][2], bf16x8 (&pbcur)[QT][2],
                  const char* next_ktile, int next_st, const char* prev_ktile, int prev_st, int keys_left, int next_sub) {
    if (keys_left < 32) {
      // ragged end of the key range: rows keys_left .. 31 of this sub-tile are copies of the
      // last valid row; push their logits far down so that they get probability zero
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float off = (8 * (r >> 2) + 4 * g + (r & 3)) >= keys_left ? -1.0e9f : 0.f;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) scur[qt][r] += off;
      }
    }
    const bool moved_now = moved;
    float alpha[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      const float dl = msc[qt] - mpend[qt];  // log2 of the rescale factor: <= 0, and 0 when nothing moved
      alpha[qt] = __builtin_amdgcn_exp2f(dl);
      if (ENT == 1) hsum[qt] = alpha[qt] * (hsum[qt] + dl * ltil[qt]);  // h <- a h + a log(a) l
      ltil[qt] *= alpha[qt];
      msc[qt] = mpend[qt];
    }
    logits(next_ktile, next_st, snext);
    accumulate(prev_ktile, prev_st, pbprev);
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) subtile_probs<ENT>(scur[qt], sc[qt], msc[qt], ltil[qt], hsum[qt], pbcur[qt]);
    add_key_bias(snext, next_sub);
    look_ahead(snext);
    // Keep this step's vector results in this step: without the pins below the compiler sinks
    // the probability code past the rescale branch to its first use, next to the MFMAs of the
    // following step, and the two streams stop overlapping.
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      asm volatile("" : "+v"(pbcur[qt][0]), "+v"(pbcur[qt][1]), "+v"(ltil[qt]), "+v"(mpend[qt]));
      if (ENT == 1) asm volatile("" : "+v"(hsum[qt]));
    }
    if (moved_now) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) scale_acc(oacc[qt][ct], alpha[qt]);
    }
  };
  if (ntiles > 0) {
    // Four LDS slots, tile t in slot t & 3: during tile t the products of the last sub-tile of
    // tile t-1 are still outstanding, tile t+1 is resident (its first sub-tile is needed one
    // step ahead) and tile t+2 is in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    f32x16 sA[QT], sB[QT];
    bf16x8 pbA[QT][2], pbB[QT][2];
    {
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int c = 0; c < 2; ++c) pbB[qt][c] = zero;  // step 0 has no predecessor: it adds P^T = 0
    }
    // A wave whose 32 query rows all lie past the end of the problem (the tail of the last query
    // block) only helps to load the tiles: it skips the arithmetic, and the energy it would burn
    // on rows nobody reads (the matrix pipe is power-limited) goes to the waves that have work.
    const bool active = qb * BQ + wave * (32 * QT) < P.nq;
    if (active) {
      logits(smem, 0, sA);
      add_key_bias(sA, 0);
      look_ahead(sA);
    }
    const int last_left = nkeys - (ntiles - 1) * BK;  // 1..64 keys in the last tile
    // Four tiles per trip so that every LDS slot offset is an instruction immediate (tile t
    // sits in slot t & 3 and a trip starts at a multiple of four).
    auto tile_iteration = [&](auto slot_c, int t) {
      constexpr int SLOT = decltype(slot_c)::value;
      if (t > 0) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // tile t+1 has landed for everyone; everyone is done with tile t-2
      }
      if (t + 2 < ntiles) issue_tile(t + 2);
      const char* kp = smem + ((SLOT + 3) & 3) * TILE_BYTES;  // tile t-1
      const char* kt = smem + SLOT * TILE_BYTES;
      const char* kn = smem + ((SLOT + 1) & 3) * TILE_BYTES;
      const int left0 = t == ntiles - 1 ? last_left : 64;
      if (active) {
        step(sA, sB, pbB, pbA, kt, 1, kp, 1, left0, 2 * t + 1);  // at t = 0: P^T = 0 against the cleared slot 3
        step(sB, sA, pbA, pbB, kn, 0, kt, 0, left0 - 32, 2 * t + 2);
      }
    };
    for (int t0 = 0; t0 < ntiles; t0 += 4) {
      tile_iteration(std::integral_constant<int, 0>{}, t0);
      if (t0 + 1 < ntiles) tile_iteration(std::integral_constant<int, 1>{}, t0 + 1);
      if (t0 + 2 < ntiles) tile_iteration(std::integral_constant<int, 2>{}, t0 + 2);
      if (t0 + 3 < ntiles) tile_iteration(std::integral_constant<int, 3>{}, t0 + 3);
    }
    if (active) accumulate(smem + ((ntiles - 1) & 3) * TILE_BYTES, 1, pbB);  // drain: the products of the last sub-tile
  }
  // ---- epilogue ----------------------------------------------------------------------------
  // Normalised rows are staged in LDS (each wave owns the 32 * QT rows it computed, swizzled
  // like the key tiles) and leave as whole rows, 16 bytes per lane.
  __syncthreads();  // every wave is done with the key/value tiles
  char* stage = smem + wave * (32 * QT * ROW_BYTES);
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float lt = ltil[qt] + __shfl_xor(ltil[qt], 32);
    const float inv = BIAS == 2 ? 1.0f : (lt > 0.f ? 1.0f / lt : 0.f);  // BIAS == 2: the weights are final as they are
    const long long row = qrow0 + grow[qt] * rs;
    if (BIAS == 2 && qvalid[qt] && g == 0) P.cl[row] = lt;              // ... and their sum is an output
    if (!SPLIT) {
      if (P.lse != nullptr && qvalid[qt] && g == 0) P.lse[row] = LN2 * (msc[qt] + __log2f(lt));
      if (ENT == 1) {
        // App. B: H = log S - L / S; here in base-2 units, c_L = -H
        float h = hsum[qt] + __shfl_xor(hsum[qt], 32);
        float H2 = __log2f(lt) - h * inv;
        if (qvalid[qt] && g == 0) P.cl[row] = -LN2 * H2;
      }
      if (ENT == 2) {
        // sum_l R_l z_l = scale * aR . (sum_l R_l K_l): c_L = scale * (aR . alpha_L) - logsumexp
        float dot = 0.f;
        const bf16_t* qp = P.q + row * D;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            uint2 w = *reinterpret_cast<const uint2*>(qp + 32 * ct + 8 * c + 4 * g);
            dot += __uint_as_float(w.x << 16) * oacc[qt][ct][4 * c + 0];
            dot += __uint_as_float(w.x & 0xffff0000u) * oacc[qt][ct][4 * c + 1];
            dot += __uint_as_float(w.y << 16) * oacc[qt][ct][4 * c + 2];
            dot += __uint_as_float(w.y & 0xffff0000u) * oacc[qt][ct][4 * c + 3];
          }
        dot += __shfl_xor(dot, 32);
        float mean_t = dot * inv * sc[qt];          // sum_l R_l (s_l sc), log2 units
        float lse2 = msc[qt] + __log2f(lt);
        if (qvalid[qt] && g == 0) P.cl[row] = LN2 * (mean_t - lse2);
      }
      // lane (q, g) holds channels 32 ct + 8 c + 4 g .. + 3 of query q: 8-byte pieces
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint2 w;
          w.x = pack_bf16(oacc[qt][ct][4 * c + 0] * inv, oacc[qt][ct][4 * c + 1] * inv);
          w.y = pack_bf16(oacc[qt][ct][4 * c + 2] * inv, oacc[qt][ct][4 * c + 3] * inv);
          *reinterpret_cast<uint2*>(stage + (32 * qt + ql) * ROW_BYTES + (((4 * ct + c) ^ swz(ql)) << 4) + 8 * g) = w;
        }
    } else {
      // partial result of this key range: normalised output and log2-sum-exp
      if (qvalid[qt]) {
        const long long nprob = P.total_blocks / (P.nqb * P.nsplit);
        const long long prow = ((long long)split * nprob + prob) * P.nq + qrow[qt];
        if (g == 0) P.part_lse[prow] = lt > 0.f ? msc[qt] + __log2f(lt) : NEG_BIG;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int ch = 32 * ct + 8 * c + 4 * g;
            float4 w = {oacc[qt][ct][4 * c + 0] * inv, oacc[qt][ct][4 * c + 1] * inv, oacc[qt][ct][4 * c + 2] * inv,
                        oacc[qt][ct][4 * c + 3] * inv};
            *reinterpret_cast<float4*>(P.part_o + prow * D + ch) = w;
          }
      }
    }
  }
  if (!SPLIT) {
    // the staged rows are private to the wave: no barrier, only the LDS writes above must land
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
    bf16_t* dst = OUT_K ? P.outk : P.outv;
    const int row_first = qb * BQ + wave * (32 * QT);
    if (dst != nullptr)  // a pass that only wants the row statistics gives no destination
#pragma unroll
    for (int ps = 0; ps < 32 * QT / RPI; ++ps) {
      const int lr = ps * RPI + lane / CH;  // row within the wave's block
      const int pc = lane % CH;
      const int lc = pc ^ swz(lr);
      int orow = row_first + lr;
      bool ovalid = orow < P.nq;
      if (P.q_index != nullptr && ovalid) {
        orow = P.q_index[orow];
        ovalid = orow >= 0 && orow < P.q_index_limit;
      }
      if (ovalid) {
        uint4 w = *reinterpret_cast<const uint4*>(stage + lr * ROW_BYTES + pc * 16);
        uint4* gp = reinterpret_cast<uint4*>(dst + (qrow0 + orow * rs) * D + lc * 8);
        if (P.blend) w = average_bf16x8(w, *gp);
        *gp = w;
      }
    }
  }
}

__device__ __forceinline__ uint32_t average_bf16x2(uint32_t a, uint32_t b) {
  const float lo = 0.5f * (__uint_as_float(a << 16) + __uint_as_float(b << 16));
  const float hi = 0.5f * (__uint_as_float(a & 0xffff0000u) + __uint_as_float(b & 0xffff0000u));
  return pack_bf16(lo, hi);
}
__device__ __forceinline__ uint4 average_bf16x8(uint4 a, uint4 b) {
  return make_uint4(average_bf16x2(a.x, b.x), average_bf16x2(a.y, b.y), average_bf16x2(a.z, b.z),
                    average_bf16x2(a.w, b.w));
}

// Merge of the key-range partials of the first-frame recomputation: weights 2^(lse - max).
__global__ void __launch_bounds__(128) merge_splits_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_lse, bf16_t* __restrict__ out,
                                                           float* __restrict__ lse, int nsplit, long long rows_per_split,
                                                           int nq, long long out_rows_per_problem,
                                                           const int* __restrict__ q_index, int q_index_limit) {
  const int D = blockDim.x;        // one thread per channel
  const long long r = blockIdx.x;  // problem * nq + row
  const int c = threadIdx.x;       // channel
  const long long prob = r / nq;
  long long row = r - prob * nq;
  if (q_index != nullptr) {
    row = q_index[row];
    if (row < 0 || row >= q_index_limit) return;  // not a row of the head: skipped
  }
  float mx = -INFINITY;
  for (int s = 0; s < nsplit; ++s) mx = fmaxf(mx, part_lse[s * rows_per_split + r]);
  float wsum = 0.f, acc = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    float w = exp2f(part_lse[s * rows_per_split + r] - mx);
    wsum += w;
    acc += w * part_o[(s * rows_per_split + r) * D + c];
  }
  out[(prob * out_rows_per_problem + row) * D + c] = f32_to_bf16(acc / wsum);
  if (lse != nullptr && c == 0) lse[prob * out_rows_per_problem + row] = LN2 * (mx + log2f(wsum));
}

constexpr int kMaxBiasedKeys = 8192 - BK;  // biased modes keep one float per key (+ one tile of padding) behind the tile slots: 32 KB

template <int D, bool OUT_K, bool OUT_V, int ENT, bool SPLIT, int BIAS = 0>
hipError_t launch_flash(const FlashParams& P, hipStream_t st) {
  constexpr int TILE_LDS = 2 * NSLOT * BK * D * 2;  // four K slots + four V slots: 128 KB at d = 128
  constexpr int MAX_LDS = TILE_LDS + (BIAS != 0 ? (kMaxBiasedKeys + BK) * 4 : 0);
  auto kern = flash_kernel<D, OUT_K, OUT_V, ENT, SPLIT, BIAS>;
  static bool configured = false;  // the attribute is per function, set once per process
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  int lds = TILE_LDS;
  if (BIAS != 0) {
    if (P.nk > kMaxBiasedKeys || P.nsplit != 1 || P.kbias == nullptr) return hipErrorInvalidValue;
    lds += ((P.nk + BK - 1) / BK + 1) * BK * 4;
  }
  hipLaunchKernelGGL(kern, dim3(P.blocks_per_xcd * 8), dim3(64 * NW), lds, st, P);
  return hipGetLastError();
}

int compute_units() {
  static int cus = 0;  // one device per process is assumed for this tuning value only
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

// Key ranges for exact attention of `nrows` query rows per head over all N keys.  One workgroup
// occupies a compute unit, and all work items take the same time, so the launch runs in
// ceil(items / CUs) rounds: the split count is the one that wastes least of the last round,
// after a charge of a few tiles' worth of time per item for its start-up and wind-down.
int first_frame_splits(const Dims& dm, int nrows) {
  const long long nqb = (nrows + BQ - 1) / BQ;
  const long long tiles = (dm.N + BK - 1) / BK;
  const long long cus = compute_units();
  int best = 1;
  double best_score = -1.0;
  for (long long s = 1; s <= 64; ++s) {
    const long long per = (tiles + s - 1) / s;  // tiles per key range
    if (s > 1 && per < 8) break;
    if ((tiles + per - 1) / per != s) continue;  // would leave an empty range: the same as a smaller count
    const long long items = (long long)dm.BH * nqb * s;
    const long long rounds = (items + cus - 1) / cus;
    const double score = (double)items / (double)(rounds * cus) * (double)per / (double)(per + 6);
    if (score > best_score * 1.005) {  // prefer fewer ranges (less merge traffic) unless clearly better
      best_score = score;
      best = (int)s;
    }
  }
  return best;
}

}  // namespace

bool flash_supported(const Dims& dm) { return dm.d == 128 || dm.d == 64; }

hipError_t launch_r_update_flash(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL,
                                 float* cL, bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min,
                                 int entropy_mode, bool fused, hipStream_t st) {
  if (fused && v != nullptr && entropy_mode == VMONARCH_ENTROPY_ONLINE)
    return launch_r_update_flash_fused(aR, cR, k, v, aL, cL, y, lse, dm, row_scale, cr_min, st);
  FlashParams P = {};
  P.q = aR; P.cR = cR; P.k = k; P.v = v; P.outk = aL; P.outv = y; P.cl = cL; P.lse = lse;
  P.q_rows_per_problem = dm.b; P.k_rows_per_problem = dm.b;
  P.nq = dm.b; P.nk = dm.b;
  P.nqb = (dm.b + BQ - 1) / BQ;
  P.nsplit = 1;
  P.keys_per_split = ((dm.b + BK - 1) / BK) * BK;
  long long total = (long long)dm.BH * dm.T * P.nqb;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = row_scale; P.cr_min = cr_min;
  const bool ident = entropy_mode == VMONARCH_ENTROPY_IDENTITY;
  // alpha_L and c_L from one pass over K; y = R V from a second pass that recomputes the
  // logits.  (One wave cannot hold both accumulator sets; flash_kv.hip shares them between two.)
  auto run = [&](auto dc) -> hipError_t {
    constexpr int D = decltype(dc)::value;
    hipError_t e = ident ? launch_flash<D, true, false, 2, false>(P, st) : launch_flash<D, true, false, 1, false>(P, st);
    if (e != hipSuccess || v == nullptr) return e;
    P.outk = nullptr;
    P.cl = nullptr;
    P.lse = nullptr;
    return launch_flash<D, false, true, 0, false>(P, st);
  };
  return dm.d == 128 ? run(std::integral_constant<int, 128>{}) : run(std::integral_constant<int, 64>{});
}

size_t first_frame_flash_scratch_bytes(const Dims& dm, int nrows) {
  const int ns = first_frame_splits(dm, nrows);
  if (ns == 1) return 0;
  size_t rows = (size_t)ns * dm.BH * nrows;
  return rows * dm.d * sizeof(float) + ((rows * sizeof(float) + 255) & ~(size_t)255);
}

// q, out and lse point at the first row to recompute of head 0 (rows of later heads sit N rows
// further on, like everything else); k and v at the heads' first tokens.
hipError_t launch_first_frame_flash(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, float* lse,
                                    void* scratch, size_t scratch_bytes, const Dims& dm, int nrows, const int* row_list,
                                    bool two_tile, hipStream_t st) {
  FlashParams P = {};
  P.q_index = row_list;  // null: the nrows rows that follow q / out / lse; else: rows[r] of every head, q / out / lse at row 0
  P.q_index_limit = (int)dm.N;
  const int ns = first_frame_splits(dm, nrows);
  P.q = q; P.cR = nullptr; P.k = k; P.v = v; P.outk = nullptr; P.outv = out; P.cl = nullptr;
  P.lse = lse;  // written by the kernel itself when one key range covers everything, else by the merge
  P.q_rows_per_problem = dm.N; P.k_rows_per_problem = dm.N;
  P.nq = nrows;
  if (dm.N > 0x7fffffffLL - BK) return hipErrorInvalidValue;
  P.nk = (int)dm.N;
  P.nqb = (nrows + BQ - 1) / BQ;
  P.nsplit = ns;
  const long long tiles = (dm.N + BK - 1) / BK;
  P.keys_per_split = (int)(((tiles + ns - 1) / ns) * BK);
  long long total = (long long)dm.BH * P.nqb * ns;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = 1.0f / sqrtf((float)dm.d);
  P.cr_min = 0.f;
  const bool d128 = dm.d == 128;
  // contiguous rows can run on the kernel with two query tiles per wave (same blocks, ranges and partial results;
  // measured 2 .. 3 % faster on the long key loops of this pass); a row list is gathered by this file's kernel only
  // (the key ranges and the partial-result buffers above are sized for this file's query blocks: the other kernel's must match)
  const bool ff2 = two_tile && row_list == nullptr && flash2_query_block() == BQ;
  if (ns == 1) {
    if (ff2) return launch_first_frame_flash2(q, k, v, out, lse, nullptr, nullptr, dm, nrows, 1, P.keys_per_split, st);
    return d128 ? launch_flash<128, false, true, 0, false>(P, st) : launch_flash<64, false, true, 0, false>(P, st);
  }
  const size_t rows = (size_t)ns * dm.BH * nrows;
  const size_t need = rows * dm.d * sizeof(float) + ((rows * sizeof(float) + 255) & ~(size_t)255);
  if (scratch == nullptr || scratch_bytes < need) return hipErrorInvalidValue;
  P.part_lse = (float*)scratch;
  P.part_o = (float*)((char*)scratch + ((rows * sizeof(float) + 255) & ~(size_t)255));
  hipError_t e = ff2 ? launch_first_frame_flash2(q, k, v, out, lse, P.part_o, P.part_lse, dm, nrows, ns, P.keys_per_split, st)
                     : (d128 ? launch_flash<128, false, true, 0, true>(P, st) : launch_flash<64, false, true, 0, true>(P, st));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(merge_splits_kernel, dim3((unsigned)((long long)dm.BH * nrows)), dim3(dm.d), 0, st, P.part_o,
                     P.part_lse, out, lse, ns, (long long)dm.BH * nrows, nrows, dm.N, row_list, (int)dm.N);
  return hipGetLastError();
}

// The temporal factor through the blocked-softmax kernel, for any number of frames T (Eq. L with Eq. alpha_R / c_R, and
// the apply-to-V of App. A).  A problem is one (head, position i); its rows are the T frames of that position, b rows
// apart in the frame-major tensors.  With u[j,k] = q_scale (Q[j] . alpha_L[k]) - c_L[k]:
//   last sweep     one pass, queries Q[j], keys alpha_L[k] with the additive term -c_L[k], values y[k]:
//                  out[j] = sum_k softmax_k(u[j,:])[k] y[k];
//   fitting sweep  pass 1, the same queries and keys without a product: lse[j] = log sum_k exp u[j,k];
//                  pass 2 with the roles exchanged, queries alpha_L[k] (fixed reference c_L[k]), keys Q[j] with the
//                  additive term -lse[j], values Q[j]: the weights exp(u[j,k] - lse[j]) = L[j,k] are final, so
//                  alpha_R[k] = sum_j L[j,k] Q[j] and c_R[k] = sum_j L[j,k] are plain unnormalised sums.
// lse_scratch: BH * N floats (fitting sweep only).
bool temporal_flash_supported(const Dims& dm) { return (dm.d == 128 || dm.d == 64) && dm.T <= kMaxBiasedKeys; }

hipError_t launch_l_update_flash(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR, float* cR,
                                 bf16_t* out, float* lse_scratch, const Dims& dm, float q_scale, hipStream_t st) {
  if (!temporal_flash_supported(dm)) return hipErrorInvalidValue;
  FlashParams P = {};
  P.q_rows_per_problem = dm.N; P.k_rows_per_problem = dm.N;
  P.inner = dm.b; P.inner_rows = 1; P.row_stride = dm.b;
  P.nq = dm.T; P.nk = dm.T;
  P.nqb = (dm.T + BQ - 1) / BQ;
  P.nsplit = 1;
  P.keys_per_split = ((dm.T + BK - 1) / BK) * BK;
  const long long total = (long long)dm.BH * dm.b * P.nqb;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = q_scale; P.cr_min = 0.f;
  P.kb_scale = -LOG2E;
  const bool d128 = dm.d == 128;
  if (y != nullptr) {
    P.q = q; P.k = aL; P.v = y; P.outv = out; P.kbias = cL;
    return d128 ? launch_flash<128, false, true, 0, false, 1>(P, st) : launch_flash<64, false, true, 0, false, 1>(P, st);
  }
  if (lse_scratch == nullptr) return hipErrorInvalidValue;
  P.q = q; P.k = aL; P.outk = nullptr; P.lse = lse_scratch; P.kbias = cL;
  hipError_t e = d128 ? launch_flash<128, true, false, 0, false, 1>(P, st) : launch_flash<64, true, false, 0, false, 1>(P, st);
  if (e != hipSuccess) return e;
  P.q = aL; P.k = q; P.outk = aR; P.cl = cR; P.lse = nullptr;
  P.kbias = lse_scratch;          // natural log, like c_L: the same scale -log2(e) applies
  P.qbias = cL; P.qb_scale = LOG2E;
  return d128 ? launch_flash<128, true, false, 0, false, 2>(P, st) : launch_flash<64, true, false, 0, false, 2>(P, st);
}

// Attention-sink averaging (Sec. 4.4): all N queries of a head against its first frame's b keys,
// one key range, the normalised rows averaged into `out` by the epilogue.
hipError_t launch_sink_average_flash(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, const Dims& dm,
                                     hipStream_t st) {
  FlashParams P = {};
  P.q = q; P.k = k; P.v = v; P.outv = out;
  P.q_rows_per_problem = dm.N; P.k_rows_per_problem = dm.N;
  if (dm.N > 0x7fffffffLL - BQ) return hipErrorInvalidValue;
  P.nq = (int)dm.N;
  P.nk = dm.b;
  P.nqb = (int)((dm.N + BQ - 1) / BQ);
  P.nsplit = 1;
  P.keys_per_split = ((dm.b + BK - 1) / BK) * BK;
  long long total = (long long)dm.BH * P.nqb;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = 1.0f / sqrtf((float)dm.d);
  P.cr_min = 0.f;
  P.blend = 1;
  return dm.d == 128 ? launch_flash<128, false, true, 0, false>(P, st) : launch_flash<64, false, true, 0, false>(P, st);
}

}  // namespace vm
