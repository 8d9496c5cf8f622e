// Last R-update of a call in one pass: alpha_L = R K, c_L and y = R V from a single evaluation
// of the logits and of the softmax (Eq. R + Eq. alpha_L/c_L and the y = R V of App. A; Alg. 1
// with the running max / sum / entropy of App. B), bf16 MFMA, d = 64 or 128.
//
// Both accumulator sets do not fit one wave's registers (two waves share a SIMD's file), so
// two waves share 32 query rows instead: wave `pair` (role 0) accumulates R K, wave `pair + 4`
// (role 1, same SIMD) accumulates R V, and they take turns producing the probabilities.  Keys
// stream in 64-row tiles.  In step s (one workgroup barrier per step):
//   both waves      O^T += X^T P(s)^T with X = K (role 0) or V (role 1), P(s) read from LDS;
//   producer of s+1 (role == (s+1) & 1) turns its logits of tile s+1 into P(s+1): row maxima,
//                   reference update, p = 2^t, running l and h for its own tiles, bf16 P^T and
//                   the reference it is relative to, written to LDS for both waves;
//   the other wave  forms the logits S^T = K Q^T of tile s+2, which it will turn into P(s+2)
//                   in the next step.
// So in every step one wave of the pair issues 32 MFMAs and the other 16 MFMAs plus the whole
// vector work, and the roles swap.  Per tile and 32 queries that is 48 MFMAs and one softmax
// against 64 and two for the two-pass form (logits and softmax evaluated once per output).
//
// References: a producer moves the pair's reference max only when a row maximum outgrew it by
// 2^RESCALE_TH, rescales its own accumulators and sums, and publishes the new reference with
// P; the partner adopts it (and rescales) before it adds that P.  l and h are per-wave partial
// sums over the tiles the wave produced, relative to the common final reference, and are added
// in the epilogue.
#include <type_traits>

#include "common.h"
#include "flash_device.h"

namespace vm {

namespace {

constexpr int KV_PAIRS = 4;           // wave pairs per workgroup
constexpr int KV_BQ = 32 * KV_PAIRS;  // query rows per workgroup
constexpr int KV_KSLOT = 4;           // K tiles: s (products), s+1 (landed), s+2 (logits), s+3 (in flight)
constexpr int KV_VSLOT = 2;           // V tiles: s (products), s+1 (in flight)

template <int D>
struct KvLds {
  static constexpr int TILE_BYTES = BK * RowGeo<D>::ROW_BYTES;
  static constexpr int V_OFF = KV_KSLOT * TILE_BYTES;
  static constexpr int PX_OFF = V_OFF + KV_VSLOT * TILE_BYTES;  // P^T exchange: [2][pair][4 operands][64 lanes][16 B]
  static constexpr int PX_BUF = KV_PAIRS * 4096;
  static constexpr int MX_OFF = PX_OFF + 2 * PX_BUF;            // references: [2][pair][64 lanes] floats
  static constexpr int MX_BUF = KV_PAIRS * 256;
  static constexpr int BYTES = MX_OFF + 2 * MX_BUF;
  // the epilogue stages 8 x 32 output rows over the K slots and exchanges (l, h) in the P area
  static_assert(8 * 32 * RowGeo<D>::ROW_BYTES <= PX_OFF, "staged rows stay clear of the exchange area");
};

template <int D>
__global__ void __launch_bounds__(512) flash_kv_kernel(FlashParams P) {
  using G = RowGeo<D>;
  using L = KvLds<D>;
  constexpr int ROW_BYTES = G::ROW_BYTES;
  constexpr int TILE_BYTES = L::TILE_BYTES;
  constexpr int KS = G::KS;
  constexpr int CT = G::CT;
  constexpr int CH = G::CH;
  constexpr int RPI = G::RPI;
  auto swz = [](int row) { return G::swz(row); };
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // XCD-aware placement, as in flash_kernel: one contiguous range of work items per XCD
  const int bid = blockIdx.x;
  const int wid = (bid & 7) * P.blocks_per_xcd + (bid >> 3);
  if (wid >= P.total_blocks) return;
  const int prob = wid / P.nqb;
  const int qb = wid - prob * P.nqb;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int ql = lane & 31;
  const int g = lane >> 5;
  const int pair = wave & (KV_PAIRS - 1);
  const int role = wave >> 2;  // 0: accumulates R K, produces even tiles; 1: R V, odd tiles

  const int nkeys = P.nk;
  const int ntiles = (nkeys + BK - 1) / BK;
  const long long qrow0 = (long long)prob * P.q_rows_per_problem;
  const bf16_t* kbase = P.k + (long long)prob * P.k_rows_per_problem * D;
  const bf16_t* vbase = P.v + (long long)prob * P.k_rows_per_problem * D;

  // ---- global -> LDS staging (see flash_kernel for the addressing and for why this is inline asm)
  static_assert(BK % (RPI * NW) == 0, "every wave issues the same number of loads per tile");
  const int st_key = RPI * wave + lane / CH;
  const int st_lc = (lane % CH) ^ swz(st_key);
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)smem;
  auto issue_rows = [&](const bf16_t* base, int t, unsigned slot_addr) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < BK / (RPI * NW); ++r) {
      const int key = min(t * BK + RPI * NW * r + st_key, nkeys - 1);  // rows past the end: copies of the last row
      const bf16_t* src = base + (long long)key * D + st_lc * 8;
      const unsigned dst = __builtin_amdgcn_readfirstlane(slot_addr + (RPI * NW * r + RPI * wave) * ROW_BYTES);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(dst) : "memory", "m0");
    }
  };
  auto issue_k = [&](int t) __attribute__((always_inline)) { issue_rows(kbase, t, lds_base + (t & (KV_KSLOT - 1)) * TILE_BYTES); };
  auto issue_v = [&](int t) __attribute__((always_inline)) { issue_rows(vbase, t, lds_base + L::V_OFF + (t & (KV_VSLOT - 1)) * TILE_BYTES); };
  issue_k(0);
  issue_v(0);
  if (ntiles > 1) issue_k(1);
  if (ntiles > 2) issue_k(2);

  // ---- queries: B operand of S^T = K Q^T, in registers ------------------------------------
  const int qr = qb * KV_BQ + pair * 32 + ql;
  const bool qvalid = qr < P.nq;
  const int qrow = qvalid ? qr : P.nq - 1;
  bf16x8 qreg[KS];
  {
    const bf16_t* qp = P.q + (qrow0 + qrow) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }
  const float sc = P.row_scale * LOG2E / fmaxf(P.cR ? P.cR[qrow0 + qrow] : 1.0f, P.cr_min);

  // row reads (A of S^T): key row = 32 st + ql, logical chunk 2 ks + g
  // Only the offsets for ks = 0 are kept in registers: chunk (2 ks + g) ^ swz = (2 ks) ^ (g ^ swz), so the
  // offset for ks is a0 ^ (ks << 5) (the row part is a multiple of the swizzled span).
  const int a0 = ql * ROW_BYTES + ((g ^ swz(ql)) << 4);
  auto a_off = [&](int ks) __attribute__((always_inline)) { return a0 ^ (ks << 5); };
  // transpose reads (A of O^T += X^T P^T), as in flash_kernel; likewise only channel tile 0 is kept:
  // chunk (4 ct + low) ^ swz = (4 ct) ^ (low ^ swz), the offset for ct is t0[hh] ^ (ct << 6)
  int t0[2];
  {
    const int rp = lane & 15;
    const int chh = (lane >> 4) & 1;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int key = 8 * hh + 4 * g + (rp >> 2);
      const int lc = 2 * chh + ((rp >> 1) & 1);
      t0[hh] = key * ROW_BYTES + ((lc ^ swz(key)) << 4) + ((rp & 1) << 3);
    }
  }
  auto t_off = [&](int ct, int hh) __attribute__((always_inline)) { return t0[hh] ^ (ct << 6); };
  static_assert(ROW_BYTES >= 128, "the xor stays inside one row");

  f32x16 oacc[CT];  // O^T tiles of this wave's product (R K or R V)
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[ct][r] = 0.f;
  float msc = NEG_BIG, ltil = 0.f, hsum = 0.f;
  f32x16 sacc[2];  // logits of the tile this wave produces next, two 32-key sub-tiles

  // ---- building blocks --------------------------------------------------------------------
  // Operands of one group of CT products O^T += X^T P^T: the B operand P^T of 16 keys (group
  // grp = 2 st + c of the tile, keys 16 grp .. 16 grp + 15) and CT transposed A operands.
  struct AccOps {
    bf16x8 pb;
    bf16x8 a[CT];
  };
  auto load_acc = [&](const char* xtile, const char* px, int grp, AccOps& o) __attribute__((always_inline)) {
    o.pb = *reinterpret_cast<const bf16x8*>(px + grp * 1024);
    const int koff = grp * 16 * ROW_BYTES;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      bf16x4 lo = lds_read_tr(xtile + koff + t_off(ct, 0));
      bf16x4 hi = lds_read_tr(xtile + koff + t_off(ct, 1));
      o.a[ct] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  auto mma_acc = [&](const AccOps& o) __attribute__((always_inline)) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[ct], o.pb, oacc[ct], 0, 0, 0);
  };
  // A operands of S^T = K Q^T for k-steps 2 q, 2 q + 1 (q = 0 .. KS/2 - 1) of both 32-key sub-tiles
  struct LogOps {
    bf16x8 a[2][2];  // [sub-tile][k-step within the group]
  };
  auto load_log = [&](const char* ktile, int q, LogOps& o) __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int e = 0; e < 2; ++e) o.a[st][e] = lds_read_b128(ktile + st * 32 * ROW_BYTES + a_off(2 * q + e));
  };
  auto mma_log = [&](const LogOps& o, int q) __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
      for (int st = 0; st < 2; ++st)  // alternate the two accumulators
        sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[st][e], qreg[2 * q + e], sacc[st], 0, 0, 0);
  };
  auto zero_sacc = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[st][r] = 0.f;
  };
  // plain forms for the prologue and the ends of the key range
  auto logits = [&](const char* ktile) __attribute__((always_inline)) {
    zero_sacc();
#pragma unroll
    for (int q = 0; q < KS / 2; ++q) {
      LogOps o;
      load_log(ktile, q, o);
      mma_log(o, q);
    }
  };
  auto accumulate = [&](const char* xtile, const char* px) __attribute__((always_inline)) {
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      AccOps o;
      load_acc(xtile, px, grp, o);
      mma_acc(o);
    }
  };
  // Rescale everything this wave holds from reference msc to reference m_new (<= 0 in log2 of the factor).
  auto move_sums = [&](float m_new) __attribute__((always_inline)) -> float {
    const float dl = msc - m_new;
    const float alpha = __builtin_amdgcn_exp2f(dl);
    hsum = alpha * (hsum + dl * ltil);  // h <- a h + a log(a) l  (App. B)
    ltil *= alpha;
    msc = m_new;
    return alpha;
  };
  auto scale_all = [&](float alpha) __attribute__((always_inline)) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) scale_acc(oacc[ct], alpha);
  };
  // Reference update for the logits in sacc (tile t): returns the rescale factor for this wave's
  // accumulators, or a negative value when the reference stays.
  auto new_reference = [&](int t, auto may_be_ragged) __attribute__((always_inline)) -> float {
    const int left = nkeys - t * BK;  // >= 1
    if (decltype(may_be_ragged)::value && left < BK) {
      // ragged end: rows left .. 63 of this tile are copies of the last valid row
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sacc[st][r] += (32 * st + 8 * (r >> 2) + 4 * g + (r & 3)) >= left ? -1.0e9f : 0.f;
    }
    const float cand = fmaxf(subtile_max(sacc[0]), subtile_max(sacc[1])) * sc;
    const bool grow = __any(cand > msc + RESCALE_TH);
    const float alpha = move_sums(grow ? fmaxf(msc, cand) : msc);
    return grow ? alpha : -1.0f;
  };
  auto p_out = [&](int t) __attribute__((always_inline)) -> char* {
    return smem + L::PX_OFF + (t & 1) * L::PX_BUF + pair * 4096 + lane * 16;
  };
  // bf16 P^T of 16 keys (group grp of tile t) from the logits in sacc, published for both waves
  auto probs_group = [&](char* px, auto grp_c) __attribute__((always_inline)) {
    constexpr int GRP = decltype(grp_c)::value;
    const bf16x8 pb = halftile_probs<GRP & 1>(sacc[GRP >> 1], sc, msc, ltil, hsum);
    *reinterpret_cast<bf16x8*>(px + GRP * 1024) = pb;
  };
  auto publish_reference = [&](int t) __attribute__((always_inline)) {
    *reinterpret_cast<float*>(smem + L::MX_OFF + (t & 1) * L::MX_BUF + pair * 256 + lane * 4) = msc;
  };
  // Turn the logits in sacc (tile t) into P(t), plain form
  auto produce = [&](int t, auto may_be_ragged) __attribute__((always_inline)) -> float {
    const float alpha = new_reference(t, may_be_ragged);
    char* px = p_out(t);
    probs_group(px, std::integral_constant<int, 0>{});
    probs_group(px, std::integral_constant<int, 1>{});
    probs_group(px, std::integral_constant<int, 2>{});
    probs_group(px, std::integral_constant<int, 3>{});
    publish_reference(t);
    return alpha;  // the caller rescales its accumulators after the products against the old reference
  };

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // K tiles 0..2 and V tile 0 have landed
  // A pair whose 32 query rows all lie past the end of the problem only helps to load the tiles.
  const bool active = qb * KV_BQ + pair * 32 < P.nq;
  if (active) {
    if (role == 0) {
      logits(smem);
      (void)produce(0, std::true_type{});  // the accumulators are still zero
    } else if (ntiles > 1) {
      logits(smem + TILE_BYTES);
    }
  }
  __syncthreads();  // P(0) is published

  // Every wave walks steps 0 .. ntiles-1 with one barrier at the end of each.  A wave alternates
  // between the two kinds of step; written as a loop over (heavy, light) pairs so that the logits
  // formed in a heavy step die in the light step that follows, with role 1 taking step 0 (light)
  // ahead of its loop.
  auto begin_step = [&](int s) __attribute__((always_inline)) {
    if (s + 3 < ntiles) issue_k(s + 3);  // into the slot of tile s-1
    if (s + 1 < ntiles) issue_v(s + 1);  // likewise
  };
  auto end_step = [&](int s) __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // P(s+1) published, tiles s+3 / s+1 landed, everyone done with tile s
  };
  auto x_tile = [&](int s) __attribute__((always_inline)) -> const char* {
    return role == 0 ? smem + (s & (KV_KSLOT - 1)) * TILE_BYTES : smem + L::V_OFF + (s & (KV_VSLOT - 1)) * TILE_BYTES;
  };
  auto p_slot = [&](int s) __attribute__((always_inline)) -> const char* { return smem + L::PX_OFF + (s & 1) * L::PX_BUF + pair * 4096 + lane * 16; };
  // Main-loop forms of the two steps, written as explicit pipelines: every chunk (between two scheduling
  // fences) issues the LDS reads of the next group of four MFMAs, then the MFMAs whose operands the
  // previous chunk fetched, then (light step) a quarter of the vector work.
#define KV_FENCE() __builtin_amdgcn_sched_barrier(0)
  // this wave produced P(s): add it, then form the logits of tile s+2
  auto heavy_work = [&](int s) __attribute__((always_inline)) {
    const char* xt = x_tile(s);
    const char* px = p_slot(s);
    const char* kt = smem + ((s + 2) & (KV_KSLOT - 1)) * TILE_BYTES;
    AccOps o0, o1;
    LogOps l0, l1;
    load_acc(xt, px, 0, o0);
    KV_FENCE();
    load_acc(xt, px, 1, o1);
    mma_acc(o0);
    KV_FENCE();
    load_acc(xt, px, 2, o0);
    mma_acc(o1);
    KV_FENCE();
    load_acc(xt, px, 3, o1);
    mma_acc(o0);
    zero_sacc();
    KV_FENCE();
    load_log(kt, 0, l0);
    mma_acc(o1);
    KV_FENCE();
#pragma unroll
    for (int q = 0; q < KS / 2; q += 2) {
      if (q + 1 < KS / 2) load_log(kt, q + 1, l1);
      mma_log(l0, q);
      KV_FENCE();
      if (q + 2 < KS / 2) load_log(kt, q + 2, l0);
      if (q + 1 < KS / 2) mma_log(l1, q + 1);
      KV_FENCE();
    }
  };
  // P(s) came from the partner: adopt its reference, add it, and turn the logits of tile s+1 into P(s+1)
  auto light_work = [&](int s, auto may_be_ragged) __attribute__((always_inline)) {
    const float m_in = *reinterpret_cast<const float*>(smem + L::MX_OFF + (s & 1) * L::MX_BUF + pair * 256 + lane * 4);
    if (__any(m_in != msc)) scale_all(move_sums(m_in));
    const char* xt = x_tile(s);
    const char* px = p_slot(s);
    char* po = p_out(s + 1);
    AccOps o0, o1;
    load_acc(xt, px, 0, o0);
    const float alpha = new_reference(s + 1, may_be_ragged);
    KV_FENCE();
    load_acc(xt, px, 1, o1);
    mma_acc(o0);
    probs_group(po, std::integral_constant<int, 0>{});
    KV_FENCE();
    load_acc(xt, px, 2, o0);
    mma_acc(o1);
    probs_group(po, std::integral_constant<int, 1>{});
    KV_FENCE();
    load_acc(xt, px, 3, o1);
    mma_acc(o0);
    probs_group(po, std::integral_constant<int, 2>{});
    KV_FENCE();
    mma_acc(o1);
    probs_group(po, std::integral_constant<int, 3>{});
    publish_reference(s + 1);
    KV_FENCE();
    if (alpha >= 0.f) scale_all(alpha);
  };
  // the same two steps near the ends of the key range, where tile s+2 / s+1 may not exist
  auto heavy_edge = [&](int s) __attribute__((always_inline)) {
    begin_step(s);
    if (active) {
      accumulate(x_tile(s), p_slot(s));
      if (s + 2 < ntiles) logits(smem + ((s + 2) & (KV_KSLOT - 1)) * TILE_BYTES);
    }
    end_step(s);
  };
  auto light_edge = [&](int s) __attribute__((always_inline)) {
    begin_step(s);
    if (active) {
      const float m_in = *reinterpret_cast<const float*>(smem + L::MX_OFF + (s & 1) * L::MX_BUF + pair * 256 + lane * 4);
      if (__any(m_in != msc)) scale_all(move_sums(m_in));
      accumulate(x_tile(s), p_slot(s));
      if (s + 1 < ntiles) {
        const float alpha = produce(s + 1, std::true_type{});
        if (alpha >= 0.f) scale_all(alpha);
      }
    }
    end_step(s);
  };
  {
    int s = 0;
    if (role == 1) {
      light_edge(0);
      s = 1;
    }
    {
      // main loop: tiles s+2 and s+3 exist and are full, no branch inside a step's arithmetic
      if (active) {
        for (; s + 3 < ntiles; s += 2) {
          begin_step(s);
          heavy_work(s);
          end_step(s);
          begin_step(s + 1);
          light_work(s + 1, std::false_type{});
          end_step(s + 1);
        }
      } else {
        for (; s + 3 < ntiles; s += 2) {
          begin_step(s);
          end_step(s);
          begin_step(s + 1);
          end_step(s + 1);
        }
      }
      for (; s < ntiles; s += 2) {
        heavy_edge(s);
        if (s + 1 < ntiles) light_edge(s + 1);
      }
    }
  }

  // ---- epilogue ------------------------------------------------------------------------------
  // Lane-dependent values are derived again from the thread index, behind an opaque copy, so that
  // nothing of the epilogue's address arithmetic stays live (or gets spilled) across the key loop.
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int lane_e = tid_e & 63;
  const int ql_e = lane_e & 31;
  const int g_e = lane_e >> 5;
  const int qr_e = qb * KV_BQ + pair * 32 + ql_e;
  const bool qvalid_e = qr_e < P.nq;
  // (l, h) of the two waves are partial sums over disjoint tiles, relative to the same reference.
  float2* xs = reinterpret_cast<float2*>(smem + L::PX_OFF) + (pair * 2) * 64;
  xs[role * 64 + lane_e] = make_float2(ltil, hsum);
  __syncthreads();
  {
    const float2 o = xs[(role ^ 1) * 64 + lane_e];
    ltil += o.x;
    hsum += o.y;
  }
  const float lt = ltil + __shfl_xor(ltil, 32);
  const float inv = lt > 0.f ? 1.0f / lt : 0.f;
  const float h = hsum + __shfl_xor(hsum, 32);
  if (role == 0 && qvalid_e && g_e == 0) {
    const long long row = (long long)prob * P.q_rows_per_problem + qr_e;
    if (P.lse != nullptr) P.lse[row] = LN2 * (msc + __log2f(lt));
    // App. B: H = log S - L / S, here in base-2 units; c_L = -H
    P.cl[row] = -LN2 * (__log2f(lt) - h * inv);
  }
  char* stage = smem + wave * (32 * ROW_BYTES);
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint2 w;
      w.x = pack_bf16(oacc[ct][4 * c + 0] * inv, oacc[ct][4 * c + 1] * inv);
      w.y = pack_bf16(oacc[ct][4 * c + 2] * inv, oacc[ct][4 * c + 3] * inv);
      *reinterpret_cast<uint2*>(stage + ql_e * ROW_BYTES + (((4 * ct + c) ^ swz(ql_e)) << 4) + 8 * g_e) = w;
    }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the staged rows are private to the wave
  __builtin_amdgcn_wave_barrier();
  bf16_t* dst = (role == 0 ? P.outk : P.outv) + (long long)prob * P.q_rows_per_problem * D;
  const int row_first = qb * KV_BQ + pair * 32;
#pragma unroll
  for (int ps = 0; ps < 32 / RPI; ++ps) {
    const int lr = ps * RPI + lane_e / CH;
    const int pc = lane_e % CH;
    const int lc = pc ^ swz(lr);
    if (row_first + lr < P.nq) {
      uint4 w = *reinterpret_cast<const uint4*>(stage + lr * ROW_BYTES + pc * 16);
      *reinterpret_cast<uint4*>(dst + (long long)(row_first + lr) * D + lc * 8) = w;
    }
  }
}

#undef KV_FENCE

template <int D>
hipError_t launch_kv(const FlashParams& P, hipStream_t st) {
  constexpr int LDS_BYTES = KvLds<D>::BYTES;
  auto kern = flash_kv_kernel<D>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(P.blocks_per_xcd * 8), dim3(512), LDS_BYTES, st, P);
  return hipGetLastError();
}

}  // namespace

// alpha_L, c_L (and lse if not null) and y of one R-update, online entropy, in one pass
hipError_t launch_r_update_flash_fused(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL,
                                       float* cL, bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min,
                                       hipStream_t st) {
  if (!(dm.d == 128 || dm.d == 64) || v == nullptr || y == nullptr) return hipErrorInvalidValue;
  FlashParams P = {};
  P.q = aR; P.cR = cR; P.k = k; P.v = v; P.outk = aL; P.outv = y; P.cl = cL; P.lse = lse;
  P.q_rows_per_problem = dm.b; P.k_rows_per_problem = dm.b;
  P.nq = dm.b; P.nk = dm.b;
  P.nqb = (dm.b + KV_BQ - 1) / KV_BQ;
  P.nsplit = 1;
  P.keys_per_split = ((dm.b + BK - 1) / BK) * BK;
  const long long total = (long long)dm.BH * dm.T * P.nqb;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  P.row_scale = row_scale; P.cr_min = cr_min;
  return dm.d == 128 ? launch_kv<128>(P, st) : launch_kv<64>(P, st);
}

}  // namespace vm
