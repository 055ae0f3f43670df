// Grouped bf16 GEMM on MFMA for expert blocks with many rows per expert (prefill-sized batches).
// FaaSMoE Sec. 3: an expert block holds several experts and computes on the tokens handed to it;
// Sec. 4.1: the tokens of one block arrive as one batch.  Here a block is an expert range
// [lo,hi) and its batch is a contiguous row range, cut per expert by expert_offsets.
//
// Two instantiations of one kernel:
//   gate/up : h[r, n]  = silu(<A[r,:], Wg[e][n,:]>) * <A[r,:], Wu[e][n,:]>      (A = Xp, Kdim = H)
//   down    : Yp[r, n] = <A[r,:], Wd[e][n,:]>                                   (A = h,  Kdim = I)
// Both operands are K-contiguous, so token rows and weight rows are staged the same way.
//
// Work decomposition.  A tile is BM token rows of ONE expert by BN weight rows (gate/up: BN/2 gate
// rows and the matching BN/2 up rows, so the SwiGLU product is formed in registers).  The number
// of tiles depends on expert_offsets, which only the device knows: the kernel is persistent, every
// workgroup first builds the per-expert tile prefix in LDS and then walks tile indices with a
// fixed stride, so there is no host synchronisation and no atomic.  Workgroup b runs on XCD
// b mod 8; the index walk hands each XCD runs of consecutive tiles that share weight and token
// panels, so they meet in that XCD's L2.
//
// Inside a tile: 4 waves, K steps of 64 through a ring of NS LDS stages.  Both panels are copied
// from global memory straight into LDS (global_load_lds, 16 bytes per lane, no registers in
// between).  Eight lanes fetch one row's 128 bytes, so every request is a whole cache line: with
// 64-byte requests the L2-to-LDS path delivered 27 B/clk per CU, with 128-byte requests 47 B/clk
// (measured), and these kernels live on that path.  NS-1 stages are in flight while one is
// multiplied.  The copies are asynchronous: a wave waits with s_waitcnt vmcnt(n) until only the
// copies of later stages are outstanding, then one workgroup barrier per K step publishes the
// stage.  A stage is multiplied in four 16-wide K slices; operand fragments are double-buffered in
// registers and every LDS read is issued one slice ahead of its use, between the MFMAs of the
// slice before.  A row's eight 16-byte chunks are stored at slot = chunk xor row%8 so the MFMA
// operand reads (32 rows, same chunk) are bank-conflict free.  MFMA 32x32x16 bf16 with the WEIGHT rows as the
// first operand and the TOKEN rows as the second: a lane then owns 4 consecutive output columns
// of one token row per accumulator quad, which makes the bf16 stores 8 bytes wide.
// Rows past the end of an expert are clamped on load (they recompute the expert's last row) and
// masked on store, which keeps the K loop free of branches.
#include <math.h>
#include <atomic>
#include <type_traits>
#include "common.h"

namespace moe {

template <int BM, int BN, int WAVES_M, int WAVES_N, bool GATEUP, int NS>
struct TileShape {
  static constexpr int BK = 64;
  static constexpr int ROWB = BK * 2;             // bytes per staged row (8 chunks of 16 bytes)
  static constexpr int WTM = BM / WAVES_M;        // token rows per wave
  static constexpr int WTN = BN / WAVES_N;        // weight rows per wave
  static constexpr int TB = WTM / 32;             // 32-row token blocks per wave
  static constexpr int NB = WTN / 32;             // 32-row weight blocks per wave
  static constexpr int NBH = GATEUP ? NB / 2 : NB;
  static constexpr int STAGE = (BM + BN) * ROWB;  // bytes per LDS stage
  static constexpr int NL = (BM + BN) / 32;       // 1 KB (8-row) copies per wave and stage
  static constexpr int NLA = BM / 32;             // the first NLA of them are token rows
  static constexpr int NF = TB + NB;              // operand fragments per wave and 16-wide K slice
  static constexpr int NM = TB * NB;              // MFMAs per wave and 16-wide K slice
  static constexpr int DIST = NS - 1;             // stages in flight while one is being multiplied
  static constexpr int NOUT = GATEUP ? BN / 2 : BN;  // output columns per tile
  static constexpr int GM = BN >= 256 ? 4 : 1;    // token tiles per locality group of the tile walk
  // The NL copies of a stage are requested in three places, so that the address unit of the CU
  // (one copy instruction of 1 KB keeps it busy for about 16 clocks) is not asked for a whole stage
  // within one K slice: ISSUE0 of them while the last slice of the stage that frees the buffer is
  // multiplied, ISSUE1 and ISSUE2 during the first two slices of the next K step.
  static constexpr int ISSUE0 = NL - 2 * (NL / 3);
  static constexpr int ISSUE1 = NL / 3;
  static constexpr int ISSUE2 = NL / 3;
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 blocks");
  static_assert(!GATEUP || NB % 2 == 0, "gate and up blocks come in pairs");
  static_assert(BM % 32 == 0 && BN % 64 == 0, "copies of 8 rows are dealt to 4 waves");
  static_assert((NS - 1) * NL < 64, "the wait counter holds 6 bits");
};

constexpr int TILE_EMAX = 256;

// Order in which the operand fragments of a K slice are read: by the MFMA that needs them first.
// MFMA j of a slice multiplies weight block j % NB with token block j / NB, so weight block 0 and
// token block 0 come first, then the other weight blocks, then the token blocks.  Returns the
// fragment number in the numbering "token blocks 0..TB-1, then weight blocks".
__host__ __device__ constexpr int fragment_read_order(int slot, int tb, int nb) {
  return slot == 0 ? tb : (slot == 1 ? 0 : (slot <= nb ? tb + slot - 1 : slot - nb));
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool GATEUP, int NS, int OCC, int KSPLIT>
__global__ __launch_bounds__(256, OCC) void expert_tile_kernel(GemmArgs a) {
  using S = TileShape<BM, BN, WAVES_M, WAVES_N, GATEUP, NS>;
  extern __shared__ __align__(16) unsigned char smem[];
  // Experts come in two classes.  One with at least HEAVY_MIN token tiles reuses every weight panel
  // that often out of L2 and is bound by the matrix pipes; one with fewer streams its weights from
  // HBM for little arithmetic and is bound by memory.  Walking the experts in id order would run
  // long stretches of one kind (all CUs waiting for HBM, then HBM idle); instead the token tiles
  // of each class are listed separately (experts in order inside a class) and the walk draws
  // locality groups from the two lists in proportion, so both kinds are in flight at any time.
  constexpr int HEAVY_MIN = 3;
  __shared__ int s_pref[2][TILE_EMAX];    // token tiles of the same class before expert i of the block
  __shared__ int s_rb[TILE_EMAX];         // first row of expert i of the block
  __shared__ uint8_t s_eid[TILE_EMAX];    // its expert id (E <= 256)
  __shared__ int s_total[2];              // token tiles per class

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  // weight sets of this launch: the routed experts of the block, then the shared sets riding along
  const int nrouted = a.offsets ? a.hi - a.lo : (a.n_shared > 0 ? 0 : 1);
  const int nexp = nrouted + a.n_shared;     // at most TILE_EMAX (checked by the caller)

  // per-expert row range and number of token tiles -> exclusive prefix per class in LDS
  if (wave == 0) {
    int v[4], cnt[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      v[i] = 0;
      if (e < nexp) {
        const bool sh = e >= nrouted;
        const int eid = sh ? e - nrouted : (a.offsets ? (a.ids ? a.ids[a.lo + e] : a.lo + e) : 0);
        const int rb = sh ? a.rows_routed + eid * a.shared_rows : (a.offsets ? a.offsets[eid] : 0);
        const int re = sh ? rb + a.shared_rows : (a.offsets ? a.offsets[eid + 1] : a.rows_fixed);
        s_eid[e] = (uint8_t)eid;
        s_rb[e] = rb;
        v[i] = (max(re - rb, 0) + BM - 1) / BM;
      }
      cnt[v[i] >= HEAVY_MIN] += v[i];
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      int incl = cnt[c];
#pragma unroll
      for (int s = 1; s < 64; s <<= 1) {
        const int o = __shfl_up(incl, s, WAVE);
        if (lane >= s) incl += o;
      }
      int base = incl - cnt[c];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = lane * 4 + i;
        if (e < nexp) s_pref[c][e] = base;
        if ((v[i] >= HEAVY_MIN) == (c == 1)) base += v[i];
      }
      if (lane == 63) s_total[c] = incl;
    }
  }
  __syncthreads();
  const int total0 = s_total[0], total1 = s_total[1];
  const int grp0 = (total0 + S::GM - 1) / S::GM, grp1 = (total1 + S::GM - 1) / S::GM;   // locality groups per class
  const int ngrp = grp0 + grp1;
  const int NT = (a.N + S::NOUT - 1) / S::NOUT;
  const int Kdim = a.Kdim;
  const int nk = Kdim / S::BK / KSPLIT;          // K steps of one work item (a tile, or a K part of it)
  const int groupTiles = S::GM * NT;
  const int Lend = ngrp * groupTiles * KSPLIT;
  // Divisions of the walk, prepared once per workgroup so that finding a tile costs multiplications only:
  // light groups among the first g groups of the merged walk = (g * light_ratio) >> 32, with light_ratio =
  // ceil(grp0 * 2^32 / ngrp): monotone in g, rises by at most one per group, and is exactly grp0 at g = ngrp,
  // so every group of either class is drawn exactly once; x / groupTiles and pair / gather_div by a
  // multiply-high with one correction step.
  const unsigned long long light_ratio = ngrp > 0 ? ((((unsigned long long)grp0) << 32) + (unsigned)ngrp - 1ull) / (unsigned)ngrp : 0ull;
  const uint32_t gt_magic = groupTiles > 1 ? (uint32_t)(0x100000000ull / (unsigned)groupTiles) : 0u;   // (2^32 itself does not fit)
  const uint32_t gd = a.gather ? (uint32_t)a.gather_div : 1u;
  const uint32_t gd_magic = gd > 1u ? (uint32_t)(0x100000000ull / gd) : 0u;

  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  // copy assignment of this lane inside an 8-row block: row lane/8, 16-byte slot lane%8; the slot
  // holds chunk (slot xor row%8) of the row, which spreads the MFMA operand reads (32 rows at the
  // same chunk) over all banks.
  const int crow = lane >> 3;
  const int cchunk = (lane & 7) ^ (lane >> 3);
  // operand reads: row lane%32 of a 32-row block, chunk 2*kk + lane/32 of the row
  const int frag_row = lane & 31;
  const int frag_half = lane >> 5;
  const int frag_swz = lane & 7;

  // Tile walk.  Workgroup b runs on XCD b % 8.  Each XCD takes runs of `run` consecutive tile
  // indices (tiles that share panels), one per workgroup slot; with fewer tiles than slots the runs
  // shrink so that all eight XCDs still get an equal share.
  const int G = gridDim.x;
  const bool xcd_walk = (G % 8) == 0;
  const int slot = xcd_walk ? (int)(blockIdx.x >> 3) : 0;
  const int run = xcd_walk ? max(1, min(G >> 3, (Lend + 7) >> 3)) : 1;
  if (xcd_walk && slot >= run) return;

    // copy i (of NL) of K step kt into stage buffer st; all NL of them
#define MOE_TILE_ISSUE1(kt, st, i)                                                                  \
    copy_to_lds_16(((i) < S::NLA ? Ag : ((GATEUP && (i) >= S::NLA + (S::NL - S::NLA) / 2) ? Bg1 : Bg0)) + (size_t)(kt) * S::ROWB, \
                   coff[i], lds0 + (uint32_t)(st) * S::STAGE + (uint32_t)wave * 1024u + (uint32_t)(i) * 4096u);
#define MOE_TILE_ISSUE(kt, st)                                                                      \
    { _Pragma("unroll") for (int i = 0; i < S::NL; ++i) MOE_TILE_ISSUE1(kt, st, i); }

  // State of a tile: the current one (being multiplied, then stored) and, while the current one is
  // stored, the next one, whose first NS stages are already requested: the latency of those copies
  // hides behind the epilogue instead of opening every tile.
  struct TileState { int row0, rowEnd, rowsValid, n0, ks, cshift; bf16_t* cbase; bool valid; };
  const unsigned char *Ag = nullptr, *Bg0 = nullptr, *Bg1 = nullptr;
  uint32_t coff[S::NL];   // byte offsets of this lane's 16 bytes for each of the NL copies of a stage (K step 0)
  int it = 0;
  auto next_tile = [&]() -> TileState {
    TileState t{};
    int L = 0, mrow = 0, nt = 0, cls = 0;
    for (;; ++it) {
      L = xcd_walk ? ((it * 8 + (int)(blockIdx.x & 7)) * run + slot) : (it * G + (int)blockIdx.x);
      if (L >= Lend) { t.valid = false; return t; }
      const int Lt = KSPLIT > 1 ? L / KSPLIT : L;
      int grp = Lt, rem = 0;
      if (groupTiles > 1) {
        grp = (int)__umulhi((uint32_t)Lt, gt_magic);   // floor(2^32/d) underestimates the quotient by at most one
        rem = Lt - grp * groupTiles;
        if (rem >= groupTiles) { ++grp; rem -= groupTiles; }
      }
      // group grp of the merged walk: light groups are spread evenly between the heavy ones
      const int before = (int)(((unsigned long long)(unsigned)grp * light_ratio) >> 32);          // light groups among the first grp
      cls = (int)(((unsigned long long)(unsigned)(grp + 1) * light_ratio) >> 32) > before ? 0 : 1;
      mrow = (cls == 0 ? before : grp - before) * S::GM + rem % S::GM;
      nt = rem / S::GM;
      if (mrow < (cls == 0 ? total0 : total1)) break;
    }
    ++it;
    t.valid = true;
    t.ks = KSPLIT > 1 ? L % KSPLIT : 0;   // K part of this work item

    // expert of this token tile: last e with s_pref[cls][e] <= mrow (an expert of the other class
    // repeats its successor's prefix, so the last one is of this class)
    int elo = 0, ehi = nexp;
    while (ehi - elo > 1) {
      const int mid = (elo + ehi) >> 1;
      if (s_pref[cls][mid] <= mrow) elo = mid; else ehi = mid;
    }
    // (the same in every lane: readfirstlane keeps them in scalar registers)
    const int e = __builtin_amdgcn_readfirstlane(elo);
    const int eg = __builtin_amdgcn_readfirstlane((int)s_eid[e]);   // expert id, or the number of the shared set
    const bool sh = e >= nrouted;
    const int rb = __builtin_amdgcn_readfirstlane(s_rb[e]);
    t.row0 = __builtin_amdgcn_readfirstlane(rb + (mrow - s_pref[cls][e]) * BM);
    t.rowEnd = sh ? rb + a.shared_rows : (a.offsets ? a.offsets[eg + 1] : a.rows_fixed);
    t.rowsValid = min(BM, t.rowEnd - t.row0);
    t.n0 = nt * S::NOUT;
    // where this tile's rows go: a shared set may have an output tensor of its own
    const bool own_c = sh && a.Cs != nullptr;
    t.cbase = own_c ? a.Cs : a.C;
    t.cshift = own_c ? a.rows_routed : 0;

    const size_t kbeg = (size_t)t.ks * nk * S::BK;
    // token rows: with a gather list they are addressed from the start of A, through the list; a
    // shared set with token rows of its own reads them in order
    const bool own_a = sh && a.As != nullptr;
    const bool gathered = a.gather != nullptr && !own_a;
    Ag = reinterpret_cast<const unsigned char*>(
        own_a ? a.As + (size_t)(t.row0 - rb) * Kdim + kbeg : a.A + (gathered ? (size_t)0 : (size_t)t.row0 * Kdim) + kbeg);
    const uint32_t ldb = sh ? (uint32_t)a.ldb_shared : (uint32_t)Kdim;   // elements between consecutive weight rows
    Bg0 = reinterpret_cast<const unsigned char*>((sh ? a.Bs0 + (size_t)eg * a.shared_b_step : a.B0 + (size_t)eg * a.N * Kdim) + kbeg);
    Bg1 = GATEUP ? reinterpret_cast<const unsigned char*>((sh ? a.Bs1 + (size_t)eg * a.shared_b_step : a.B1 + (size_t)eg * a.N * Kdim) + kbeg)
                 : nullptr;
#pragma unroll
    for (int i = 0; i < S::NL; ++i) {
      const int row = (i * 4 + wave) * 8 + crow;        // row inside the stage: tokens first, then weights
      int grow;
      uint32_t ld = (uint32_t)Kdim;
      if (i < S::NLA) {
        grow = min(row, t.rowsValid - 1);
        if (gathered) {
          const uint32_t pair = (uint32_t)a.gather[t.row0 + grow];
          uint32_t tok = pair;
          if (gd > 1u) {
            tok = __umulhi(pair, gd_magic);
            if (pair - tok * gd >= gd) ++tok;
          }
          grow = (int)tok;
        }
      } else {
        int r = row - BM;
        if (GATEUP && i >= S::NLA + (S::NL - S::NLA) / 2) r -= BN / 2;   // second half: the up branch
        grow = min(t.n0 + r, a.N - 1);
        ld = ldb;
      }
      coff[i] = (uint32_t)grow * ld * 2u + (uint32_t)cchunk * 16u;
    }
    // all NS stages of the tile are requested up front
#pragma unroll
    for (int s = 0; s < NS; ++s) MOE_TILE_ISSUE(min(s, nk - 1), s);
    return t;
  };

  // Clock record of this workgroup (a measurement aid).  The clocks are read whether or not a record was asked
  // for (two scalar reads per tile): a branch between a K loop's last MFMAs and the epilogue's first read of the
  // accumulators would sit exactly where the compiler has to pad that pair with wait states, and it does not
  // look across such a branch (build.py checks the emitted code for this).  Only the final store is conditional.
  const bool clocked = a.clocks != nullptr && (int)blockIdx.x < a.clock_groups;
  long long clk_kloops = 0, clk_tiles = 0;
  const long long clk_begin = clock64(), wall_begin = wall_clock64();

  TileState cur = next_tile();
  while (cur.valid) {
    const int row0 = cur.row0, rowEnd = cur.rowEnd, rowsValid = cur.rowsValid, n0 = cur.n0, ks = cur.ks;
    bf16_t* const cbase = cur.cbase;
    const int cshift = cur.cshift;
    f32x16 acc[S::NB][S::TB];
#pragma unroll
    for (int nb = 0; nb < S::NB; ++nb)
#pragma unroll
      for (int tb = 0; tb < S::TB; ++tb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][tb][i] = 0.0f;

    // fragment f of the 16-wide K slice kk_ of a stage, LDS -> registers: f < TBc is the token block
    // f, otherwise the weight block f - TBc.  TBc <= TB is the number of 32-row token blocks of this
    // wave that hold rows of the expert: blocks of pure padding are neither read nor multiplied.
#define MOE_TILE_READ1(fa_, fb_, stage_, kk_, f_)                                                   \
    {                                                                                               \
      const unsigned char* As_ = smem + (stage_) * S::STAGE;                                         \
      const int cr_ = (((kk_) * 2 + frag_half) ^ frag_swz) << 4;                                     \
      if ((f_) < TBc) {                                                                             \
        fa_[(f_) < TBc ? (f_) : 0] = as_bf16x8(*reinterpret_cast<const u32x4*>(                    \
            As_ + (wm * S::WTM + (f_) * 32 + frag_row) * S::ROWB + cr_));                            \
      } else {                                                                                      \
        const int nb_ = (f_) < TBc ? 0 : (f_) - TBc;                                                \
        const int brow_ = GATEUP ? ((nb_ < S::NBH ? 0 : BN / 2) + wn * (S::WTN / 2) + (nb_ % S::NBH) * 32) \
                                 : (wn * S::WTN + nb_ * 32);                                         \
        fb_[nb_] = as_bf16x8(*reinterpret_cast<const u32x4*>(                                        \
            As_ + BM * S::ROWB + (brow_ + frag_row) * S::ROWB + cr_));                               \
      }                                                                                             \
    }
#define MOE_TILE_READ(fa_, fb_, stage_, kk_)                                                        \
    { _Pragma("unroll") for (int f = 0; f < NFc; ++f) MOE_TILE_READ1(fa_, fb_, stage_, kk_, f); }
#define MOE_TILE_MFMA1(fa_, fb_, j_)                                                                \
    acc[(j_) % S::NB][(j_) / S::NB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                       \
        fb_[(j_) % S::NB], fa_[(j_) / S::NB], acc[(j_) % S::NB][(j_) / S::NB], 0, 0, 0);
#define MOE_TILE_MMA(fa_, fb_)                                                                      \
    { _Pragma("unroll") for (int j = 0; j < NMc; ++j) MOE_TILE_MFMA1(fa_, fb_, j); }
    // One K slice: multiply the fragments in set X and, spread between the MFMAs, read the
    // fragments of slice kk_ of stage_ into set Y.  The scheduling fences pin that interleaving, so
    // no LDS read is issued in front of an idle matrix pipe.
#define MOE_TILE_SLICE(faX, fbX, faY, fbY, stage_, kk_)                                             \
    { _Pragma("unroll") for (int j = 0; j < NMc; ++j) {                                             \
        MOE_TILE_MFMA1(faX, fbX, j);                                                                \
        _Pragma("unroll") for (int f = 0; f < NFc; ++f)                                             \
          if (f * NMc / NFc == j) MOE_TILE_READ1(faY, fbY, stage_, kk_, fragment_read_order(f, TBc, S::NB)); \
        __builtin_amdgcn_sched_barrier(0x6);                                                        \
    } }
    // The same with copies I0 .. I1-1 of K step kt_issue_ (into buffer st_issue_) requested in between.
#define MOE_TILE_SLICE_ISSUE(faX, fbX, faY, fbY, stage_, kk_, kt_issue_, st_issue_, I0, I1)         \
    { _Pragma("unroll") for (int j = 0; j < NMc; ++j) {                                             \
        MOE_TILE_MFMA1(faX, fbX, j);                                                                \
        _Pragma("unroll") for (int q = 0; q < ((I1) - (I0)) + NFc; ++q)                             \
          if (q * NMc / (((I1) - (I0)) + NFc) == j) {                                               \
            constexpr int NE_ = S::NB + 1 < NFc ? S::NB + 1 : NFc;   /* reads needed early: before the copies */ \
            constexpr int NC_ = (I1) - (I0);                                                        \
            if (q < NE_) MOE_TILE_READ1(faY, fbY, stage_, kk_, fragment_read_order(q < NE_ ? q : 0, TBc, S::NB)) \
            else if (q < NE_ + NC_) { MOE_TILE_ISSUE1(kt_issue_, st_issue_, (q >= NE_ && q < NE_ + NC_) ? (I0) + q - NE_ : 0); } \
            else MOE_TILE_READ1(faY, fbY, stage_, kk_, fragment_read_order(q >= NE_ + NC_ ? q - NC_ : 0, TBc, S::NB)) \
          }                                                                                         \
        __builtin_amdgcn_sched_barrier(0x6);                                                        \
    } }
    // Last slice of a stage: multiply set B; between the MFMAs first request the first copies of the
    // stage that reuses the buffer just freed, then read slice 0 of the next stage into set A.
#define MOE_TILE_SLICE_LAST(next_stage_, kt_issue_, st_issue_)                                      \
    { _Pragma("unroll") for (int j = 0; j < NMc; ++j) {                                             \
        MOE_TILE_MFMA1(faB, fbB, j);                                                                \
        _Pragma("unroll") for (int q = 0; q < S::ISSUE0 + NFc; ++q)                                 \
          if (q * NMc / (S::ISSUE0 + NFc) == j) {                                                   \
            constexpr int NE_ = S::NB + 1 < NFc ? S::NB + 1 : NFc;                                  \
            if (q < NE_) MOE_TILE_READ1(faA, fbA, next_stage_, 0, fragment_read_order(q < NE_ ? q : 0, TBc, S::NB)) \
            else if (q < NE_ + S::ISSUE0) { MOE_TILE_ISSUE1(kt_issue_, st_issue_, (q >= NE_ && q < NE_ + S::ISSUE0) ? q - NE_ : 0); } \
            else MOE_TILE_READ1(faA, fbA, next_stage_, 0, fragment_read_order(q >= NE_ + S::ISSUE0 ? q - S::ISSUE0 : 0, TBc, S::NB)) \
          }                                                                                         \
        __builtin_amdgcn_sched_barrier(0x6);                                                        \
    } }

    // Pipeline.  All NS stages have been requested (next_tile); while stage kt is multiplied, stages
    // kt+1 .. kt+NS-1 are in flight.  Fragment sets A and B alternate over the four slices of a
    // stage; slice 0 of the NEXT stage is read (after the barrier that publishes it) while the last
    // slice is multiplied.  That barrier also tells every wave that stage kt has been read
    // completely, so its buffer can take the copy of stage kt+NS.
    // (Past the end of K the requests repeat the last K step into a buffer nobody reads again:
    // every iteration then issues the same number of copies and the wait counts stay constant.)
    auto pipeline = [&](auto tbc_) {
      constexpr int TBc = decltype(tbc_)::value;
      constexpr int NMc = TBc * S::NB;   // MFMAs per 16-wide K slice
      constexpr int NFc = TBc + S::NB;   // operand fragments per slice
      wait_copies_but<S::DIST * S::NL>();   // stage 0 (requested before the previous tile was stored) has landed
      workgroup_barrier();
      bf16x8 faA[S::TB], fbA[S::NB], faB[S::TB], fbB[S::NB];
      MOE_TILE_READ(faA, fbA, 0, 0);
      int st = 0;                                  // buffer of the stage being multiplied: kt % NS
      for (int kt = 0; kt + 1 < nk; ++kt) {
        const int st1 = st + 1 == NS ? 0 : st + 1;
        // the rest of the copies of K step kt-1+NS, whose first part went out during the last slice
        // of K step kt-1 (at kt = 0 this repeats copies of the prologue: same bytes, same place)
        const int ktd = min(kt - 1 + NS, nk - 1);
        const int std_ = st == 0 ? NS - 1 : st - 1;
        MOE_TILE_SLICE_ISSUE(faA, fbA, faB, fbB, st, 1, ktd, std_, S::ISSUE0, S::ISSUE0 + S::ISSUE1);
        MOE_TILE_SLICE_ISSUE(faB, fbB, faA, fbA, st, 2, ktd, std_, S::ISSUE0 + S::ISSUE1, S::NL);
        MOE_TILE_SLICE(faA, fbA, faB, fbB, st, 3);
        // this wave has finished reading stage kt once the last-slice fragments are in registers
        // (the empty asm makes the compiler wait for them; the fence keeps that wait behind the MFMAs)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tb = 0; tb < TBc; ++tb) asm volatile("" : "+v"(faB[tb]));
#pragma unroll
        for (int nb = 0; nb < S::NB; ++nb) asm volatile("" : "+v"(fbB[nb]));
        wait_copies_but<(S::DIST - 1) * S::NL>();
        workgroup_barrier();  // stage kt+1 is complete for everyone; stage kt is free for everyone
        MOE_TILE_SLICE_LAST(st1, min(kt + NS, nk - 1), st);
        st = st1;
      }
      MOE_TILE_SLICE(faA, fbA, faB, fbB, st, 1);
      MOE_TILE_SLICE(faB, fbB, faA, fbA, st, 2);
      MOE_TILE_SLICE(faA, fbA, faB, fbB, st, 3);
      MOE_TILE_MMA(faB, fbB);
      wait_lds_reads();
      wait_copies_but<0>();  // the repeated last-step copies of the final iterations: none may outlive the tile
      workgroup_barrier();   // the next tile's first copies overwrite stages other waves may still read
    };
    // token blocks of this wave that hold rows of the expert (at least one, so that the copies and
    // operand reads keep their places between MFMAs)
    const int tbv = min(S::TB, max(1, (rowsValid - wm * S::WTM + 31) >> 5));
    const long long clk_k0 = clock64();
    switch (tbv) {
      case 1: pipeline(std::integral_constant<int, 1>{}); break;
      case 2: if constexpr (S::TB >= 2) pipeline(std::integral_constant<int, 2>{}); break;
      case 3: if constexpr (S::TB >= 3) pipeline(std::integral_constant<int, 3>{}); break;
      case 4: if constexpr (S::TB >= 4) pipeline(std::integral_constant<int, 4>{}); break;
      default: if constexpr (S::TB >= 5) pipeline(std::integral_constant<int, 5>{}); break;
    }
    static_assert(S::TB <= 5, "token blocks per wave");
    clk_kloops += clock64() - clk_k0;
    ++clk_tiles;
#undef MOE_TILE_READ1
#undef MOE_TILE_MFMA1
#undef MOE_TILE_SLICE
#undef MOE_TILE_SLICE_LAST
#undef MOE_TILE_SLICE_ISSUE
#undef MOE_TILE_READ
#undef MOE_TILE_MMA

    // the stage buffers are free (final barrier of the pipeline): request the next tile's first
    // stages now, their way from L2 overlaps the stores below
    const TileState nxt = next_tile();

    // epilogue: accumulator element i of block (nb, tb) is output column
    // 8*(i/4) + 4*(lane/32) + i%4 of the block, token row lane%32: lanes l and l+32 hold the two
    // halves of every 8-column group of a row.  In the down projection the two lanes trade one
    // group each (lane l gives its half of group q+1 and takes the partner's half of group q), so
    // each then owns 8 consecutive columns and stores 16 bytes: half as many store instructions,
    // and a row receives whole 32-byte pieces.  Stores count in the same counter as the copy ring,
    // so the first K steps of the next tile wait for them (without any stores the routed down
    // projection at T=4096 takes 114 instead of 144 us); the wider stores bring it to 134 us.  The
    // gate/up kernels, whose tiles store half as much behind the SwiGLU arithmetic, keep 8-byte
    // stores (16-byte ones: equal for the routed experts, 2 % slower for the shared one).
    auto out_value = [&](int nb, int tb, int i) -> float {
      if (GATEUP) {
        const float g = acc[nb][tb][i];
        const float u = acc[nb + S::NBH][tb][i];
        return __fdividef(g, 1.0f + __expf(-g)) * u;
      }
      return acc[nb][tb][i];
    };
#pragma unroll
    for (int tb = 0; tb < S::TB; ++tb) {
      const int m = row0 + wm * S::WTM + tb * 32 + frag_row;
      if (m < rowEnd) {
        bf16_t* crow_out = cbase + (size_t)(m - cshift) * a.N;
#pragma unroll
        for (int nb = 0; nb < S::NBH; ++nb) {
          const int nblock = n0 + (GATEUP ? wn * (S::WTN / 2) : wn * S::WTN) + nb * 32;   // first column of the 32-column block
          if (nblock < a.N) {   // N is a multiple of 64 and nblock of 32: the block is inside or outside as a whole
            if (KSPLIT > 1) {   // fp32 partial sum of K part ks; summed in order by the reduce kernel
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int n = nblock + 4 * frag_half + 8 * q;
                float* part = a.Cpart + ((size_t)ks * a.rows_total + m) * a.N + n;
                *reinterpret_cast<float4*>(part) = make_float4(out_value(nb, tb, 4 * q), out_value(nb, tb, 4 * q + 1),
                                                               out_value(nb, tb, 4 * q + 2), out_value(nb, tb, 4 * q + 3));
              }
            } else if (GATEUP) {
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                uint2 o;
                o.x = pack_bf16x2(out_value(nb, tb, 4 * q), out_value(nb, tb, 4 * q + 1));
                o.y = pack_bf16x2(out_value(nb, tb, 4 * q + 2), out_value(nb, tb, 4 * q + 3));
                *reinterpret_cast<uint2*>(crow_out + nblock + 4 * frag_half + 8 * q) = o;
              }
            } else {
#pragma unroll
              for (int q = 0; q < 4; q += 2) {
                uint32_t ox = pack_bf16x2(out_value(nb, tb, 4 * q), out_value(nb, tb, 4 * q + 1));
                uint32_t oy = pack_bf16x2(out_value(nb, tb, 4 * q + 2), out_value(nb, tb, 4 * q + 3));
                uint32_t oz = pack_bf16x2(out_value(nb, tb, 4 * q + 4), out_value(nb, tb, 4 * q + 5));
                uint32_t ow = pack_bf16x2(out_value(nb, tb, 4 * q + 6), out_value(nb, tb, 4 * q + 7));
                // (x,y) = own half of group q, (z,w) = own half of group q+1.  After the trade lanes 0-31
                // hold group q complete in (x,y,z,w), lanes 32-63 group q+1.
                trade_halves(ox, oz);
                trade_halves(oy, ow);
                *reinterpret_cast<u32x4*>(crow_out + nblock + 8 * (q + frag_half)) = u32x4{ox, oy, oz, ow};
              }
            }
          }
        }
      }
    }
    cur = nxt;
  }
#undef MOE_TILE_ISSUE1
#undef MOE_TILE_ISSUE
  if (clocked && tid == 0) {
    long long* rec = a.clocks + 4 * (size_t)blockIdx.x;
    rec[0] = clock64() - clk_begin;
    rec[1] = wall_clock64() - wall_begin;
    rec[2] = clk_kloops;
    rec[3] = clk_tiles;
  }
}

static thread_local long long* t_clock_buffer = nullptr;
static thread_local int t_clock_groups = 0;
void set_tile_clock_buffer(long long* clocks, int groups) {
  t_clock_buffer = groups > 0 ? clocks : nullptr;
  t_clock_groups = clocks != nullptr && groups > 0 ? groups : 0;
}

// Compute units of the current device (asked on every launch: nothing is cached across devices or threads).
static int num_cus() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  return n;
}

// Sum of the KSPLIT fp32 partial outputs in ascending K part, rounded once to bf16.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int ksplit, long n4, long stride4,
                                                            bf16_t* __restrict__ C) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const float4* p = reinterpret_cast<const float4*>(part);
  float4 s = p[i];
  for (int k = 1; k < ksplit; ++k) {
    const float4 v = p[i + (long)k * stride4];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  uint2 o;
  o.x = pack_bf16x2(s.x, s.y);
  o.y = pack_bf16x2(s.z, s.w);
  reinterpret_cast<uint2*>(C)[i] = o;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool GATEUP, int NS, int OCC, int KSPLIT = 1>
static int launch_tile_t(const GemmArgs& a, hipStream_t st) {
  using S = TileShape<BM, BN, WAVES_M, WAVES_N, GATEUP, NS>;
  auto kern = expert_tile_kernel<BM, BN, WAVES_M, WAVES_N, GATEUP, NS, OCC, KSPLIT>;
  static_assert(KSPLIT == 1 || !GATEUP, "the SwiGLU product needs complete sums");
  if (a.Kdim % (S::BK * KSPLIT) != 0) return -2;
  if (KSPLIT > 1 && a.Cpart == nullptr) return -3;
  static_assert(OCC * (NS * S::STAGE + 3600) <= 160 * 1024, "LDS of the resident workgroups must fit a CU");
  // The kernel's LDS limit is raised once per device: one bit per device id, set after the call has
  // succeeded there (two threads may both make the call; it is idempotent).
  static std::atomic<uint64_t> attr_done{0};
  const int lds = NS * S::STAGE;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -4;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev >= 64 || !(attr_done.load(std::memory_order_acquire) & bit)) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return -4;
    if (dev < 64) attr_done.fetch_or(bit, std::memory_order_release);
  }
  const int nexp = (a.offsets ? a.hi - a.lo : (a.n_shared > 0 ? 0 : 1)) + a.n_shared;
  if (nexp > TILE_EMAX) return -2;
  const int NT = (a.N + S::NOUT - 1) / S::NOUT;
  const long mt_bound = (long)a.rows_total / BM + nexp;
  const long bound = ((mt_bound + S::GM - 1) / S::GM) * S::GM * NT * KSPLIT;
  // persistent workgroups: as many as fit on the chip at once (two per CU for the smaller tile)
  const long resident = (long)num_cus() * OCC;
  int grid = (int)(bound < resident ? bound : resident);
  if (grid <= 0) return 0;
  GemmArgs launched = a;
  launched.clocks = t_clock_buffer;
  launched.clock_groups = t_clock_groups;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, launched);
  if (hipGetLastError() != hipSuccess) return -4;
  if (KSPLIT > 1) {
    const long n4 = (long)a.rows_total * a.N / 4;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, a.Cpart, KSPLIT, n4, n4, a.C);
    if (hipGetLastError() != hipSuccess) return -4;
  }
  return 0;
}

// Tile shape codes: 256 = 256x256, 128/129 = 128 token rows x 256 weight rows, 130 = 128x128,
// 64 = 128x64 (for the down projection with a K cut into parts summed in order by a second kernel
// when the caller provides room for the partial sums); 0 = choose from layer-wide sizes only
// (never from the block bounds).
//
// One weight set on a known number of rows (the shared expert): the shape with the least estimated
// time.  A launch takes ceil(items / CUs) rounds of one tile each, a tile costs rows x columns x K
// times a per-shape factor (smaller tiles move more bytes per flop through LDS).  The factors come
// from timing the four shapes at T = 128 ... 8192 on the Qwen shape; the K cut pays a reduction
// pass over its fp32 partial sums.
int tile_down_ksplit(int Kdim) { return Kdim % 512 == 0 ? 8 : Kdim % 256 == 0 ? 4 : Kdim % 128 == 0 ? 2 : 1; }
int pick_tile_shape(int rows, int N, int Kdim, bool gateup, bool allow_kcut, bool leave_room) {
  struct Cand { int code, bm, nout; double c; };
  const Cand cands[4] = {{256, 256, gateup ? 128 : 256, 1.0}, {129, 128, gateup ? 128 : 256, 1.1},
                         {130, 128, gateup ? 64 : 128, 1.42}, {64, 128, gateup ? 32 : 64, 1.77}};
  const double cus = (double)num_cus();
  const double units_per_us = 2.1e6;   // 256x256x5632 tile: about 175 us
  int best = 129;
  double best_cost = 0.0;
  for (const Cand& k : cands) {
    int parts = 1;
    if (k.code == 256 && leave_room) continue;   // 256x256 holds all 512 registers of every SIMD
    if (k.code == 64) {
      if (!gateup && !allow_kcut) continue;   // 32 column tiles would leave most CUs idle
      if (!gateup) parts = tile_down_ksplit(Kdim);
    }
    const double items = (double)((rows + k.bm - 1) / k.bm) * (double)((N + k.nout - 1) / k.nout) * parts;
    const double rounds = (double)(long)((items + cus - 1) / cus);
    double cost = rounds * k.bm * k.nout * ((double)Kdim / parts) * k.c;
    if (parts > 1) cost += (4.0 + (double)rows * N * parts * 4.0 / 4.0e6) * units_per_us;
    if (best_cost == 0.0 || cost < best_cost) { best_cost = cost; best = k.code; }
  }
  return best;
}

// Routed experts: the row counts are known only on the device, so the tile height comes from the
// layer-wide mean (never from the block bounds).  An expert near the upper end of the expected
// spread (mean + 1.5 sqrt(mean) rows, the binomial spread of uniform routing) should fit its tiles
// with the least padded work: candidates 128, 160 and 256 rows, each row of a tile costing 1.41,
// 1.23 and 1.0 (smaller tiles move more panel bytes per flop; factors fitted at T = 8192).
// Measured on uniform routing at T = 768 ... 8192 the pick is the fastest shape or within 3 % of
// it; Zipf-skewed routing (mean 273, median 130) and the multi-tenant batch (mean 137) also run
// fastest on its choice (160).
static int pick_tile_rows(const GemmArgs& a, int tile_rows, int nout, bool down) {
  (void)nout;
  if (tile_rows != 0) return tile_rows;
  if (a.offsets == nullptr) return pick_tile_shape(a.rows_total, a.N, a.Kdim, !down, a.Cpart != nullptr, a.leave_room != 0);
  const double m = (double)a.mean_rows + 1.5 * sqrt((double)a.mean_rows);
  const int heights[3] = {129, 160, 256};
  const double factor[3] = {1.41, 1.23, 1.0};
  int best = 129;
  double best_cost = 0.0;
  for (int i = 0; i < 3; ++i) {
    const int bm = heights[i] == 129 ? 128 : heights[i];
    const double cost = ceil(m / bm) * bm * factor[i];
    if (best_cost == 0.0 || cost < best_cost) { best_cost = cost; best = heights[i]; }
  }
  return best;
}
int launch_tile_gateup(const GemmArgs& a, int tile_rows, hipStream_t st) {
  const int t = pick_tile_rows(a, tile_rows, 128, false);
  if (t == 64) return launch_tile_t<128, 64, 4, 1, true, 6, 1>(a, st);
  if (t == 130) return launch_tile_t<128, 128, 2, 2, true, 4, 1>(a, st);
  if (t >= 256) return launch_tile_t<256, 256, 2, 2, true, 2, 1>(a, st);
  if (t == 160) return launch_tile_t<160, 256, 1, 4, true, 3, 1>(a, st);
  return launch_tile_t<128, 256, 1, 4, true, 3, 1>(a, st);
}
int launch_tile_down(const GemmArgs& a, int tile_rows, hipStream_t st) {
  const int t = pick_tile_rows(a, tile_rows, 256, true);
  if (t == 64) {
    switch (a.Cpart ? tile_down_ksplit(a.Kdim) : 1) {   // without a buffer for the parts: whole K per tile
      case 8: return launch_tile_t<128, 64, 4, 1, false, 6, 1, 8>(a, st);
      case 4: return launch_tile_t<128, 64, 4, 1, false, 6, 1, 4>(a, st);
      case 2: return launch_tile_t<128, 64, 4, 1, false, 6, 1, 2>(a, st);
      default: return launch_tile_t<128, 64, 4, 1, false, 6, 1, 1>(a, st);
    }
  }
  if (t == 130) return launch_tile_t<128, 128, 2, 2, false, 4, 1>(a, st);
  if (t >= 256) return launch_tile_t<256, 256, 2, 2, false, 2, 1>(a, st);
  if (t == 160) return launch_tile_t<160, 256, 1, 4, false, 3, 1>(a, st);
  return launch_tile_t<128, 256, 1, 4, false, 3, 1>(a, st);
}

}  // namespace moe
