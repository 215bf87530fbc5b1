// Fault-injecting GEMM, R trials per workgroup, persistent workgroups (gfx950).
//
// Every trial of a campaign multiplies the SAME operands (paper Sec. IV-A: one fault per run of
// the unchanged application); only the accumulators differ once a fault has been applied.  So a
// workgroup can stage one A/B k-tile in LDS, read one set of MFMA fragments per wave, and feed
// them to R independent accumulator sets - one per trial.  Each trial still executes all of its
// 2*M*N*K flops on the matrix cores; what is shared is operand traffic: L2 -> LDS bytes and
// ds_read_b128 per MFMA both fall by the factor the tile shrinks less than R grows
// (R = 8 on a 128x64 tile: 3/8 of the bytes per flop of one 256x256 tile per trial).
//
// Handles trials whose fault is NONE, an accumulator flip (k-blocks are multiples of the
// 16-wide MFMA step, so every flip falls between two steps) or the paper's product-term fault
// (Sec. III-E: written back after the 16-term step holding the term), on problems with
// K % 64 == 0.  The library's partition kernel splits a batch into these trials and the
// operand-fault trials and writes one 6-word descriptor per trial in list order:
// {trial, row, col, event, w0, w1} - event = the MFMA step of the event or -1; a flip has
// w0 = the XOR mask; a product-term fault has bit 30 of event set and w0, w1 = the words of re
// and re_err; an operand fault has bit 29 set, w0 = the 16-bit mask, w1 = FI_SITE_A / _B.
//
// Operand faults run in a second instantiation (VAR_OPERAND) of the same kernel: the staged
// tile is shared and stays clean; at the one MFMA step that consumes the faulted word, the
// waves whose fragment registers hold it XOR the word in those registers just before THAT
// trial's MFMAs and XOR it back after them - the trial sees the MFMA inputs a trial of its own
// would have staged, the other trials see clean ones.  The extra code sits in copies of the
// k-tile that only waves with an event in the current item execute; two instantiations keep
// it out of the plain one altogether.
//
// Work item = (output tile, group of R trials).  The register budget (R*TM*TN*16 accumulator
// VGPRs per lane) admits one or two workgroups per CU, so little would hide a workgroup's
// start-up (descriptor fetch, first operand tile) or wind-down behind another's MFMAs.  Instead
// the grid is one or two workgroups per CU and each walks its items with the k-loop running
// straight through: during the last k-tile of an item the first k-tile of the next item is
// already loading into the free LDS stage, and the next item's descriptors were fetched earlier.
//
// The per-element arithmetic is that of gemm_fi_kernel: the same sequence of
// v_mfma_f32_32x32x16 steps in ascending k, hence bit-identical fault-free results.
#pragma once

#include "gemm_fi.hpp"

namespace fi {

constexpr int kMultiDescWords = 6;   // trial, row, col, event, w0, w1
// cache policy of the output stores: non-temporal (written once, read by another kernel later),
// so that they do not displace the operand panels in L2
constexpr int kStreamStore = 2;

// VAR: which part of the work this instantiation takes.
enum { VAR_PLAIN = 0, VAR_OPERAND = 1, VAR_PROPAGATE = 2 };

template <int DT, int R, int BM, int BN, int WM, int WN, int VAR>
__global__ void __launch_bounds__(WM* WN * 64, 2) gemm_fi_multi_kernel(const GemmArgs p) {
  constexpr bool OPS = VAR == VAR_OPERAND;
  // PROP: the next layer of a two-layer workload.  Work item = (output tile, trial); trial t
  // stages ITS OWN A operand (A + t * a_trial_stride) and the shared B, no fault is injected,
  // and every output element is compared with the fault-free result.
  constexpr bool PROP = VAR == VAR_PROPAGATE;
  static_assert(!PROP || R == 1, "trials of the next layer share no A operand: one trial per item");
  constexpr int BK = 64;
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * 128;
  constexpr int A_G = BM / 8 / NW, B_G = BN / 8 / NW;      // 8-row groups staged per wave
  constexpr int NO_HOOK = 0x7fffffff;
  // Fetch the epilogue's threshold inputs when an item starts (hides their latency) where the
  // register budget has room for them; else when the epilogue starts.
  constexpr bool EARLY_T = TM * TN == 1;
  // The threshold inputs of the whole wave tile sit in registers during the epilogue (else they
  // are loaded tile by tile: 8 tiles' worth would spill).
  constexpr bool HAVE_T = TM * TN <= 4;
  // Large wave tiles leave few registers: the next item is located (its staging offsets
  // computed, its descriptors requested) just before the current item's last k-tile instead of
  // a whole item ahead, and golden values are fetched in the epilogue instead of up front.
  constexpr bool LATE_NEXT = TM * TN >= 4;
  constexpr bool PRE_GOLDEN = R >= 4;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is a multiple of the 32x32 MFMA");
  static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "row groups divide among the waves");
  static_assert(R * TM * TN * 16 <= 128, "accumulators fit half the register file");
  static_assert(2 * STAGE <= 160 * 1024, "two stages fit the 160 KB LDS");
  static_assert(R * kMultiDescWords <= 64, "a group's descriptors fit one word per lane");

  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lhi = lane >> 5;

  // ---- work list: n_tiles x ceil(n_fast / R) items, walked with the grid as stride
  // OPS: the second part of the batch; its descriptors follow the first part's, padded to 8.
  const int n_fast = PROP ? p.n_trials : (int)p.part_counts[OPS ? 1 : 0];
  const uint32_t* const desc =
      PROP ? nullptr : p.desc + (OPS ? (size_t)((p.part_counts[0] + 7u) & ~7u) * kMultiDescWords : 0);
  const int n_groups = (n_fast + R - 1) / R;
  const uint32_t n_work = (uint32_t)(p.tiles_m * p.tiles_n) * (uint32_t)n_groups;
  uint32_t w_cur = blockIdx.x;
  if (w_cur >= n_work) return;                            // uniform, before any barrier
  if (p.clocks && blockIdx.x == 0 && tid == 0) {
    p.clocks[4 * VAR + 0] = __builtin_readcyclecounter();
    p.clocks[4 * VAR + 1] = __builtin_amdgcn_s_memrealtime();
  }

  // ---- staging: global -> LDS directly, as in gemm_fi_kernel
  const int lrow = lane >> 3, lslot = lane & 7;
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void glb_void;

  struct Item {
    int m0, n0, grp;
    uint32_t a_goff[A_G], b_goff[B_G];
    size_t a_base;                                       // PROP: element offset of the trial's A operand
  };
  Item cur, nxt;                                         // the current item and the one after it
  int stage = 0;                                         // LDS stage of the current k-tile
  auto locate = [&](uint32_t w, Item& it) {
    int tile;
    work_of_index(w, n_work, p.tiles_m * p.tiles_n, n_groups, p.group, tile, it.grp);
    it.m0 = (tile / p.tiles_n) * BM;
    it.n0 = (tile % p.tiles_n) * BN;
    it.a_base = PROP ? (size_t)it.grp * (size_t)p.a_trial_stride : 0;
#pragma unroll
    for (int c = 0; c < A_G; ++c) {
      const int row = (wave * A_G + c) * 8 + lrow;
      it.a_goff[c] = (uint32_t)min(it.m0 + row, p.M - 1) * p.lda + (uint32_t)((lslot ^ lds_swizzle(row)) * 8);
    }
#pragma unroll
    for (int c = 0; c < B_G; ++c) {
      const int row = (wave * B_G + c) * 8 + lrow;
      it.b_goff[c] = (uint32_t)min(it.n0 + row, p.N - 1) * p.ldb + (uint32_t)((lslot ^ lds_swizzle(row)) * 8);
    }
  };
  // Staging goes through buffer loads with the LDS as destination: the operand's base sits in a
  // scalar resource descriptor, the lane's part of the address is one 32-bit byte offset that
  // never changes within an item, and the k offset is a scalar - a load needs no vector
  // arithmetic and ships 4 bytes of address per lane instead of 8.  num_records is the operand's
  // extent, so a load beyond it (there is none) would return zeros instead of faulting.
  const uint32_t a_bytes = (uint32_t)(((size_t)(p.M - 1) * p.lda + (size_t)p.K) * 2);
  const uint32_t b_bytes = (uint32_t)(((size_t)(p.N - 1) * p.ldb + (size_t)p.K) * 2);
  const __amdgpu_buffer_rsrc_t rsrc_b =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.B), 0, (int)b_bytes, 0x00020000);
  auto rsrc_a_of = [&](const Item& it) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(PROP ? p.A + it.a_base : p.A), 0, (int)a_bytes,
                                             0x00020000);
  };
  auto issue_tile = [&](const Item& it, int kt, int stage) {
    const int kb0 = kt * BK * 2;                           // bytes
    const __amdgpu_buffer_rsrc_t rsrc_a = rsrc_a_of(it);
    uint8_t* sA = smem + stage * STAGE + wave * (A_G * 1024);
    uint8_t* sB = smem + stage * STAGE + BM * 128 + wave * (B_G * 1024);
#pragma unroll
    for (int c = 0; c < A_G; ++c)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_void*)(sA + c * 1024), 16, (int)(it.a_goff[c] * 2u), kb0, 0, 0);
#pragma unroll
    for (int c = 0; c < B_G; ++c)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_void*)(sB + c * 1024), 16, (int)(it.b_goff[c] * 2u), kb0, 0, 0);
  };
  // One of the NLOADS loads of issue_tile (k < A_G: the k-th A row group, else B).
  auto issue_one = [&](const Item& it, int kt, int stage, auto kk) __attribute__((always_inline)) {
    constexpr int k = decltype(kk)::value;
    const int kb0 = kt * BK * 2;
    if constexpr (k < A_G) {
      uint8_t* sA = smem + stage * STAGE + wave * (A_G * 1024);
      const __amdgpu_buffer_rsrc_t rsrc_a = rsrc_a_of(it);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_void*)(sA + k * 1024), 16, (int)(it.a_goff[k] * 2u), kb0, 0, 0);
    } else {
      constexpr int c = k - A_G;
      uint8_t* sB = smem + stage * STAGE + BM * 128 + wave * (B_G * 1024);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_void*)(sB + c * 1024), 16, (int)(it.b_goff[c] * 2u), kb0, 0, 0);
    }
  };
  // The same with the choice made at run time: the next k-tile of the current item, or (last)
  // the first k-tile of the next item.  Offsets are selected value by value, never through a
  // pointer to one of the two items (which would move them to scratch memory).
  auto issue_tile_of = [&](bool last, int kt, int stage) {
    const int kb0 = last ? 0 : (kt + 1) * BK * 2;
    const __amdgpu_buffer_rsrc_t rsrc_a = rsrc_a_of(cur);  // items with events exist in campaigns only: one A
    uint8_t* sA = smem + stage * STAGE + wave * (A_G * 1024);
    uint8_t* sB = smem + stage * STAGE + BM * 128 + wave * (B_G * 1024);
#pragma unroll
    for (int c = 0; c < A_G; ++c) {
      const uint32_t off = last ? nxt.a_goff[c] : cur.a_goff[c];
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_void*)(sA + c * 1024), 16, (int)(off * 2u), kb0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < B_G; ++c) {
      const uint32_t off = last ? nxt.b_goff[c] : cur.b_goff[c];
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_void*)(sB + c * 1024), 16, (int)(off * 2u), kb0, 0, 0);
    }
  };
  // A group's R descriptors, one word per lane; fields are picked out with v_readlane.
  auto load_desc = [&](int grp) -> uint32_t {
    if constexpr (PROP) return lane == 0 ? (uint32_t)grp : lane == 3 ? 0xFFFFFFFFu : 0u;   // {trial, -, -, no event}
    else {
      // a buffer load: scalar base and group offset, the lane's word as a 32-bit offset (a 64-bit
      // per-lane pointer kept across the k-loop cost two registers the 128 x 64 shape does not have)
      const __amdgpu_buffer_rsrc_t rs =
          __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(desc), 0, -1, 0x00020000);
      const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(
          rs, (lane < R * kMultiDescWords ? lane : 0) * 4, grp * (R * kMultiDescWords * 4), 0);
      return lane < R * kMultiDescWords ? w : 0u;
    }
  };

  // ---- fragments and accumulators
  const int sw = lds_swizzle(l32);
  const int a_rd = (wm * WTM + l32) * 128;
  const int b_rd = BM * 128 + (wn * WTN + l32) * 128;

  f32x16 acc[R][TM][TN];

  struct Frags { u32x4 a[TM]; u32x4 b[TN]; };
  auto read_frags = [&](Frags& f, const uint8_t* s, int kk) {
    const int slot = ((2 * kk + lhi) ^ sw) << 4;
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = *reinterpret_cast<const u32x4*>(s + a_rd + i * 4096 + slot);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = *reinterpret_cast<const u32x4*>(s + b_rd + j * 4096 + slot);
  };
  // One fragment set, R accumulator sets.  FIRST: the first MFMA step of an item, whose
  // accumulators start from zero - the matrix instruction takes the constant 0 as its addend, so
  // an item never spends vector instructions on clearing 128 accumulator registers.  `mid` (a
  // fragment read for the next step) is issued after the first few MFMAs: the read lands under
  // the rest of the burst instead of being waited for in front of it.
  // `load(k)` issues the k-th staging load of the next k-tile (k a compile-time index that
  // runs over the steps of a k-tile): the loads go out one by one between the MFMAs of the
  // bursts, LOAD_STRIDE MFMAs apart, instead of in one block in front of a burst.
  constexpr int NMMA = R * TM * TN;                      // MFMAs per step and wave
  constexpr int NLOADS = A_G + B_G;                      // staging loads per k-tile and wave
  constexpr int LOAD_STRIDE = NLOADS <= 3 * ((NMMA - 2) / 2 + 1) ? 2 : 1;
  constexpr int LOADS_PER_STEP = (NMMA - 2) / LOAD_STRIDE + 1;   // after MFMA 1, 1 + stride, ...
  static_assert(NMMA >= 2 && NLOADS <= 3 * LOADS_PER_STEP, "the loads of a k-tile fit its first three bursts");
  auto mma_step_mid = [&](const Frags& f, auto first, auto step_in_tile, auto&& mid, auto&& load) __attribute__((always_inline)) {
    constexpr bool FIRST = decltype(first)::value;
    constexpr int SIT = decltype(step_in_tile)::value;   // 0 .. 3; loads go with 0 .. 2
    [[maybe_unused]] Frags q = f;
    static_for<NMMA>([&](auto t) {
      constexpr int r = t / (TM * TN), i = (t / TN) % TM, j = t % TN;
      if constexpr (t == (NMMA >= 8 ? 2 : 1)) {
        __builtin_amdgcn_sched_barrier(0);
        mid();
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (SIT < 3 && t >= 1 && (t - 1) % LOAD_STRIDE == 0) {
        constexpr int k = SIT * LOADS_PER_STEP + (t - 1) / LOAD_STRIDE;
        if constexpr (k < NLOADS) {
          __builtin_amdgcn_sched_barrier(0);
          load(std::integral_constant<int, k>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if constexpr (FIRST) {
        // The R trials start from the same zero with the same fragments, so their first MFMAs
        // are equal expressions and a compiler may compute one and copy it R - 1 times.  Every
        // trial executes its own MFMAs: between trials one fragment register passes through an
        // empty asm statement (no instruction, no extra register), after which the compiler can
        // no longer take the next trial's inputs to be the previous trial's.
        if constexpr (r > 0 && i == 0 && j == 0) asm volatile("" : "+v"(q.a[0]));
        acc[r][i][j] = mfma_32x32x16<DT>(q.a[i], q.b[j],
            f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f});
      } else {
        acc[r][i][j] = mfma_32x32x16<DT>(f.a[i], f.b[j], acc[r][i][j]);
      }
    });
  };

  // ---- state of the current item
  uint32_t desc_cur, desc_nxt = 0;                       // lane-distributed descriptor words
  int n_act = 0;                                         // trials in this group
  // hook_step[r]: the MFMA step of trial r's event if this wave takes part in it (it owns the
  // accumulator element, or its fragments hold the faulted operand word), else -1.
  int trial[R], hook_step[R];
  bool has_events = false;                               // some hook_step[r] >= 0
  auto desc_field = [&](int r, int field) -> uint32_t {
    return (uint32_t)__builtin_amdgcn_readlane((int)desc_cur, r * kMultiDescWords + field);
  };
  // Fault-free value and magnitude sum of the element(s) of the faulted output ROW this lane
  // holds, per trial with an event here: fetched when the item starts (they come from HBM, and
  // an epilogue that fetched them trial after trial would expose one memory round trip each).
  float cs_pre[R][TN], sa_pre[R][TN];
  auto prefetch_row_golden = [&](auto rr) __attribute__((always_inline)) {
    constexpr int r = rr;
    if constexpr (!PRE_GOLDEN) return;
    const size_t row_off = (size_t)desc_field(r, 1) * (size_t)p.N;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const size_t idx = row_off + (size_t)min(cur.n0 + wn * WTN + l32 + 32 * j, p.N - 1);
      cs_pre[r][j] = p.c_star[idx];
      sa_pre[r][j] = p.s_abs[idx];
    }
  };

  auto decode = [&]() {
    n_act = min(R, n_fast - cur.grp * R);
    has_events = false;
    if constexpr (!PROP) {
      // Nearly every item holds no event of this wave.  One lane-parallel test over the R
      // descriptors settles that (a few shuffles and compares, one ballot) instead of R
      // scalar decodes of some 45 instructions each.  Lane l looks at the descriptor of trial
      // l / 6, whose words sit in lanes 6 * (l / 6) .. + 5 of desc_cur (recomputed per item: two
      // registers held across the k-loop would not fit the 128 x 64 shape).
      const int d_trial = lane / kMultiDescWords, d_base = d_trial * kMultiDescWords;
      const int row = __shfl((int)desc_cur, d_base + 1, 64), col = __shfl((int)desc_cur, d_base + 2, 64);
      const int ev = __shfl((int)desc_cur, d_base + 3, 64);
      const int li = row - cur.m0, lj = col - cur.n0;
      bool hit;
      if (OPS && ((ev >> 29) & 1)) {
        const bool isA = __shfl((int)desc_cur, d_base + 5, 64) == FI_SITE_A;
        const int wl = isA ? li - wm * WTM : lj - wn * WTN;
        hit = wl >= 0 && wl < (isA ? WTM : WTN);          // inside the wave's rows / columns of this tile
      } else {
        const int wi = li - wm * WTM, wj = lj - wn * WTN;
        hit = wi >= 0 && wi < WTM && wj >= 0 && wj < WTN;
      }
      if (__ballot(hit && ev >= 0 && d_trial < n_act && lane < R * kMultiDescWords) == 0) {
        static_for<R>([&](auto rr) {
          trial[rr] = (int)desc_field(rr, 0);
          hook_step[rr] = -1;
        });
        return;
      }
    }
    static_for<R>([&](auto rr) {
      constexpr int r = rr;
      trial[r] = (int)desc_field(r, 0);
      hook_step[r] = -1;
      const int ev = PROP ? -1 : (int)desc_field(r, 3);
      const int hs = ev & 0xFFFF;
      if (r < n_act && ev >= 0) {
        const int li = (int)desc_field(r, 1) - cur.m0, lj = (int)desc_field(r, 2) - cur.n0;
        if (OPS && ((ev >> 29) & 1)) {
          // A: row i = desc row, every tile of that tile row differs; B: column j = desc col.
          const bool isA = desc_field(r, 5) == FI_SITE_A;
          const int l = isA ? li : lj;
          if (l >= 0 && l < (isA ? BM : BN)) {
            const int wl = isA ? l - wm * WTM : l - wn * WTN;
            if (wl >= 0 && wl < (isA ? WTM : WTN)) {
              hook_step[r] = hs;
              has_events = true;
              if (isA) prefetch_row_golden(rr);
            }
          }
        } else if (li >= 0 && li < BM && lj >= 0 && lj < BN) {
          const int wi = li - wm * WTM, wj = lj - wn * WTN;
          if (wi >= 0 && wi < WTM && wj >= 0 && wj < WTN) {
            hook_step[r] = hs;
            has_events = true;
            prefetch_row_golden(rr);
          }
        }
      }
    });
  };

  // Accumulator flip of trial r (this wave owns its site); once per trial in the whole grid.
  auto accumulator_fault = [&](auto rr) {
    constexpr int r = rr;
    const int wi = (int)desc_field(r, 1) - cur.m0 - wm * WTM, wj = (int)desc_field(r, 2) - cur.n0 - wn * WTN;
    const bool product = ((desc_field(r, 3) >> 30) & 1u) != 0;      // else an XOR of the word
    const uint32_t w0 = desc_field(r, 4), w1 = desc_field(r, 5);
    const float re = __uint_as_float(w0), re_err = __uint_as_float(w1);
    const int ri = wi & 31, rj = wj & 31;
    const int sel_t = (wi >> 5) * TN + (wj >> 5);
    const int sel_v = 4 * (ri >> 3) + (ri & 3);
    const int sel_lane = rj + 32 * ((ri >> 2) & 1);
    uint32_t before = 0, after = 0;
    static_for<TM * TN>([&](auto tt) {
      constexpr int i = tt / TN, j = tt % TN;
      if (tt == sel_t) {
        f32x16 t = acc[r][i][j];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const bool here = v == sel_v;
          const uint32_t w = __float_as_uint(t[v]);
          const uint32_t nw = product ? __float_as_uint(write_back(t[v], re, re_err)) : (w ^ w0);
          before = here ? w : before;
          after = here ? nw : after;
          t[v] = __uint_as_float((here && lane == sel_lane) ? nw : w);
        }
        acc[r][i][j] = t;
      }
    });
    if (lane == sel_lane) {
      p.results[trial[r]].site_word_before = before;
      p.results[trial[r]].site_word_after = after;
    }
    // Leave nothing of this rare path in flight: the compiler places its waits statically, and
    // memory traffic pending here would make every iteration of the main loop wait for it.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  };
  // Bit r: trial r's event falls on MFMA step g (and this wave takes part in it).
  auto hit_mask = [&](int g) __attribute__((always_inline)) -> uint32_t {
    uint32_t m = 0;
    static_for<R>([&](auto rr) { m |= hook_step[rr] == g ? 1u << rr : 0u; });
    return m;
  };
  // Accumulator faults due after an MFMA step (at most one wave per trial owns one).
  auto hooks = [&](uint32_t m) __attribute__((always_inline)) {
    static_for<R>([&](auto rr) {
      if ((m >> rr) & 1u) accumulator_fault(rr);
    });
  };
  // Operand fault of trial r (OPS): XOR the faulted 16-bit word in the fragment registers the R
  // trials share (lane l holds row / column l % 32, k = 8*(l/32) .. +7 of the step, two k per
  // register, even k in the low half).  Called right before trial r's MFMAs of the step that
  // consumes the word and again right after them, which restores the clean fragment: trial r
  // gets exactly the MFMA inputs a run of its own would have staged, the other trials the clean
  // ones, and the MFMAs themselves sit outside every branch.
  auto toggle_operand = [&](Frags& f, auto rr) __attribute__((always_inline)) {
    constexpr int r = rr;
    const bool isA = desc_field(r, 5) == FI_SITE_A;
    const int k = (int)(isA ? desc_field(r, 2) : desc_field(r, 1));
    const int wl = isA ? (int)desc_field(r, 1) - cur.m0 - wm * WTM : (int)desc_field(r, 2) - cur.n0 - wn * WTN;
    const int sel_lane = (wl & 31) + 32 * ((k >> 3) & 1);
    const int sel_w = (k & 7) >> 1;
    const uint32_t x = (lane == sel_lane) ? (desc_field(r, 4) & 0xFFFFu) << (16 * (k & 1)) : 0u;
    // Every register is named statically (a register picked through a run-time index or a
    // pointer to "the A or the B fragment" would move the fragments to scratch memory).
    const uint32_t xa = isA ? x : 0u, xb = isA ? 0u : x;
    static_for<TM * 4>([&](auto t) {
      constexpr int ii = t / 4, w = t % 4;
      f.a[ii][w] ^= (ii == (wl >> 5) && w == sel_w) ? xa : 0u;
    });
    static_for<TN * 4>([&](auto t) {
      constexpr int jj = t / 4, w = t % 4;
      f.b[jj][w] ^= (jj == (wl >> 5) && w == sel_w) ? xb : 0u;
    });
  };
  // One MFMA step in a k-tile that holds an operand fault of this wave (OPS): bit r of m says
  // that the step consumes trial r's faulted word.  The MFMAs stay in straight-line code; the
  // toggles sit in cold blocks behind one scalar bit test each.
  auto mma_step_ops = [&](Frags& f, uint32_t m, auto&& mid) __attribute__((always_inline)) {
    constexpr int R_MID = TM * TN >= 2 ? 0 : 1;          // `mid` goes behind the first two MFMAs
    static_for<R>([&](auto rr) {
      constexpr int r = rr;
      if (__builtin_expect((m >> r) & 1u, 0)) toggle_operand(f, rr);
      // A convergent no-op next to the MFMAs: the block holding them is then never duplicated
      // into the two arms of the (repeated) test, which would put MFMAs behind a branch.
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_sched_barrier(0);
      static_for<TM * TN>([&](auto t) {
        constexpr int i = t / TN, j = t % TN;
        acc[r][i][j] = mfma_32x32x16<DT>(f.a[i], f.b[j], acc[r][i][j]);
      });
      __builtin_amdgcn_sched_barrier(0);
      if (__builtin_expect((m >> r) & 1u, 0)) toggle_operand(f, rr);
      if constexpr (r == (R_MID < R ? R_MID : R - 1)) {
        __builtin_amdgcn_sched_barrier(0);
        mid();
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  };

  // ---- epilogue of the current item, trial by trial: detector, corrector, optional store;
  // deviation counters where the trial's fault can reach.  Thresholds are the same for every
  // trial (same rows and columns), so they are formed once; elements outside the problem get
  // T = +Inf and, in ragged tiles, a zeroed accumulator (clamped staging rows made them copies
  // of the last row).  kra4 / cbj: the rows' and columns' threshold factors this lane needs.
  f32x4 kra4[TM][4];
  float cbj[TN];
  auto fetch_threshold_inputs = [&]() {                 // arrays are padded: no guards
    const int row_base = cur.m0 + wm * WTM + 4 * lhi;
    const int col_base = cur.n0 + wn * WTN + l32;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        kra4[i][q] = *reinterpret_cast<const f32x4*>(p.kra + row_base + 32 * i + 8 * q);
#pragma unroll
    for (int j = 0; j < TN; ++j) cbj[j] = p.cb[min(col_base + 32 * j, p.N - 1)];
  };
  auto epilogue = [&]() {
    // Larger wave tiles have no registers for the threshold inputs while the k-loop runs: they
    // are fetched here, all at once (one memory round trip for the whole item, not one per tile).
    if constexpr (HAVE_T && !EARLY_T) fetch_threshold_inputs();
    const int m0 = cur.m0, n0 = cur.n0;
    const int row_base = m0 + wm * WTM + 4 * lhi;       // + 32*i + 8*q + e
    const int col_base = n0 + wn * WTN + l32;           // + 32*j
    const bool ragged = m0 + BM > p.M || n0 + BN > p.N;
    auto thresholds = [&](auto tt) {
      constexpr int i = tt / TN, j = tt % TN;
      const int col = col_base + 32 * j;
      f32x16 T;
      const float cb_here = HAVE_T ? cbj[j] : p.cb[min(col, p.N - 1)];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 kra_here =
            HAVE_T ? kra4[i][q] : *reinterpret_cast<const f32x4*>(p.kra + row_base + 32 * i + 8 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int row = row_base + 32 * i + 8 * q + e;
          const float t = p.bound_global ? p.t_global : __fmul_rn(__fmul_rn(kra_here[e], cb_here), p.gamma);
          T[4 * q + e] = (row < p.M && col < p.N) ? t : __builtin_inff();
        }
      }
      return T;
    };
    if (ragged) {
      static_for<R * TM * TN>([&](auto t) {
        constexpr int r = t / (TM * TN), i = (t / TN) % TM, j = t % TN;
        f32x16 a = acc[r][i][j];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
          a[v] = (row < p.M && col_base + 32 * j < p.N) ? a[v] : 0.0f;
        }
        acc[r][i][j] = a;
      });
    }
    // Detector (and corrector, when outputs are wanted) on every element of every trial.  Without
    // outputs the common case costs one compare and one scalar OR per element: lane masks of
    // the flags are merged, and only a trial-tile with any flag set is counted exactly.
    // PROP: the fault-free words of this wave's 32 x 32 tiles travel kGoldAhead tiles ahead of
    // their use; the first ones are requested here, before the detector pass.
    constexpr int kGoldAhead = 2;
    [[maybe_unused]] f32x16 cs_buf[PROP ? kGoldAhead + 1 : 1];
    // They come through buffer loads: the lane's part of the address is one 32-bit offset for the
    // whole item, the tile's and row's part is scalar - no vector address arithmetic, no address
    // registers per load.  The allocation is padded to whole tiles, so rows and columns beyond a
    // ragged problem read allocated memory (such elements are never compared).
    const __amdgpu_buffer_rsrc_t rsrc_gold =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.c_star), 0, (int)p.c_star_bytes, 0x00020000);
    const int gold_lane = (4 * lhi * p.N + l32) * 4;                  // bytes
    auto load_golden = [&](auto tt, f32x16& dst) __attribute__((always_inline)) {
      constexpr int i = tt / TN, j = tt % TN;
      const uint32_t tile_off = __builtin_amdgcn_readfirstlane(
          (int)((((uint32_t)(m0 + wm * WTM + 32 * i) * (uint32_t)p.N) + (uint32_t)(n0 + wn * WTN + 32 * j)) * 4u));
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const uint32_t row_off = (uint32_t)(8 * (v >> 2) + (v & 3)) * (uint32_t)p.N * 4u;
        dst[v] = __uint_as_float(
            __builtin_amdgcn_raw_buffer_load_b32(rsrc_gold, gold_lane, (int)(tile_off + row_off), 0));
      }
    };
    if constexpr (PROP) {
      static_for<kGoldAhead>([&](auto tt) {
        if constexpr (tt < TM * TN) load_golden(tt, cs_buf[tt]);
      });
    }
    uint32_t n_flag[R];
    static_for<R>([&](auto rr) { n_flag[rr] = 0; });
    // output stores of 16 bytes per lane need 16-byte aligned rows (and two KB of LDS per wave)
    static_assert(A_G >= 2, "a wave's staging slice holds a 2 KB transposition buffer");
    const bool wide_c = p.c_out && (p.N & 3) == 0 && (reinterpret_cast<uintptr_t>(p.c_out) & 15u) == 0;
    const bool wide_h = p.h_out && (p.N & 7) == 0 && (reinterpret_cast<uintptr_t>(p.h_out) & 15u) == 0;
    uint8_t* const scr = smem + (stage ^ 1) * STAGE + wave * (A_G * 1024);
    // The lane's parts of the wide stores' addresses are formed here, per item: left to the
    // compiler they are hoisted to the top of the kernel and cost the k-loop registers it does
    // not have (the empty asm statement pins them below this point).
    int ln = lane;
    asm volatile("" : "+v"(ln));
    auto detect = [&](auto with_out) __attribute__((always_inline)) {
      constexpr bool OUT = decltype(with_out)::value;
      static_for<TM * TN>([&](auto tt) {
        constexpr int i = tt / TN, j = tt % TN;
        const f32x16 T = thresholds(tt);
        const int col = col_base + 32 * j;
        static_for<R>([&](auto rr) {
          constexpr int r = rr;
          if (r < n_act) {
            const f32x16 t = acc[r][i][j];
            uint64_t any = 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) any |= __ballot(!(fabsf(t[v]) <= T[v]));
            if (any != 0) {
#pragma unroll
              for (int v = 0; v < 16; ++v)
                n_flag[r] += (uint32_t)__builtin_popcountll(__ballot(!(fabsf(t[v]) <= T[v])));
            }
            if constexpr (OUT) {
              const size_t out0 = (size_t)trial[r] * (size_t)p.M * (size_t)p.N;
              // Nearly every trial-tile: nothing flagged, no ragged edge.  The values go out as
              // they are, through buffer stores whose address is a per-item lane offset plus a
              // scalar (trial, tile, row) offset: no vector arithmetic, no branch per element.
              if (any == 0 && !ragged && p.c_star_bytes != 0) {
                const uint32_t tile_off = (uint32_t)(m0 + wm * WTM + 32 * i) * (uint32_t)p.N +
                                          (uint32_t)(n0 + wn * WTN + 32 * j);           // elements
                const int lane_off = 4 * lhi * p.N + l32;
                const uint32_t mn = (uint32_t)p.M * (uint32_t)p.N;
                // Where rows are 16-byte aligned the 32 x 32 tile goes through LDS first - the
                // accumulator layout gives a lane one column of 16 rows, a store wants it a piece
                // of one row - and leaves as 16 bytes per lane: 2 (16-bit) or 4 (FP32) store
                // instructions per tile instead of 16.  The scratch is this wave's own staging
                // slice of the LDS stage the item has just finished with (nobody reads it any
                // more, and only this wave will write it again: the next item's second k-tile).
                if (p.c_out) {
                  const __amdgpu_buffer_rsrc_t rs =
                      __builtin_amdgcn_make_buffer_rsrc(p.c_out + out0, 0, (int)(mn * 4u), 0x00020000);
                  if (wide_c) {
                    const int voff = ((ln >> 3) * p.N + (ln & 7) * 4) * 4;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
                      for (int v = 8 * half; v < 8 * half + 8; ++v)      // rows 16 * half .. + 15
                        *reinterpret_cast<float*>(scr + (8 * ((v >> 2) & 1) + 4 * (ln >> 5) + (v & 3)) * 128 + (ln & 31) * 4) = t[v];
                      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
                      for (int ps = 0; ps < 2; ++ps) {
                        const u32x4 q = *reinterpret_cast<const u32x4*>(scr + (8 * ps + (ln >> 3)) * 128 + (ln & 7) * 16);
                        __builtin_amdgcn_raw_buffer_store_b128(
                            q, rs, voff, (int)((tile_off + (uint32_t)(16 * half + 8 * ps) * (uint32_t)p.N) * 4u), kStreamStore);
                      }
                    }
                  } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                      __builtin_amdgcn_raw_buffer_store_b32(
                          __float_as_uint(t[v]), rs, lane_off * 4,
                          (int)((tile_off + (uint32_t)(8 * (v >> 2) + (v & 3)) * (uint32_t)p.N) * 4u), kStreamStore);
                  }
                }
                if (p.h_out) {
                  const __amdgpu_buffer_rsrc_t rs =
                      __builtin_amdgcn_make_buffer_rsrc(p.h_out + out0, 0, (int)(mn * 2u), 0x00020000);
                  if (wide_h) {
                    const int voff = ((ln >> 2) * p.N + (ln & 3) * 8) * 2;
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                      const float cc = t[v];
                      *reinterpret_cast<uint16_t*>(scr + (8 * (v >> 2) + 4 * (ln >> 5) + (v & 3)) * 64 + (ln & 31) * 2) =
                          (uint16_t)relu_round16<DT>(cc);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
                    for (int ps = 0; ps < 2; ++ps) {
                      const u32x4 q = *reinterpret_cast<const u32x4*>(scr + (16 * ps + (ln >> 2)) * 64 + (ln & 3) * 16);
                      __builtin_amdgcn_raw_buffer_store_b128(
                          q, rs, voff, (int)((tile_off + (uint32_t)(16 * ps) * (uint32_t)p.N) * 2u), kStreamStore);
                    }
                  } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                      const float cc = t[v];
                      __builtin_amdgcn_raw_buffer_store_b16(
                          (unsigned short)round16<DT>((cc > 0.0f || cc != cc) ? cc : 0.0f), rs, lane_off * 2,
                          (int)((tile_off + (uint32_t)(8 * (v >> 2) + (v & 3)) * (uint32_t)p.N) * 2u), kStreamStore);
                    }
                  }
                }
              } else
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
                float cc = t[v];
                if (!(fabsf(cc) <= T[v])) {
                  if (p.policy == FI_CORRECT_ZERO) cc = 0.0f;
                  else if (p.policy == FI_CORRECT_RECOMPUTE) cc = p.c_star[(size_t)row * p.N + col];
                }
                if (row < p.M && col < p.N) {
                  const size_t at = out0 + (size_t)row * p.N + col;
                  if (p.c_out) p.c_out[at] = cc;
                  // the hand-over between two layers fused into this epilogue: relu keeps a NaN
                  // and maps negatives and -0 to +0, then the integer round-to-format
                  if (p.h_out) p.h_out[at] = (uint16_t)round16<DT>((cc > 0.0f || cc != cc) ? cc : 0.0f);
                }
              }
            }
          }
        });
      });
    };
    if (p.c_out || p.h_out) detect(std::true_type{}); else detect(std::false_type{});
    static_for<R>([&](auto rr) {
      constexpr int r = rr;
      if (r < n_act && n_flag[r] != 0 && lane == 0) atomicAdd(&p.results[trial[r]].n_flagged, n_flag[r]);
    });
    if constexpr (PROP) {
      // Every element of the trial's output against the fault-free result.  Two phases per
      // 32 x 32 tile: the fault-free words (requested tiles ahead) are compared bit for bit
      // (most tiles of most trials are untouched by what the previous layer's fault changed: no
      // counter can move there); only a tile with a differing (or NaN) element runs the full
      // accounting, four rows at a time so that it needs few registers.
      uint32_t n_bit = 0, n_pre = 0, n_post = 0, n_bT = 0, n_btau = 0;
      float mx_pre = 0.0f, mx_post = 0.0f;
      static_for<TM * TN>([&](auto tt) {
        constexpr int i = tt / TN, j = tt % TN, cb = tt % (kGoldAhead + 1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (tt + kGoldAhead < TM * TN)
          load_golden(std::integral_constant<int, tt + kGoldAhead>{}, cs_buf[(tt + kGoldAhead) % (kGoldAhead + 1)]);
        const f32x16 t = acc[0][i][j];
        const f32x16 cs = cs_buf[cb];
        const int col = col_base + 32 * j;
        uint32_t differs = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
          const bool act = !ragged || (row < p.M && col < p.N);
          differs |= (act && (__float_as_uint(t[v]) != __float_as_uint(cs[v]) || t[v] != t[v])) ? 1u : 0u;
        }
        if (__ballot(differs != 0) != 0) {
          static_for<4>([&](auto qq) {
            constexpr int q = qq;
            __builtin_amdgcn_sched_barrier(0);
            const int row0 = row_base + 32 * i + 8 * q;
            const f32x4 kra_q = HAVE_T ? kra4[i][q] : *reinterpret_cast<const f32x4*>(p.kra + row0);
            const float cb_j = HAVE_T ? cbj[j] : p.cb[min(col, p.N - 1)];
            float sa[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              sa[e] = p.s_abs[(size_t)min(row0 + e, p.M - 1) * p.N + min(col, p.N - 1)];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              constexpr int dummy = 0; (void)dummy;
              const int v = 4 * q + e;
              const bool act = row0 + e < p.M && col < p.N;
              const float c = t[v], cse = cs[v];
              const float Tv = !act ? __builtin_inff()
                                    : p.bound_global ? p.t_global : __fmul_rn(__fmul_rn(kra_q[e], cb_j), p.gamma);
              const float tau = sa[e] * 0.000244140625f;        // 2^-12, exact scaling
              const bool flag = !(fabsf(c) <= Tv);
              float cc = c;
              if (flag && p.policy == FI_CORRECT_ZERO) cc = 0.0f;
              if (flag && p.policy == FI_CORRECT_RECOMPUTE) cc = cse;
              const float dpre = finite_or_inf(fabsf(c - cse));
              const float dpost = finite_or_inf(fabsf(cc - cse));
              const bool changed = act && __float_as_uint(c) != __float_as_uint(cse);
              n_bit += changed ? 1u : 0u;
              n_pre += (act && !(dpre <= tau)) ? 1u : 0u;
              n_post += (act && !(dpost <= tau)) ? 1u : 0u;
              mx_pre = fmaxf(mx_pre, act ? dpre : 0.0f);
              mx_post = fmaxf(mx_post, act ? dpost : 0.0f);
              const float band = fmaxf(2.0f * tau, Tv * 0.015625f);
              const float mag = fabsf(c);
              n_bT += (changed && mag <= 3.4028234e38f && fabsf(mag - Tv) <= band) ? 1u : 0u;
              n_btau += (changed && tau > 0.0f && dpre >= 0.5f * tau && dpre <= 2.0f * tau) ? 1u : 0u;
            }
          });
        }
      });
      // most trial tiles equal the fault-free result bit for bit: one ballot, nothing to reduce
      if (__ballot((n_bit | n_pre | n_post) != 0) == 0) return;
      uint32_t mp = __float_as_uint(mx_pre), mq = __float_as_uint(mx_post);   // non-negative: ordered like words
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        n_bit += __shfl_xor(n_bit, o, 64); n_pre += __shfl_xor(n_pre, o, 64); n_post += __shfl_xor(n_post, o, 64);
        n_bT += __shfl_xor(n_bT, o, 64); n_btau += __shfl_xor(n_btau, o, 64);
        const uint32_t a = __shfl_xor(mp, o, 64), b = __shfl_xor(mq, o, 64);
        mp = a > mp ? a : mp; mq = b > mq ? b : mq;
      }
      if (lane == 0) {
        fi_trial_result* res = p.results + trial[0];
        if (n_bit) atomicAdd(&res->n_bitdiff, n_bit);
        if (n_pre) atomicAdd(&res->n_dev_pre, n_pre);
        if (n_post) atomicAdd(&res->n_dev_post, n_post);
        if (n_bT) atomicAdd(&res->n_border_T, n_bT);
        if (n_btau) atomicAdd(&res->n_border_tau, n_btau);
        if (mp) atomicMax(reinterpret_cast<uint32_t*>(&res->max_dev_pre), mp);
        if (mq) atomicMax(reinterpret_cast<uint32_t*>(&res->max_dev_post), mq);
      }
      return;
    }
    // Deviation counters of the trials whose fault can reach an element this wave holds (rare):
    // the wave owning the element, or the waves holding its output row (A) / column (B).
    // Counts are sums of lane masks (ballot + popcount: no cross-lane traffic); the two maxima
    // of all trials are reduced together at the end, so the shuffles' latencies overlap.
    uint32_t owned = 0;
    static_for<R>([&](auto rr) { owned |= hook_step[rr] >= 0 ? 1u << rr : 0u; });
    if (owned == 0) return;
    float mxp[R], mxq[R];                                   // per lane: largest deviation before / after correction
    static_for<R>([&](auto rr) { mxp[rr] = 0.0f; mxq[rr] = 0.0f; });
    // B-operand faults reach one output column.  Lane k < 32 takes row k of each 32-row tile of
    // this wave: its threshold factor, and per trial the fault-free value and the magnitude sum
    // of (row, faulted column) - requested for all trials before any is looked at, so that the
    // trials share one memory round trip.
    constexpr bool COL_GATHER = OPS && TM * TN <= 4;
    [[maybe_unused]] float col_kra[TM], col_cs[COL_GATHER ? R : 1][TM], col_sa[COL_GATHER ? R : 1][TM];
    if constexpr (COL_GATHER) {
      static_for<TM>([&](auto ii) { col_kra[ii] = p.kra[m0 + wm * WTM + 32 * ii + l32]; });   // padded array
      static_for<R>([&](auto rr) {
        constexpr int r = rr;
        if (((owned >> r) & 1u) && ((desc_field(r, 3) >> 29) & 1u) && desc_field(r, 5) == FI_SITE_B) {
          const size_t col = desc_field(r, 2);
          static_for<TM>([&](auto ii) {
            const size_t idx = (size_t)min(m0 + wm * WTM + 32 * ii + l32, p.M - 1) * (size_t)p.N + col;
            col_cs[r][ii] = p.c_star[idx];
            col_sa[r][ii] = p.s_abs[idx];
          });
        }
      });
    }
    static_for<R>([&](auto rr) {
      constexpr int r = rr;
      if ((owned >> r) & 1u) {
        fi_trial_result* res = p.results + trial[r];
        const int site_row = (int)desc_field(r, 1), site_col = (int)desc_field(r, 2);
        // what the fault can reach: the element, or (OPS) its output row (A) / column (B)
        const bool op = OPS && ((desc_field(r, 3) >> 29) & 1u);
        const bool need_row = !op || desc_field(r, 5) == FI_SITE_A;
        const bool need_col = !op || desc_field(r, 5) == FI_SITE_B;
        uint32_t n_bit = 0, n_pre = 0, n_post = 0, n_bT = 0, n_btau = 0;   // wave-uniform
        float mx_pre = 0.0f, mx_post = 0.0f;
        // `act`: this lane's element is one the fault can reach.  Called by all lanes together.
        auto account = [&](bool act, float c, float Tv, float cs, float sabs) __attribute__((always_inline)) {
          const float tau = sabs * 0.000244140625f;           // 2^-12, exact scaling
          const bool flag = !(fabsf(c) <= Tv);
          float cc = c;
          if (flag && p.policy == FI_CORRECT_ZERO) cc = 0.0f;
          if (flag && p.policy == FI_CORRECT_RECOMPUTE) cc = cs;
          const float dpre = finite_or_inf(fabsf(c - cs));
          const float dpost = finite_or_inf(fabsf(cc - cs));
          const bool changed = act && __float_as_uint(c) != __float_as_uint(cs);
          n_bit += (uint32_t)__builtin_popcountll(__ballot(changed));
          n_pre += (uint32_t)__builtin_popcountll(__ballot(act && !(dpre <= tau)));
          n_post += (uint32_t)__builtin_popcountll(__ballot(act && !(dpost <= tau)));
          mx_pre = fmaxf(mx_pre, act ? dpre : 0.0f);
          mx_post = fmaxf(mx_post, act ? dpost : 0.0f);
          const float band = fmaxf(2.0f * tau, Tv * 0.015625f);
          const float mag = fabsf(c);
          n_bT += (uint32_t)__builtin_popcountll(__ballot(changed && mag <= 3.4028234e38f && fabsf(mag - Tv) <= band));
          n_btau += (uint32_t)__builtin_popcountll(__ballot(changed && tau > 0.0f && dpre >= 0.5f * tau && dpre <= 2.0f * tau));
        };
        if (need_row) {
          // One row: it lives in one 32-row tile, one register index and one lane half
          // (accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4).
          const int wr = site_row - m0 - wm * WTM;            // 0 .. WTM-1: this wave holds the row
          const int ri = wr & 31;
          const int sel_v = 4 * (ri >> 3) + (ri & 3), sel_hi = (ri >> 2) & 1;
          static_for<TM * TN>([&](auto tt) {
            constexpr int i = tt / TN, j = tt % TN;
            if (i == (wr >> 5)) {
              const f32x16 T = thresholds(tt);
              const f32x16 t = acc[r][i][j];
              float c = t[0], Tv = T[0];
#pragma unroll
              for (int v = 1; v < 16; ++v) {
                c = (v == sel_v) ? t[v] : c;
                Tv = (v == sel_v) ? T[v] : Tv;
              }
              const int col = col_base + 32 * j;
              float cs = 0.0f, sabs = 0.0f;
              if constexpr (PRE_GOLDEN) {
                cs = cs_pre[r][j];
                sabs = sa_pre[r][j];
              } else {
                const size_t idx = (size_t)site_row * (size_t)p.N + (size_t)min(col, p.N - 1);
                cs = p.c_star[idx];
                sabs = p.s_abs[idx];
              }
              account(lhi == sel_hi && (!need_col || col == site_col) && col < p.N, c, Tv, cs, sabs);
            }
          });
        } else if constexpr (COL_GATHER) {
          // One column: it lives in one 32-column tile and one lane of each half-wave, spread
          // over the 16 accumulator registers (rows).  Its 32 values per tile are gathered into
          // lanes 0 .. 31 (row k to lane k) and accounted for in one pass.
          const int wc = site_col - n0 - wn * WTN;            // 0 .. WTN-1: this wave holds the column
          const int sel = wc & 31;
          const float cb_c = p.cb[site_col];
          static_for<TM * TN>([&](auto tt) {
            constexpr int i = tt / TN, j = tt % TN;
            if (j == (wc >> 5)) {
              const f32x16 t = acc[r][i][j];
              int x = 0;
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int w = (int)__float_as_uint(t[v]);
                const int k0 = 8 * (v >> 2) + (v & 3);          // row of register v in lanes 0 .. 31; + 4 in lanes 32 .. 63
                const int s_lo = __builtin_amdgcn_readlane(w, sel), s_hi = __builtin_amdgcn_readlane(w, sel + 32);
                x = lane == k0 ? s_lo : x;
                x = lane == k0 + 4 ? s_hi : x;
              }
              const int row = m0 + wm * WTM + 32 * i + l32;
              const float Tv = row >= p.M        ? __builtin_inff()
                               : p.bound_global ? p.t_global
                                                : __fmul_rn(__fmul_rn(col_kra[i], cb_c), p.gamma);
              account(lane < 32 && row < p.M, __uint_as_float((uint32_t)x), Tv, col_cs[r][i], col_sa[r][i]);
            }
          });
        } else if constexpr (OPS) {
          // One column, wave tiles of 8 accumulator tiles (no registers to spare for the gather):
          // the lanes holding the column read their rows' golden values; the other lanes read
          // their own columns of the same rows (same cache lines) and count nothing.
          static_for<TM * TN>([&](auto tt) {
            constexpr int i = tt / TN, j = tt % TN;
            const f32x16 T = thresholds(tt);
            const f32x16 t = acc[r][i][j];
            const int col = col_base + 32 * j;
            float cs[16], sa[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
              const size_t idx = (size_t)min(row, p.M - 1) * p.N + min(col, p.N - 1);
              cs[v] = p.c_star[idx];
              sa[v] = p.s_abs[idx];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
              account(col == site_col && row < p.M, t[v], T[v], cs[v], sa[v]);
            }
          });
        }
        if (lane == 0) {
          if (n_bit) atomicAdd(&res->n_bitdiff, n_bit);
          if (n_pre) atomicAdd(&res->n_dev_pre, n_pre);
          if (n_post) atomicAdd(&res->n_dev_post, n_post);
          if (n_bT) atomicAdd(&res->n_border_T, n_bT);
          if (n_btau) atomicAdd(&res->n_border_tau, n_btau);
        }
        mxp[r] = mx_pre;
        mxq[r] = mx_post;
      }
    });
    // non-negative floats (and +Inf) order like their words
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      static_for<R>([&](auto rr) {
        mxp[rr] = fmaxf(mxp[rr], __shfl_xor(mxp[rr], o, 64));
        mxq[rr] = fmaxf(mxq[rr], __shfl_xor(mxq[rr], o, 64));
      });
    }
    static_for<R>([&](auto rr) {
      constexpr int r = rr;
      if (((owned >> r) & 1u) && lane == 0) {
        fi_trial_result* res = p.results + trial[r];
        if (mxp[r] > 0.0f) atomicMax(reinterpret_cast<uint32_t*>(&res->max_dev_pre), __float_as_uint(mxp[r]));
        if (mxq[r] > 0.0f) atomicMax(reinterpret_cast<uint32_t*>(&res->max_dev_post), __float_as_uint(mxq[r]));
      }
    });
  };

  // ---- start-up of the first item (the only exposed one)
  locate(w_cur, cur);
  desc_cur = load_desc(cur.grp);
  issue_tile(cur, 0, 0);
  uint32_t w_nxt = w_cur + gridDim.x;
  bool has_next = w_nxt < n_work;
  auto locate_next = [&]() __attribute__((always_inline)) {
    if (has_next) {
      locate(w_nxt, nxt);
      desc_nxt = load_desc(nxt.grp);
    }
  };
  if constexpr (!LATE_NEXT) locate_next();
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();
  Frags f0, f1;
  read_frags(f0, smem, 0);
  const int nkt = p.K / BK;

  // ---- items.  Within one: double-buffered LDS, one barrier per k-tile.  The barrier sits
  // before the last of the four MFMA steps of a tile: by then a wave holds the tile's last
  // fragments in registers, so right after the barrier it reads the first fragments of the next
  // tile (of this item or the next) while R*TM*TN MFMAs are still to issue - the LDS latency
  // that follows a barrier is covered by work instead of idling the pipe.
  for (;;) {
    decode();
    if constexpr (EARLY_T) fetch_threshold_inputs();

    // One k-tile.  Every fragment read is issued inside the MFMA burst of the step before the
    // one that uses it (after the first few MFMAs), so a wave never waits for a read it has just
    // issued; the barrier sits before the last step, whose fragments the wave already holds, and
    // the first fragments of the next tile are read inside that last burst.  FIRST: the k-tile
    // that opens an item (its first step starts the accumulators from zero).  LAST: the k-tile
    // that ends an item - the tile loading into the other stage then belongs to the next item.
    // EV: the k-tile holds an event of this wave - an accumulator fault after one of its steps,
    // or (OPS) an operand word one of its steps consumes.
    auto k_tile = [&](auto with_events, auto is_first, auto last_mode, auto stage_c, int kt) __attribute__((always_inline)) {
      constexpr bool EV = decltype(with_events)::value;
      constexpr bool FIRST = decltype(is_first)::value;
      // last_mode: 0 not the last k-tile, 1 the last, 2 decided at run time (items with events)
      constexpr int LM = decltype(last_mode)::value;
      static_assert(!(EV && FIRST), "items with events clear their accumulators up front");
      // stage_c: 0 or 1 when the LDS stage is known at compile time (the addresses of the
      // fragment reads then fold into immediates), -1 to use the running variable.
      constexpr int SC = decltype(stage_c)::value;
      if constexpr (SC >= 0) stage = SC;
      const bool last = LM == 2 ? kt == nkt - 1 : LM == 1;
      const bool more = !last || has_next;                // a tile follows in the other stage
      if constexpr (EV) {
        // Nothing of the rare paths stays in flight across the tile prefetch: the compiler
        // places its waits statically, and a pending access would make the hot code wait for it.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_sched_barrier(0);
      }
      // The next k-tile's loads: spread over the bursts of steps 0 .. 2 in the check-free copies
      // that know at compile time what follows; in one block up front in the rare copies.
      constexpr bool SPREAD = !EV && LM != 2;
      if constexpr (!SPREAD) {
        if constexpr (LM == 0) issue_tile(cur, kt + 1, stage ^ 1);
        else if constexpr (LM == 1) { if (has_next) issue_tile(nxt, 0, stage ^ 1); }
        else if (more) issue_tile_of(last, kt, stage ^ 1);
      }
      const uint8_t* s = smem + stage * STAGE;
      const uint8_t* s_other = smem + (stage ^ 1) * STAGE;
      auto load = [&](auto kk) __attribute__((always_inline)) {
        if constexpr (SPREAD) {
          if constexpr (LM == 0) issue_one(cur, kt + 1, stage ^ 1, kk);
          else if (has_next) issue_one(nxt, 0, stage ^ 1, kk);
        }
      };
      auto step = [&](Frags& f, int g, auto first, auto sit, auto&& mid) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (EV) {
          const uint32_t m = hit_mask(g);
          if constexpr (OPS) {
            mma_step_ops(f, m, mid);
          } else {
            mma_step_mid(f, first, sit, mid, load);
            __builtin_amdgcn_sched_barrier(0);
            if (__builtin_expect(m != 0, 0)) hooks(m);
          }
        } else {
          mma_step_mid(f, first, sit, mid, load);
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      using s0 = std::integral_constant<int, 0>;
      using s1 = std::integral_constant<int, 1>;
      using s2 = std::integral_constant<int, 2>;
      using s3 = std::integral_constant<int, 3>;
      step(f0, 4 * kt, std::integral_constant<bool, FIRST>{}, s0{}, [&]() { read_frags(f1, s, 1); });
      step(f1, 4 * kt + 1, std::false_type{}, s1{}, [&]() { read_frags(f0, s, 2); });
      step(f0, 4 * kt + 2, std::false_type{}, s2{}, [&]() { read_frags(f1, s, 3); });
      // Every fragment of this stage is in registers (the barrier's fence waits for the reads);
      // once all waves are here the next tile has landed and this stage may be overwritten.
      if (more) __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's loads have landed
      __syncthreads();
      step(f1, 4 * kt + 3, std::false_type{}, s3{}, [&]() { if (more) read_frags(f0, s_other, 0); });
      stage ^= 1;
    };
    using dyn = std::integral_constant<int, -1>;
    using st0 = std::integral_constant<int, 0>;
    using st1 = std::integral_constant<int, 1>;
    using yes = std::true_type;
    using no = std::false_type;
    using mid_tile = std::integral_constant<int, 0>;
    using last_tile = std::integral_constant<int, 1>;
    using any_tile = std::integral_constant<int, 2>;
    if (PROP || !has_events) {
      // Nearly every wave of nearly every item: no event check anywhere.
      if (nkt == 1) {
        if constexpr (LATE_NEXT) locate_next();
        k_tile(no{}, yes{}, last_tile{}, dyn{}, 0);
      } else if ((nkt & 1) == 0 && stage == 0) {
        // an even number of k-tiles: every item starts in stage 0 and the stages alternate statically
        k_tile(no{}, yes{}, mid_tile{}, st0{}, 0);
        if (nkt > 2) {
          k_tile(no{}, no{}, mid_tile{}, st1{}, 1);
          for (int kt = 2; kt + 2 < nkt; kt += 2) {
            k_tile(no{}, no{}, mid_tile{}, st0{}, kt);
            k_tile(no{}, no{}, mid_tile{}, st1{}, kt + 1);
          }
          k_tile(no{}, no{}, mid_tile{}, st0{}, nkt - 2);
        }
        if constexpr (LATE_NEXT) locate_next();
        k_tile(no{}, no{}, last_tile{}, st1{}, nkt - 1);
      } else {
        k_tile(no{}, yes{}, mid_tile{}, dyn{}, 0);
        for (int kt = 1; kt + 1 < nkt; ++kt) k_tile(no{}, no{}, mid_tile{}, dyn{}, kt);
        if constexpr (LATE_NEXT) locate_next();
        k_tile(no{}, no{}, last_tile{}, dyn{}, nkt - 1);
      }
    } else if constexpr (!PROP) {
      // A wave with events in this item alternates runs of check-free k-tiles with single
      // k-tiles of the checking copy, one per k-tile that holds an event.  (A choice between the
      // two copies inside one loop body - MFMAs over all accumulators in both arms of a branch -
      // makes the register allocator spill; a loop followed by a conditional tile does not.)
      // Both copies execute the same barriers, so the waves of a workgroup may take different
      // ones.  These copies keep to the running LDS stage, find out at run time whether a k-tile
      // is the item's last, and the accumulators are cleared up front: rare path, and every copy
      // of a k-tile costs code.
      if constexpr (LATE_NEXT) locate_next();
      static_for<R * TM * TN>([&](auto t) {
        acc[t / (TM * TN)][(t / TN) % TM][t % TN] =
            f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      });
      for (int kt = 0; kt < nkt;) {
        int ev_tile = nkt;                                // first k-tile at or after kt with an event
        static_for<R>([&](auto rr) {
          const int t = hook_step[rr] >> 2;               // -1 >> 2 == -1: no event
          ev_tile = (t >= kt && t < ev_tile) ? t : ev_tile;
        });
        for (; kt < ev_tile; ++kt) k_tile(no{}, no{}, any_tile{}, dyn{}, kt);
        if (kt < nkt) {
          k_tile(yes{}, no{}, any_tile{}, dyn{}, kt);
          ++kt;
        }
      }
    }

    epilogue();
    if (!has_next) break;                                // uniform: every wave leaves here
    cur = nxt;
    desc_cur = desc_nxt;
    w_cur = w_nxt;
    w_nxt = w_cur + gridDim.x;
    has_next = w_nxt < n_work;
    if constexpr (!LATE_NEXT) locate_next();
  }
  if (p.clocks && blockIdx.x == 0 && tid == 0) {
    p.clocks[4 * VAR + 2] = __builtin_readcyclecounter();
    p.clocks[4 * VAR + 3] = __builtin_amdgcn_s_memrealtime();
  }
}

}  // namespace fi
