// The main kernel of the bf16 MFMA path (k_attn_bf16) and its launchers, as templates.  The
// instantiations are spread over several translation units (pv_attn_bf16_inst.hip compiled once
// per head size and set of group sizes) so that they build in parallel; pv_attn_bf16.hip holds the
// dispatch.
#ifndef PV_ATTN_BF16_MAIN_H_
#define PV_ATTN_BF16_MAIN_H_

#include "pv_attn_common.h"
#include "pv_short_rows.h"

namespace pv {

// ---------------------------------------------------------------- main kernel
// FOLD: the softmax scale (times log2 e) is folded into Q before its single bf16 rounding, which
// is free when Q is rotated anyway.  Without rotation Q enters the MFMA exactly as given and the
// scale multiplies the fp32 score inside the exponent instead.
// QT ("query-tile workgroups", G == 4 waves): the four waves are four consecutive query tiles of ONE
// query head instead of the heads of a group; used for group sizes that would leave wave slots of
// a compute unit empty.  `tile` is then the union descriptor of the four tiles (it drives the key
// loop and the staging) and every wave loads, masks and stores with its own tile `mine`.
template <int D, int G, bool FOLD, bool QT = false>
__global__ __launch_bounds__(G * 64, 2) __attribute__((amdgpu_waves_per_eu(2))) void k_attn_bf16(
    const int32_t* __restrict__ plan, PlanHeader h, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ krot, const uint16_t* __restrict__ vt,
    const float2* __restrict__ cs, void* __restrict__ out, float* __restrict__ lse, int hq, int hkv,
    float qscale, bool rope, bool out_f32, int split, float* __restrict__ part, KvSource raw_kv,
    float scale, int n_short_blocks) {
  constexpr int KT = D / 16;            // MFMA steps along the feature dim for S^T
  constexpr int DB = D / 32;            // 32-feature blocks of O^T
  constexpr int CH32 = 32 * D / 8;      // 16-byte chunks per 32-key K (or V^T) slot
  constexpr int CPR = D / 8;            // chunks per key row
  constexpr int NS = (D == 128) ? 5 : 8;                 // slots per ring (32 keys each)
  constexpr int HPW = (CH32 / 64) / G;                   // staging loads every wave issues per slot
  constexpr unsigned SLOT_BYTES = CH32 * 16;
  // One LDS array on purpose: with several LDS variables the compiler attaches alias scopes and
  // then makes every LDS read wait for all outstanding global->LDS loads, which would serialise
  // the staging pipeline.  Ordering is enforced here with explicit vmcnt waits and barriers.
  // Layout: K ring (NS slots), then V^T ring (NS slots).  Step s lives in slot s % NS of each.
  __shared__ uint4 smem[2 * NS * CH32];

  // The last n_short_blocks workgroups of a whole-pass launch evaluate the rows with very few keys
  // in fp32, one (row, kv head) each, from the caller's K/V and the table of rotary angles.  They
  // are light and start when the grid's items are all taken, in the tail of the launch.
  if constexpr (G >= 4) {
    if (n_short_blocks > 0 && blockIdx.x >= gridDim.x - (unsigned)n_short_blocks) {
      static_assert(2 * PV_SHORT_ROW_KEYS * D * 4 <= sizeof(smem), "short-row tiles must fit");
      const int idx = (int)(blockIdx.x - (gridDim.x - (unsigned)n_short_blocks));
      const int4 desc = reinterpret_cast<const int4*>(plan + h.off_short)[idx / hkv];
      ShortRowArgs a;
      a.q = q; a.out = out; a.lse = lse; a.hq = hq; a.scale = scale; a.out_f32 = out_f32;
      a.seg_only = false; a.table = cs;
      float (*ks)[D] = reinterpret_cast<float (*)[D]>(&smem[0]);
      short_row_block<D, G>(plan, h, raw_kv, nullptr, hkv, rope, a, desc, idx % hkv, ks, ks + PV_SHORT_ROW_KEYS);
      return;
    }
  }

  // split == 0: the whole pass, one workgroup per entry of the work list and kv head.
  // split >= 1: segment rows only, one workgroup per (tile holding segment rows, kv head, piece);
  //             piece c of `split` covers the c-th share of the tile's listed key tiles.
  const int piece = split ? (int)blockIdx.x % split : 0;
  const int item = split ? (int)blockIdx.x / split : (int)blockIdx.x;   // (tile, kv head)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);      // wave index as a scalar
  const int qrow = lane & 31, hh = lane >> 5;
  int kvh, head;
  QTile tile, mine;
  if constexpr (QT) {
    static_assert(G == 4, "query-tile workgroups have four waves");
    head = (int)blockIdx.x % hq;
    kvh = head / (hq / hkv);
    tile = reinterpret_cast<const QTile*>(plan + h.off_quadwork)[(int)blockIdx.x / hq];
    mine = tile;                              // a wave without a tile of its own: no row, never masks
    mine.t0 = tile.t0 + 32 * wave_s;
    mine.rows = 0;
    mine.n_full = 1 << 24;
    if (32 * wave_s < tile.rows)              // tile.n_full: index of the group's first tile
      mine = reinterpret_cast<const QTile*>(plan + h.off_tiles)[tile.n_full + wave_s];
  } else {
    kvh = item % hkv;
    head = kvh * G + wave;
    tile = reinterpret_cast<const QTile*>(plan + (split ? h.off_segwork : h.off_work))[item / hkv];
    mine = tile;
  }
  const bool valid = qrow < mine.rows;
  const int64_t g = (int64_t)mine.tok_base + mine.t0 + qrow;
  int a_end = 0, b_start = 0;
  if (valid) { a_end = plan[h.off_aend + g]; b_start = plan[h.off_bstart + g]; }

  bf16x8 qf[KT];          // Q operand of this wave's head (filled below, once the tile is in LDS)

  // ---- key steps.  A key tile of the plan (64 keys) is two steps of 32 keys; tiles run over
  // [0, n_a) then [jb0, jb1).  The number of steps is even.
  const int n_listed = tile.n_a + (tile.jb1 - tile.jb0);
  const int kt0 = split ? piece * n_listed / split : 0;                 // first listed key tile
  const int n_tiles = (split ? (piece + 1) * n_listed / split : n_listed) - kt0;
  const int n_steps = 2 * n_tiles;
  const int last = n_steps - 1;
  // partial result of this wave (split > 1): float [32][D], then float2 [32] = (nmref, row sum)
  float* part_o = part + ((int64_t)((int64_t)item * split + piece) * G + wave) * (32 * (D + 2));
  if (n_steps == 0) {                       // fewer key tiles than pieces: this piece is empty
    if (hh == 0) reinterpret_cast<float2*>(part_o + 32 * D)[qrow] = make_float2(0.0f, 0.0f);
    return;
  }
  // the plan lists the longest items first: they bound the run time, so their waves go first
  // wherever they share a SIMD with a shorter item
  if (blockIdx.x < gridDim.x / 4) __builtin_amdgcn_s_setprio(3);
  const int64_t head_base = ((int64_t)kvh * h.padded_keys + tile.kpad_base) * D;   // elements
  auto step_key0 = [&](int j) {           // first key (request-local) of step j
    const int idx = (j >> 1) + kt0;
    const int jt = idx < tile.n_a ? idx : tile.jb0 + (idx - tile.n_a);
    return jt * 64 + (j & 1) * 32;
  };
  // Direct global->LDS staging: a wave instruction moves 64 consecutive 16-byte chunks, lane l
  // landing at chunk (base + l).  Both workspaces are already in MFMA operand order, so a slot is
  // a plain copy and operand reads are linear (lane l reads chunk l of its k-step: no conflicts).
  constexpr int NREP = (CH32 / 64 + G - 1) / G;                  // staging instructions per wave
  const unsigned lane16 = (unsigned)lane * 16;
  // the row's own index in its request (-1: no row).  Recomputed where it is needed, in the mask
  // code and the epilogue, from a lane index the compiler cannot hoist: the register file is full,
  // and a value that lives through the loops for the sake of a rare path ends up in scratch memory.
  auto own_row = [&]() {
    unsigned l16 = lane16;
    asm volatile("" : "+v"(l16));
    const int r = (int)((l16 >> 4) & 31u);
    return r < mine.rows ? mine.t0 + r : -1;
  };
  const unsigned smem_base =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)(char*)&smem[0];
  const unsigned vring = smem_base + NS * SLOT_BYTES;
  const char* krot_b = reinterpret_cast<const char*>(krot) + head_base * 2;
  const char* vt_b = reinterpret_cast<const char*>(vt) + head_base * 2;
  // stage the K (or V^T) half of step s into its ring slot; nothing is issued beyond the last step
  auto stage_slot = [&](const char* src, unsigned lds0) {
#pragma unroll
    for (int n = 0; n < NREP; ++n) {
      const int c = wave_s + n * G;
      if ((CH32 / 64) % G != 0 && c >= CH32 / 64) break;
      unsigned lo = lane16;
      asm volatile("" : "+v"(lo));     // keeps the address in (scalar base + 32-bit lane offset) form
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src + c * 1024 + lo),
          (__attribute__((address_space(3))) void*)(uintptr_t)(lds0 + c * 1024), 16, 0, 0);
    }
  };
  auto stage_k_to = [&](int s, int slot) {             // step s (<= last) into K slot `slot`
    stage_slot(krot_b + (int64_t)step_key0(s) * (D * 2), smem_base + (unsigned)slot * SLOT_BYTES);
  };
  auto stage_v_to = [&](int s, int slot) {
    stage_slot(vt_b + (int64_t)step_key0(s) * (D * 2), vring + (unsigned)slot * SLOT_BYTES);
  };
  auto stage_k = [&](int s) { if (s <= last) stage_k_to(s, s % NS); };
  auto stage_v = [&](int s) { if (s <= last) stage_v_to(s, s % NS); };
  // wait until at most n slots' worth of this wave's staging loads are outstanding (every wave
  // issues at least HPW loads per slot, so n * HPW never exceeds what is really in flight)
  auto wait_slots = [&](auto max_n, int n) {           // n <= max_n
    constexpr int MAXN = decltype(max_n)::value;
    bool done = false;
    static_for<0, MAXN>([&](auto c) {
      constexpr int v = MAXN - decltype(c)::value;
      // (the counter has 6 bits: what stays in flight plus the loads of one more step must fit)
      if constexpr (v * HPW + 2 * NREP <= 63) {
        if (!done && n >= v) { __builtin_amdgcn_s_waitcnt(vmcnt_imm(v * HPW)); done = true; }
      }
    });
    if (!done) __builtin_amdgcn_s_waitcnt(0x0f70);
  };
  bf16x8 kf[KT];          // K operand of the next S^T
  bf16x8 vf[2][DB];       // V^T operands of the current step
  // per-lane LDS byte addresses inside slot 0: k-step t of K is 1 KB further per t
  const unsigned k_off = smem_base + lane16;
  const unsigned v_off = vring + (unsigned)((hh * D + qrow) * 16);
  auto load_k = [&](int slot) {
    const unsigned a = k_off + (unsigned)slot * SLOT_BYTES;
    static_for<0, KT>([&](auto t) { kf[t] = lds_read_b128<decltype(t)::value * 1024>(a); });
  };
  auto wait_kv = [&]() {   // every outstanding LDS read of this wave has landed
    if constexpr (D == 128) {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]),
                     "+v"(kf[6]), "+v"(kf[7]), "+v"(vf[0][0]), "+v"(vf[0][1]), "+v"(vf[0][2]),
                     "+v"(vf[0][3]), "+v"(vf[1][0]), "+v"(vf[1][1]), "+v"(vf[1][2]), "+v"(vf[1][3]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(vf[0][0]),
                     "+v"(vf[0][1]), "+v"(vf[1][0]), "+v"(vf[1][1]));
    }
  };

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.0f;
  // The probability of a score s is 2^(esc * s - mref): mref, in log2 units, is a per-row reference
  // that is only re-centred when a row sum leaves a safe window (see recentre below); l_run and o
  // are relative to it.  nmref = -mref is what the exponent adds.
  float nmref = 0.0f, l_run = 0.0f;
  const float esc = FOLD ? 1.0f : qscale;   // FOLD: the scale is already in Q
  // FOLD: the exponent is score + nmref with nothing to multiply, and the matrix pipe does that
  // addition: every lane's 16 scores belong to one query row, so S^T accumulates on top of a tile
  // that holds nmref in all 16 registers (cref) instead of on top of zero, and a score tile is
  // "biased": it already is the exponent.  A change of the reference (rare) also corrects the
  // biased tiles that exist at that moment.
  f32x16 cref;
#pragma unroll
  for (int r = 0; r < 16; ++r) cref[r] = 0.0f;
  auto prob = [&](float x) {
    return __builtin_amdgcn_exp2f(FOLD ? x : __builtin_fmaf(x, esc, nmref));
  };
  auto qk = [&](f32x16& acc) {
    if constexpr (FOLD) {
      acc = cref;
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    }
#pragma unroll
    for (int t = 0; t < KT; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], acc, 0, 0, 0);
  };
  // The 16 scores of a lane are keys key0 + 4 hh + c, c = 8 (r / 4) + r % 4, of one query row: the row's
  // visible keys among the step's 32 become a bit mask (three clamped "low n bits" masks), and every
  // score is kept or replaced by -inf with a bit-field extract and a bit-field insert.
  auto apply_mask = [&](f32x16& sc, int key0) __attribute__((always_inline)) {
    const int base = key0 + 4 * hh;
    auto low_bits = [](int n) {                         // bits [0, n) of 32, n clamped to [0, 32]
      const unsigned m = (1u << (n & 31)) - 1u;
      return n <= 0 ? 0u : n >= 32 ? 0xffffffffu : m;
    };
    const int i_loc = own_row();
    const unsigned vis = low_bits(a_end - base) | (low_bits(i_loc - base + 1) & ~low_bits(b_start - base));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const unsigned keep = (unsigned)__builtin_amdgcn_sbfe((int)vis, 8 * (r / 4) + (r % 4), 1);   // all ones or zero
      sc[r] = __uint_as_float((__float_as_uint(sc[r]) & keep) | (0xff800000u & ~keep));
    }
  };
  // p rounded to bf16 once; the row sum is taken over the rounded values (v_dot2c with a pair of
  // ones), so that O is an exact convex combination of V rows with the weights the MFMA sees
  auto probs = [&](const f32x16& sc, unsigned (&pw)[8]) __attribute__((always_inline)) {
    float rs = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pw[e] = pack_bf16(prob(sc[2 * e]), prob(sc[2 * e + 1]));
      rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[e]),
                                           __builtin_bit_cast(bf16x2, 0x3f803f80u), rs, false);
    }
    return rs;
  };
  // The window test of a step: its partial row sum `rs` must not exceed 2^40, and the running sum
  // with it must have reached 2^-40.  (The lower bound is on the total, not on the step: a step
  // whose keys are all masked for a lane, every step of a diagonal tile for some lane, or whose
  // scores lie 40 octaves below a healthy history adds nothing, and nothing needs correcting.)
  auto out_of_window = [&](float rs) {
    return __builtin_amdgcn_ballot_w64(!(l_run + rs >= 0x1p-40f && rs <= 0x1p40f)) != 0;
  };
  // One exact online-softmax step for the whole wave: taken when the window test fails (it also
  // catches inf/NaN, and a running sum still at 0).  Rare: first steps of a row while no key is
  // visible to it, or scores rising by more than 40 octaves.  The reference moves to this step's
  // row maximum, but never so far down that the history (l, O) would leave fp32 range:
  // mref_new >= mref + log2(l) - 20.  `sc` are the scores being exponentiated.  Both half-waves of
  // a row take identical decisions.  `other` is the score tile of the step after `sc`'s (FOLD: it is
  // biased with the old reference as well).
  auto recentre = [&](f32x16& sc, unsigned (&pw)[8], f32x16& other) __attribute__((always_inline)) {
    float mx = sc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
    mx = pair_max(mx);
    const float l_tot = pair_sum(l_run);
    if (mx > -INFINITY && mx < INFINITY) {      // rows with no visible key keep their reference
      // FOLD: mx is biased, the row maximum itself is mx - nmref
      float nm_new = FOLD ? nmref - mx : -mx * esc, alpha = 0.0f;   // empty history: nothing to rescale
      if (l_tot > 0.0f) {
        nm_new = fminf(nm_new, nmref - (__builtin_amdgcn_logf(l_tot) - 20.0f));
        alpha = __builtin_amdgcn_exp2f(nm_new - nmref);
      }
      if constexpr (FOLD) {
        const float delta = nm_new - nmref;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sc[r] += delta; other[r] += delta; cref[r] = nm_new; }
      }
      nmref = nm_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    return probs(sc, pw);
  };

  // ---- Q tile (and its cos/sin rows) through LDS.  A lane needs 16-byte pieces of 32 different
  // rows, which as direct global loads is one cache line per lane; instead the waves copy whole
  // rows with global->LDS loads (swizzled like K) into the END of the ring memory, read their
  // operands from there, and only then stage what belongs to that memory.  The K slots in front of
  // that area are staged right away, so their latency overlaps that of the Q tile.
  constexpr int QCH = G * 32 * CPR;                 // 16-byte chunks of the Q tile
  constexpr int CSR = D / 4;                        // chunks per table row (D/2 float2)
  constexpr int CSCH = 32 * CSR;
  static_assert(QCH + CSCH <= 2 * NS * CH32, "Q tile and table must fit the rings");
  constexpr int QAREA0 = 2 * NS * CH32 - (QCH + CSCH);            // first chunk of the area
  // K slots staged together with the Q tile: those in front of the area, as far as the loads of
  // one wave (Q tile, table, K slots) stay within the range of the 6-bit load counter
  constexpr int QLOADS = QCH / 64 / G + (CSCH / 64 + G - 1) / G;
  constexpr int NK0_FIT = (56 - QLOADS) / NREP > 0 ? (56 - QLOADS) / NREP : 0;
  constexpr int NK0_FREE = (QAREA0 / CH32) < NS ? (QAREA0 / CH32) : NS;
  constexpr int NK0 = NK0_FREE < NK0_FIT ? NK0_FREE : NK0_FIT;
  {
    const int rows_m1 = tile.rows - 1;
    const int64_t tok0 = (int64_t)tile.tok_base + tile.t0;
    const unsigned q_area = smem_base + QAREA0 * 16, cs_area = q_area + QCH * 16;
#pragma unroll
    for (int n = 0; n < QCH / 64 / G; ++n) {          // 32*CPR/64 instructions per wave
      const int c = wave_s + n * G;
      const int P = c * 64 + lane;
      const int R = P >> 4, pos = P & 15;
      const int Pg = (R << 4) + (pos ^ (R & 15));     // global chunk that lands at LDS chunk P
      const int row = Pg / CPR, ch = Pg % CPR;
      // rows [32 hl, 32 hl + 32) of the area: head hl of the group, or (QT) tile hl of this head
      const int hl = row >> 5;
      const int tok = QT ? min(32 * hl + (row & 31), rows_m1) : min(row & 31, rows_m1);
      const int src_head = QT ? head : kvh * G + hl;
      const uint16_t* src = q + (caller_row(plan, h, tok0 + tok) * hq + src_head) * D + (ch << 3);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)src,
          (__attribute__((address_space(3))) void*)(uintptr_t)(q_area + c * 1024), 16, 0, 0);
    }
    // cos/sin rows: one set for the whole workgroup through LDS, or (QT: four times as many rows)
    // every lane's own 16-byte pieces straight from the table
    uint4 cs_own[QT && FOLD ? (KT / 2) * 4 : 1];
    if constexpr (QT && FOLD) {
      const uint4* row = reinterpret_cast<const uint4*>(cs + (tok0 + min(32 * wave_s + qrow, rows_m1)) * (D / 2));
#pragma unroll
      for (int t = 0; t < KT / 2; ++t)
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) cs_own[t * 4 + k2] = row[8 * t + 4 * hh + k2];
    }
    if (FOLD && !QT) {
#pragma unroll
      for (int n = 0; n < (CSCH / 64 + G - 1) / G; ++n) {
        const int c = wave_s + n * G;
        if ((CSCH / 64) % G != 0 && c >= CSCH / 64) break;
        const int P = c * 64 + lane;
        const int R = P >> 4, pos = P & 15;
        const int Pg = (R << 4) + (pos ^ (R & 15));
        const int tok = min(Pg / CSR, rows_m1), ch = Pg % CSR;
        const float2* src = cs + (tok0 + tok) * (D / 2) + (ch << 1);
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)src,
            (__attribute__((address_space(3))) void*)(uintptr_t)(cs_area + c * 1024), 16, 0, 0);
      }
    }
#pragma unroll
    for (int s = 0; s < NK0; ++s) stage_k(s);
    wait_slots(std::integral_constant<int, NK0>{}, min(NK0, n_steps));   // Q tile and table have landed
    __builtin_amdgcn_s_barrier();
    const uint4* q_lds = &smem[QAREA0];
    const uint4* cs_lds = q_lds + QCH;
    auto swz = [](int L) { const int R = L >> 4, pos = L & 15; return (R << 4) + (pos ^ (R & 15)); };
    float x[KT][8];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const uint4 raw = q_lds[swz((wave * 32 + qrow) * CPR + 2 * t + hh)];
      const unsigned* pr = reinterpret_cast<const unsigned*>(&raw);
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[t][2 * e] = bf16_lo(pr[e]); x[t][2 * e + 1] = bf16_hi(pr[e]); }
    }
    if (FOLD) {             // FOLD <=> rotary embedding on: pair (c, c + D/2), c = 16 t + 8 hh + e
#pragma unroll
      for (int t = 0; t < KT / 2; ++t) {
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
          const uint4 w = (QT && FOLD) ? cs_own[(QT && FOLD) ? t * 4 + k2 : 0]
                                       : cs_lds[swz(qrow * CSR + 8 * t + 4 * hh + k2)];
          const float c0 = __uint_as_float(w.x), s0r = __uint_as_float(w.y);
          const float c1 = __uint_as_float(w.z), s1r = __uint_as_float(w.w);
          const float lo0 = x[t][2 * k2], hi0 = x[t + KT / 2][2 * k2];
          const float lo1 = x[t][2 * k2 + 1], hi1 = x[t + KT / 2][2 * k2 + 1];
          x[t][2 * k2] = lo0 * c0 - hi0 * s0r;
          x[t + KT / 2][2 * k2] = hi0 * c0 + lo0 * s0r;
          x[t][2 * k2 + 1] = lo1 * c1 - hi1 * s1r;
          x[t + KT / 2][2 * k2 + 1] = hi1 * c1 + lo1 * s1r;
        }
      }
    }
    const float f = FOLD ? qscale : 1.0f;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      uint4 pk;
      pk.x = pack_bf16(x[t][0] * f, x[t][1] * f);
      pk.y = pack_bf16(x[t][2] * f, x[t][3] * f);
      pk.z = pack_bf16(x[t][4] * f, x[t][5] * f);
      pk.w = pack_bf16(x[t][6] * f, x[t][7] * f);
      qf[t] = as_bf16x8(pk);
    }
    __syncthreads();                                  // the area may now be overwritten
  }

  // ---- pipeline prologue: P(0), S(1), K operand of step 2, V operand of step 0
  f32x16 sA, sB;           // score tiles, alternating roles from step to step
  unsigned pA[8], pB[8];   // probability tiles (bf16 pairs), likewise
  // the slots that could not be staged before the Q tile: K(NK0 ..), then all of V^T
  constexpr int NL = 2 * NS - NK0;
  auto stage_late = [&](auto i) {
    constexpr int I = decltype(i)::value;
    if constexpr (I < NS - NK0) stage_k(NK0 + I);
    else if constexpr (I < NL) stage_v(I - (NS - NK0));
  };
  if constexpr (NK0 >= 2) {
    // K of steps 0 and 1 has landed (every wave waited for its loads before the barriers of the Q
    // tile), so S(0) starts right away and the late slots are staged between its MFMAs.
    load_k(0);
    wait_kv();
#pragma unroll
    for (int r = 0; r < 16; ++r) sA[r] = 0.0f;
    static_for<0, KT>([&](auto t) {
      constexpr int T = decltype(t)::value;
      sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[T], qf[T], sA, 0, 0, 0);
      static_for<0, (NL + KT - 1) / KT>([&](auto m) {
        stage_late(std::integral_constant<int, T + decltype(m)::value * KT>{});
      });
    });
  } else {
    static_for<0, NL>([&](auto i) { stage_late(i); });
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __builtin_amdgcn_s_barrier();      // not __syncthreads(): that would wait for the loads in flight
    load_k(0);
    wait_kv();
    qk(sA);                                          // S(0)
  }
  __builtin_amdgcn_sched_barrier(0);
  load_k(min(1, last) % NS);
  if (step_key0(0) >= mine.n_full * 64) apply_mask(sA, step_key0(0));
  float rs0 = probs(sA, pA);
  wait_kv();
  qk(sB);                                            // S(1)
  __builtin_amdgcn_sched_barrier(0);
  // Everything staged so far is needed from here on, and every wave is done with K slots 0 and 1:
  // refill them (steps NS, NS+1).  From now on iteration j issues K(j+2+NS) and V^T(j+NS).
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __syncthreads();
  stage_k(NS);
  stage_k(NS + 1);
  {   // same issue order as inside the loop: V^T t, K t, V^T t+1, ...
    const unsigned sbk = (unsigned)(min(2, last) % NS) * SLOT_BYTES;
    static_for<0, KT>([&](auto t) {
      constexpr int uu = decltype(t)::value / DB, db = decltype(t)::value % DB;
      vf[uu][db] = lds_read_b128<(uu * 2 * D + db * 32) * 16>(v_off);
      kf[t] = lds_read_b128<decltype(t)::value * 1024>(k_off + sbk);
    });
  }
  if (out_of_window(rs0)) rs0 = recentre(sA, pA, sB);
  l_run += rs0;

  // One step: O^T += V^T P^T of step j and S^T of step j+2 on the MFMA pipe, the probabilities of
  // step j+1 on the VALU, and the LDS reads of the next step's operands (V^T of step j+1, K of
  // step j+3), each issued as soon as the register it refills has been consumed.
  //   s_in  scores of step j+1 (input)          s_out  scores of step j+2 (result)
  //   p_in  probabilities of step j (input)     p_out  probabilities of step j+1 (result)
  int slot_v = min(1, last) % NS, slot_k = min(3, last) % NS;   // slots of step j+1 and step j+3
  //   kSteady     both refills of this step exist and the pipeline is full: the wait is a constant and
  //               the staging loads are issued from inside the MFMA block (no branch splits it)
  //   kFill       both refills exist, the pipeline is still filling: staging as in steady state, the
  //               wait counted at run time
  //   kDrain      nothing is left to stage: no staging code, and the wait is for every load
  //   kGeneric    anything else: counts and staging decided at run time.  kPartial is the same code
  //               under a second name for the steps in which only some refills are left: one copy
  //               of the step per loop (the compiler kept the step's registers out of scratch memory
  //               that way, and not with one copy called from two loops)
  constexpr int kGeneric = 0, kSteady = 1, kFill = 2, kDrain = 3, kPartial = 4;
  // Steady state runs in whole periods of the slot rotation as long as it can (PP pairs of steps,
  // unrolled): a step at position SP = 2 p + e of a period knows its slots at compile time, so the
  // LDS addresses are immediates, and it finds its staging sources by advancing two byte offsets
  // instead of looking the key tile up.  SP = -1: slots and sources computed at run time.
  constexpr int JS = (NS - 2 + 1) & ~1;                 // first step of steady state
  constexpr int PP = (NS % 2) ? NS : NS / 2;
  constexpr unsigned HALF = 32 * D * 2;                 // bytes of one step's K (or V^T) rows
  // steps from s_mask on hold keys that some row does not see (keys rise with the step)
  const int idx_mask = mine.n_full < tile.n_a ? mine.n_full : tile.n_a + max(0, mine.n_full - tile.jb0);
  const int s_mask = 2 * (idx_mask - kt0);
  // step s_jump is the first one of the second listed range: its rows lie gap_bytes further on
  const int s_jump = 2 * (tile.n_a - kt0);
  const unsigned gap_bytes = (unsigned)(tile.jb0 - tile.n_a) * (64 * D * 2);
  // byte offsets of the rows that step j stages (steps j+2+NS and j+NS), advanced by every step
  // (32 bits: the host admits at most 2^24 keys per request, 2^32 bytes of rows at D = 128)
  unsigned off_k = (unsigned)step_key0(min(2 + NS, last)) * (D * 2);
  unsigned off_v = (unsigned)step_key0(min(NS, last)) * (D * 2);
  int jrel = 0, mrel = 0;                               // s_jump and s_mask relative to the period's first step
  int sj = 0;                                           // j % NS
  auto step = [&](int j, f32x16& s_in, f32x16& s_out, unsigned (&p_in)[8], unsigned (&p_out)[8],
                  auto last_of_pair, auto mode, auto pos) __attribute__((always_inline)) {
    constexpr int MODE = decltype(mode)::value;
    constexpr int SP = decltype(pos)::value;
    constexpr bool ST = SP >= 0;                         // slots known at compile time
    static_assert(!ST || MODE == kSteady, "whole periods run in steady state only");
    constexpr int PH = ST ? (JS + SP) % NS : 0;          // j % NS
    constexpr bool STEADY = MODE == kSteady || MODE == kFill;   // staging from inside the MFMA block
    const bool have1 = ST || !decltype(last_of_pair)::value || j + 1 <= last;
    if (__builtin_expect(ST ? mrel <= 1 + SP : have1 && j + 1 >= s_mask, 0)) apply_mask(s_in, step_key0(j + 1));
    const int slot_ks = ST ? (PH + 2) % NS : sj + 2 >= NS ? sj + 2 - NS : sj + 2;   // (j + 2) % NS
    const bf16x8 pfa = as_bf16x8(make_uint4(p_in[0], p_in[1], p_in[2], p_in[3]));
    const bf16x8 pfb = as_bf16x8(make_uint4(p_in[4], p_in[5], p_in[6], p_in[7]));
    float rs = 0.0f;
    constexpr unsigned SBV = ST ? ((PH + 1) % NS) * SLOT_BYTES : 0, SBK = ST ? ((PH + 3) % NS) * SLOT_BYTES : 0;
    const unsigned sbv = ST ? 0u : (unsigned)slot_v * SLOT_BYTES, sbk = ST ? 0u : (unsigned)slot_k * SLOT_BYTES;
    // The step is 2 KT groups of one MFMA, at most one operand refill and a share of the VALU
    // work, and the issue order is fixed group by group.  (Left to itself the scheduler clusters
    // the MFMAs, and the VALU work then runs while the matrix pipe idles.)  The wave issues in
    // order, so a VALU instruction waiting for its input also holds back the next MFMA: the
    // softmax work of a score is therefore spread over consecutive groups,
    //   exponent argument -> exp2 -> (pair) bf16 pack -> (pair) row-sum dot,
    // each stage one group after the stage it depends on.
    constexpr int NG = 2 * KT, SPG = 16 / NG;          // groups; scores entering per group
    constexpr int HB = KT / 4;                         // k-steps issued before the barrier
    float ea[16], ex[16];                              // exponent arguments, exponentials
    auto v_arg = [&](auto i) {
      constexpr int I = decltype(i)::value;
      if constexpr (I < 16) ea[I] = FOLD ? s_in[I] : __builtin_fmaf(s_in[I], esc, nmref);
    };
    auto v_exp = [&](auto i) {
      constexpr int I = decltype(i)::value;
      if constexpr (I < 16) {
        ex[I] = __builtin_amdgcn_exp2f(ea[I]);
        asm volatile("" :: "v"(ex[I]));                // a use in this group: not sunk to the pack
      }
    };
    auto valu_group = [&](auto g) {                    // the VALU share of group g (g = -1: before)
      constexpr int GI = decltype(g)::value;
      static_for<0, SPG>([&](auto k) {
        constexpr int I = (GI + 1) * SPG + decltype(k)::value;   // exp2 runs one group ahead
        v_exp(std::integral_constant<int, I>{});
        v_arg(std::integral_constant<int, I + SPG>{});
      });
      static_for<0, 8>([&](auto e) {
        constexpr int E = decltype(e)::value;
        constexpr int GC = (2 * E + 1) / SPG;            // group after the pair's second exp2
        if constexpr (GC == GI) p_out[E] = pack_bf16(ex[2 * E], ex[2 * E + 1]);
        if constexpr (GC + 1 == GI)
          rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p_out[E]),
                                               __builtin_bit_cast(bf16x2, 0x3f803f80u), rs, false);
      });
    };
    // n-th staging instruction of this wave for a slot
    auto stage_one = [&](const char* src, unsigned lds0, auto n) {
      constexpr int N = decltype(n)::value;
      const int c = wave_s + N * G;
      if ((CH32 / 64) % G == 0 || c < CH32 / 64) {
        unsigned lo = lane16;
        asm volatile("" : "+v"(lo));
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(src + c * 1024 + lo),
            (__attribute__((address_space(3))) void*)(uintptr_t)(lds0 + c * 1024), 16, 0, 0);
      }
    };
    const char* src_k = nullptr;
    const char* src_v = nullptr;
    src_k = krot_b + off_k;
    src_v = vt_b + off_v;
    {
      // on to the next step: the other half of the key tile, or the first half of the next listed
      // one, which at step s_jump lies gap_bytes further on.  Steps j+2+NS and j+NS have the parity
      // of NS + j; j is even for the first step of a pair.
      constexpr bool ODD = ((NS + (decltype(last_of_pair)::value ? 1 : 0)) & 1) != 0;
      const bool jump_k = ODD && (ST ? jrel == SP + 3 + NS : j + 3 + NS == s_jump);
      const bool jump_v = ODD && (ST ? jrel == SP + 1 + NS : j + 1 + NS == s_jump);
      off_k += HALF + (jump_k ? gap_bytes : 0u);
      off_v += HALF + (jump_v ? gap_bytes : 0u);
    }
    const unsigned lds_ks = smem_base + (unsigned)slot_ks * SLOT_BYTES;
    const unsigned lds_vs = vring + (unsigned)(ST ? PH : sj) * SLOT_BYTES;
    // The 2 NREP staging instructions of this step (K slot first, then V^T slot) are spread evenly
    // over the body groups, the first one in the first group: instruction X goes to group
    // floor(X * BG / (2 NREP)).  (Measured at D = 128, G = 4: four instructions in groups 0, 3, 6, 9
    // of 12 are 1.5 us per launch faster than in groups 0..3, and any later start is slower.)
    constexpr int BG = 2 * (KT - HB);                  // body groups
    auto stage_part2 = [&](auto bg) {
      static_for<0, 2 * NREP>([&](auto x) {
        constexpr int X = decltype(x)::value;
        if constexpr (X * BG / (2 * NREP) == decltype(bg)::value) {
          if constexpr (X < NREP) stage_one(src_k, lds_ks, x);
          else stage_one(src_v, lds_vs, std::integral_constant<int, X - NREP>{});
        }
      });
    };
    auto mfma_pv = [&](auto t) {
      constexpr int T = decltype(t)::value;
      constexpr int uu = T / DB, db = T % DB;
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[uu][db], uu ? pfb : pfa, o[db], 0, 0, 0);
    };
    auto mfma_qk = [&](auto t) {
      constexpr int T = decltype(t)::value;
      if constexpr (T == 0 && FOLD) {
        s_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], cref, 0, 0, 0);
      } else {
        if constexpr (T == 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s_out[r] = 0.0f;   // becomes the constant-zero accumulator input
        }
        s_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], s_out, 0, 0, 0);
      }
    };
    auto wait_operand = [&](bf16x8& r, auto n) {
      constexpr int N = decltype(n)::value;
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r) : "n"(N));
    };
    auto refill_v = [&](auto t) {
      constexpr int T = decltype(t)::value;
      constexpr int uu = T / DB, db = T % DB;
      lds_refill_b128<(uu * 2 * D + db * 32) * 16 + SBV>(vf[uu][db], v_off + sbv);
    };
    auto refill_k = [&](auto t) {
      constexpr int T = decltype(t)::value;
      lds_refill_b128<T * 1024 + SBK>(kf[t], k_off + sbk);
    };

    static_for<0, SPG>([&](auto k) { v_arg(k); });
    valu_group(std::integral_constant<int, -1>{});
    __builtin_amdgcn_sched_barrier(0);
    // Head: the first MFMAs need nothing from LDS, so they are issued before the barrier and run
    // while this wave waits for the staging loads and for the other waves.
    static_for<0, HB>([&](auto t) {
      constexpr int T = decltype(t)::value;
      // LDS reads land in order: the operand read as number x of the previous step's 16 is there
      // once at most 15 - x younger reads are outstanding
      wait_operand(vf[T / DB][T % DB], std::integral_constant<int, 2 * KT - 1 - 2 * T>{});
      mfma_pv(t);
      valu_group(std::integral_constant<int, 2 * T>{});
      __builtin_amdgcn_sched_barrier(0);
      wait_operand(kf[T], std::integral_constant<int, 2 * KT - 2 - 2 * T>{});
      mfma_qk(t);
      valu_group(std::integral_constant<int, 2 * T + 1>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    wait_kv();                                         // all reads of the previous step are done
    // Every wave is past the operand reads of the previous step: its V^T slot (step j) and K slot
    // (step j+2) can be refilled.  Steps up to j+3 (K) and j+1 (V^T) must be visible; everything
    // issued after them may stay in flight:
    //   K(j+4) .. K(j+1+NS) and V^T(j+2) .. V^T(j+NS-1), as far as they exist and were issued.
    if constexpr (MODE == kSteady && (2 * NS - 4) * HPW + 2 * NREP <= 63) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((2 * NS - 4) * HPW));
    } else if constexpr (MODE == kDrain) {
      __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
    } else {
      const int cnt_k = min(NS - 2, j + 2), cnt_v = min(NS - 2, j);
      const int none_k = min(max(j + 1 + NS - last, 0), cnt_k);
      const int none_v = min(max(j + NS - 1 - last, 0), cnt_v);
      wait_slots(std::integral_constant<int, 2 * NS - 4>{}, cnt_k - none_k + cnt_v - none_v);
    }
    __builtin_amdgcn_s_barrier();
    if constexpr (MODE == kGeneric || MODE == kPartial) {
      if (j + 2 + NS <= last) stage_slot(src_k, lds_ks);
      if (j + NS <= last) stage_slot(src_v, lds_vs);
    }
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, HB>([&](auto t) { refill_v(t); refill_k(t); });
    __builtin_amdgcn_sched_barrier(0);
    // Body: every MFMA is followed by the refill of its operand; in steady state the staging
    // instructions of this step are spread over the groups, K first.
    static_for<HB, KT>([&](auto t) {
      constexpr int T = decltype(t)::value;
      constexpr int R = T - HB;                        // 0, 1, ...
      mfma_pv(t);
      __builtin_amdgcn_sched_barrier(0);               // the MFMA first, its group's other work behind it
      refill_v(t);
      valu_group(std::integral_constant<int, 2 * T>{});
      if constexpr (STEADY) stage_part2(std::integral_constant<int, 2 * R>{});
      __builtin_amdgcn_sched_barrier(0);
      mfma_qk(t);
      __builtin_amdgcn_sched_barrier(0);
      refill_k(t);
      valu_group(std::integral_constant<int, 2 * T + 1>{});
      if constexpr (STEADY) stage_part2(std::integral_constant<int, 2 * R + 1>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    valu_group(std::integral_constant<int, NG>{});     // what is left: the last row-sum term
    asm volatile("" : "+v"(rs));                      // the row sum belongs to this block
    __builtin_amdgcn_sched_barrier(0);
    if (have1) {
      if (__builtin_expect(out_of_window(rs), 0)) rs = recentre(s_in, p_out, s_out);
      l_run += rs;
    }
    if constexpr (!ST) {     // (a whole period leaves them as they are)
      slot_v = (j + 2 <= last) ? (slot_v + 1 == NS ? 0 : slot_v + 1) : slot_v;
      slot_k = (j + 4 <= last) ? (slot_k + 1 == NS ? 0 : slot_k + 1) : slot_k;
      sj = sj + 1 == NS ? 0 : sj + 1;
    }
  };
  // Loops over pairs of steps: filling the pipeline (j < JS), steady state (the pipeline is full,
  // j >= NS - 2, and step j + 1 still refills a K slot, j + 3 + NS <= last), the few steps in which
  // some but not all refills are left, and draining (nothing left to stage).  An item long enough
  // to reach steady state fills with the staging inside the MFMA block as well.
  auto pair_of_steps = [&](int j, auto mode) __attribute__((always_inline)) {
    step(j, sB, sA, pA, pB, std::false_type{}, mode, std::integral_constant<int, -1>{});
    step(j + 1, sA, sB, pB, pA, std::true_type{}, mode, std::integral_constant<int, -1>{});
  };
  int j = 0;
  if (JS + 3 + NS <= last) {
#pragma nounroll
    for (; j < JS; j += 2) pair_of_steps(j, std::integral_constant<int, kFill>{});
  }
  for (; j < n_steps && j < JS; j += 2) pair_of_steps(j, std::integral_constant<int, kGeneric>{});
  if (j == JS && j + 2 * PP + 1 + NS <= last) {          // whole periods of the slot rotation
    do {
      jrel = s_jump - j;
      mrel = s_mask - j;
      static_for<0, PP>([&](auto p) __attribute__((always_inline)) {
        constexpr int P2 = 2 * decltype(p)::value;
        step(j + P2, sB, sA, pA, pB, std::false_type{}, std::integral_constant<int, kSteady>{},
             std::integral_constant<int, P2>{});
        step(j + P2 + 1, sA, sB, pB, pA, std::true_type{}, std::integral_constant<int, kSteady>{},
             std::integral_constant<int, P2 + 1>{});
      });
      j += 2 * PP;
    } while (j + 2 * PP + 1 + NS <= last);
  }
  for (; j + 3 + NS <= last; j += 2) pair_of_steps(j, std::integral_constant<int, kSteady>{});
  for (; j < n_steps && j + NS <= last; j += 2) pair_of_steps(j, std::integral_constant<int, kPartial>{});
  for (; j < n_steps; j += 2) pair_of_steps(j, std::integral_constant<int, kDrain>{});
  wait_kv();

  // ---- epilogue: normalise, then transpose through LDS so that every output row leaves as one
  // contiguous run (2 D bytes in bf16; fp32 goes in two halves of D/2 features to bound the area)
  const float l_tot = pair_sum(l_run);
  __syncthreads();                                    // every wave is done with the stages
  {
    const bool partial = split > 1;                   // this piece's result goes to the workspace
    const float inv = partial ? 1.0f : 1.0f / l_tot;
    const int64_t tok0 = (int64_t)mine.tok_base + mine.t0;
    // rows with few visible keys are produced in fp32 by the preparation kernel: not stored here
    // (lane r < 32 holds the descriptor of row r: one ballot gives the row mask to every lane);
    // the segment-only call stores segment rows only (b_start > 0 marks them)
    const unsigned stored_rows = (unsigned)__builtin_amdgcn_ballot_w64(
        valid && a_end + own_row() - b_start + 1 > PV_SHORT_ROW_KEYS && (split == 0 || b_start > 0));
    auto stored = [&](int row) { return partial || ((stored_rows >> row) & 1u) != 0; };
    constexpr int RS = 2 * D + 16;                    // row stride: 16 B of padding spreads the banks
    char* tr = reinterpret_cast<char*>(&smem[0]) + (size_t)wave * (32 * RS);
    // where row `row` of this wave's result goes, as fp32: the caller's tensor, or the partial tile
    auto f32_row = [&](int row) {
      return partial ? part_o + row * D
                     : reinterpret_cast<float*>(out) + (caller_row(plan, h, tok0 + row) * hq + head) * D;
    };
    if (partial && hh == 0) reinterpret_cast<float2*>(part_o + 32 * D)[qrow] = make_float2(nmref, l_tot);
    if (out_f32 || partial) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int dbh = 0; dbh < DB / 2; ++dbh)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const int db = half * (DB / 2) + dbh;
            const float4 w = make_float4(o[db][4 * gq] * inv, o[db][4 * gq + 1] * inv,
                                         o[db][4 * gq + 2] * inv, o[db][4 * gq + 3] * inv);
            *reinterpret_cast<float4*>(tr + qrow * RS + (dbh * 32 + 8 * gq + 4 * hh) * 4) = w;
          }
        constexpr int LPR = D / 8;                    // lanes per row: D/2 floats = 2 D bytes
#pragma unroll
        for (int it = 0; it < 32 * LPR / 64; ++it) {
          const int row = it * (64 / LPR) + lane / LPR, c = lane % LPR;
          const float4 w = *reinterpret_cast<const float4*>(tr + row * RS + c * 16);
          if (stored(row)) *reinterpret_cast<float4*>(f32_row(row) + half * (D / 2) + c * 4) = w;
        }
      }
    } else {
      uint16_t* op = reinterpret_cast<uint16_t*>(out);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          uint2 w;
          w.x = pack_bf16(o[db][4 * gq] * inv, o[db][4 * gq + 1] * inv);
          w.y = pack_bf16(o[db][4 * gq + 2] * inv, o[db][4 * gq + 3] * inv);
          *reinterpret_cast<uint2*>(tr + qrow * RS + (db * 32 + 8 * gq + 4 * hh) * 2) = w;
        }
      constexpr int LPR = D / 8;                      // lanes per row: 2 D bytes in 16-byte pieces
#pragma unroll
      for (int it = 0; it < 32 * LPR / 64; ++it) {
        const int row = it * (64 / LPR) + lane / LPR, c = lane % LPR;
        const uint4 w = *reinterpret_cast<const uint4*>(tr + row * RS + c * 16);
        if (stored(row))
          *reinterpret_cast<uint4*>(op + (caller_row(plan, h, tok0 + row) * hq + head) * D + c * 8) = w;
      }
    }
    if (lse && !partial && hh == 0 && stored(qrow))
      lse[(int64_t)head * h.total_tokens + caller_row(plan, h, g)] =
          (log2f(l_tot) - nmref) * 0.6931471805599453f;
  }
}

template <int D, int G>
hipError_t launch_main(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                              const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                              float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                              int split, float* part, const KvSource& raw_kv, float scale, int n_short,
                              hipStream_t s) {
  dim3 grid;
  const int64_t blocks = (split ? (int64_t)h.n_seg_tiles * hkv * split : (int64_t)h.n_q_tiles * hkv) + n_short;
  if (!grid_1d(blocks, G * 64, &grid)) return hipErrorInvalidConfiguration;
  if (rope)
    k_attn_bf16<D, G, true><<<grid, dim3(G * 64), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                          qscale, rope, out_f32, split, part, raw_kv, scale,
                                                          n_short);
  else
    k_attn_bf16<D, G, false><<<grid, dim3(G * 64), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                           qscale, rope, out_f32, split, part, raw_kv, scale,
                                                           n_short);
  return hipGetLastError();
}

// Workgroups of four query tiles of one head (see QT above): one per (group of tiles, query head).
template <int D>
hipError_t launch_query_tiles(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                                     const uint16_t* krot, const uint16_t* vt, const float2* cs,
                                     void* out, float* lse, int hq, int hkv, float qscale, bool rope,
                                     bool out_f32, const KvSource& raw_kv, float scale, int n_short,
                                     hipStream_t s) {
  dim3 grid;
  if (!grid_1d((int64_t)h.n_quads * hq + n_short, 256, &grid)) return hipErrorInvalidConfiguration;
  if (rope)
    k_attn_bf16<D, 4, true, true><<<grid, dim3(256), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                             qscale, rope, out_f32, 0, nullptr, raw_kv, scale,
                                                             n_short);
  else
    k_attn_bf16<D, 4, false, true><<<grid, dim3(256), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                              qscale, rope, out_f32, 0, nullptr, raw_kv, scale,
                                                              n_short);
  return hipGetLastError();
}


}  // namespace pv
#endif
