// Main attention kernel for head_dim 128 and an even GQA group (4 or 8 query heads per kv head).
//
// Why this shape.  Every MFMA of the generic kernel needs one fresh 1 KB operand from LDS, and
// with eight 32-row waves per CU the LDS (reads plus the global->LDS staging writes) saturates
// long before the matrix pipe does.  Here a wave owns TWO 32-row blocks (two query heads of the
// same 32 tokens), so every K and V^T operand read from LDS feeds two MFMAs, and the workgroup
// runs one wave per SIMD with the full 512-register budget.
//
//   workgroup = one query tile (32 tokens) x one kv head, 4 waves
//   wave      = head pair hp (heads 2hp, 2hp+1 of the group) x key group ks
//   key split = with 4 heads per group there are only two head pairs, so the four waves form two
//               key groups that take alternate 32-key steps and merge their (O, l, reference)
//               at the end through LDS.  This also halves the serial length of the longest
//               work item, which matters when a problem has few, long items.
//
// Each key group runs a software pipeline over its steps i (32 keys each).  Iteration i issues,
// as ONE block of 32 MFMAs, S^T of step i+2 and O^T += V^T P^T of step i, while the VALU forms
// the probabilities of step i+1; the LDS reads of the operands for the next iteration (K of step
// i+3, V^T of step i+1) are issued between those MFMAs, as soon as the register they overwrite
// has been consumed.  K/V stages arrive by direct global->LDS loads, NSG stages per key group.
#include "pv_attn_common.h"

namespace pv {

namespace {

constexpr int D = 128;
constexpr int KT = 8;             // MFMA k-steps over the feature dim (S^T) = V^T operands per step
constexpr int DB = 4;             // 32-feature blocks of O^T
constexpr int CPR = 16;           // 16-byte chunks per key row
constexpr int CH32 = 512;         // chunks per 32-key K (or V^T) stage half
constexpr unsigned STAGE_BYTES = 2 * CH32 * 16;

// s_waitcnt lgkmcnt(n) tied to the operand it makes valid.  LDS reads complete in order, and in
// the steady-state block every operand is needed when exactly 15 younger reads may be outstanding
// (16 per block, issued V^T 0..7 then K 0..7, consumed in the same order one block later).
#define PV_WAIT_ONE(n, a) asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+a"(a))

// 16-byte LDS read into accumulation registers (AGPRs): the K and V^T operands are only ever
// touched by ds_read and MFMA, so they stay out of the VGPR file that the VALU work needs.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128_acc(unsigned addr) {
  bf16x8 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=a"(r) : "v"(addr), "n"(OFF));
  return r;
}

template <int HP, int KS, bool FOLD>
__global__ __launch_bounds__(256, 1) void k_attn_m64(
    const int32_t* __restrict__ plan, PlanHeader h, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ krot, const uint16_t* __restrict__ vt,
    const float2* __restrict__ cs, void* __restrict__ out, float* __restrict__ lse, int hq, int hkv,
    float qscale, bool out_f32) {
  static_assert(HP * KS == 4, "four waves, one per SIMD");
  constexpr int G = 2 * HP;
  constexpr int NSG = (KS == 2) ? 5 : 8;              // LDS stages per key group
  constexpr int NREP = 8 / HP;                        // staging instructions per wave, K and V each
  constexpr int LPS = 2 * NREP;                       // staging loads a wave issues per stage
  // One LDS array on purpose (several LDS variables make the compiler serialise LDS reads behind
  // all outstanding global->LDS loads); ordering is enforced with explicit waits and barriers.
  __shared__ uint4 smem[KS][NSG][2][CH32];

  const int kvh = blockIdx.x % hkv;
  const QTile tile = reinterpret_cast<const QTile*>(plan + h.off_work)[blockIdx.x / hkv];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hp = wave % HP, ks = wave / HP;
  const int qrow = lane & 31, hh = lane >> 5;
  const bool valid = qrow < tile.rows;
  const int64_t g = (int64_t)tile.tok_base + tile.t0 + qrow;
  const int i_loc = valid ? tile.t0 + qrow : -1;
  int a_end = 0, b_start = 0;
  if (valid) { a_end = plan[h.off_aend + g]; b_start = plan[h.off_bstart + g]; }
  const int head0 = kvh * G + 2 * hp;                 // heads of the two row blocks: head0, head0+1

  bf16x8 qf[2][KT];      // Q operands of the two row blocks (filled below, once the tile is in LDS)

  // ---- steps.  A key tile of the plan (64 keys) is two steps of 32 keys; tiles run over
  // [0, n_a) then [jb0, jb1).  Key group ks owns the global steps i*KS + ks, i = 0..n_i-1.
  const int n_tiles = tile.n_a + (tile.jb1 - tile.jb0);
  const int n_steps = 2 * n_tiles;
  const int n_i = n_steps / KS;                       // n_steps is even, KS is 1 or 2
  const int last = n_i - 1;
  auto step_key0 = [&](int i) {                       // first key (request-local) of local step i
    const int j = i * KS + ks;
    const int idx = j >> 1;
    const int jt = idx < tile.n_a ? idx : tile.jb0 + (idx - tile.n_a);
    return jt * 64 + (j & 1) * 32;
  };
  const int64_t head_base = ((int64_t)kvh * h.padded_keys + tile.kpad_base) * D;   // elements

  // ---- staging: scalar bases, per-lane offsets (the K bank swizzle, chunk pos ^ row within each
  // 256-byte row, is applied by choosing which global chunk a lane fetches)
  unsigned gk_off[NREP], gv_off[NREP];
#pragma unroll
  for (int n = 0; n < NREP; ++n) {
    const int P = (hp + n * HP) * 64 + lane;
    const int R = P >> 4, pos = P & 15;
    gk_off[n] = (unsigned)(((R << 4) + (pos ^ (R & 15))) * 16);
    gv_off[n] = (unsigned)(P * 16);
  }
  const unsigned smem_base =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)(char*)&smem[0][0][0][0];
  const unsigned group_base = smem_base + (unsigned)ks * (NSG * STAGE_BYTES);
  const char* krot_b = reinterpret_cast<const char*>(krot) + head_base * 2;
  const char* vt_b = reinterpret_cast<const char*>(vt) + head_base * 2;
  auto stage = [&](int i, int buf) {
    if (i > last) return;
    const int64_t off = (int64_t)step_key0(i) * (D * 2);
    const char* gk = krot_b + off;
    const char* gv = vt_b + off;
    const unsigned lds0 = group_base + (unsigned)buf * STAGE_BYTES;
#pragma unroll
    for (int n = 0; n < NREP; ++n) {
      const int c = hp + n * HP;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(gk + gk_off[n]),
          (__attribute__((address_space(3))) void*)(uintptr_t)(lds0 + c * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(gv + gv_off[n]),
          (__attribute__((address_space(3))) void*)(uintptr_t)(lds0 + CH32 * 16 + c * 1024), 16, 0, 0);
    }
  };

  // ---- LDS operand reads (inline assembly, see lds_read_b128)
  bf16x8 kf[KT];          // K operand x of the next S^T (8 features-of-16 slices of 32 keys)
  bf16x8 vf[KT];          // V^T operand x = (slab uu = x / 4, feature block db = x % 4)
  unsigned k_off[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const int L = qrow * CPR + 2 * t + hh;
    const int R = L >> 4, pos = L & 15;
    k_off[t] = group_base + (unsigned)(((R << 4) + (pos ^ (R & 15))) * 16);
  }
  const unsigned v_off = group_base + (unsigned)((CH32 + hh * D + qrow) * 16);
  auto read_k1 = [&](auto x, int buf) { kf[x] = lds_read_b128_acc<0>(k_off[x] + (unsigned)buf * STAGE_BYTES); };
  auto read_v1 = [&](auto x, int buf) {
    constexpr int uu = decltype(x)::value / DB, db = decltype(x)::value % DB;
    vf[x] = lds_read_b128_acc<(uu * 2 * D + db * 32) * 16>(v_off + (unsigned)buf * STAGE_BYTES);
  };
  auto wait_all = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+a"(kf[0]), "+a"(kf[1]), "+a"(kf[2]), "+a"(kf[3]), "+a"(kf[4]), "+a"(kf[5]),
                   "+a"(kf[6]), "+a"(kf[7]), "+a"(vf[0]), "+a"(vf[1]), "+a"(vf[2]), "+a"(vf[3]),
                   "+a"(vf[4]), "+a"(vf[5]), "+a"(vf[6]), "+a"(vf[7]));
  };

  // ---- softmax state per row block.  p = 2^(esc * (s - mref)); the reference mref is NOT the
  // running maximum: it is only re-centred when a row sum leaves a safe window, so the common path
  // has no max reduction and no rescaling of O.  l_run and o are relative to mref.
  f32x16 o[2][DB];
  float mref[2] = {0.0f, 0.0f}, l_run[2] = {0.0f, 0.0f};
#pragma unroll
  for (int b = 0; b < 2; ++b) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[b][db][r] = 0.0f;
  }
  const float esc = FOLD ? 1.0f : qscale;   // exponent scale: p = 2^(esc * (s - mref))
  auto prob = [&](float x, float m) { return __builtin_amdgcn_exp2f(FOLD ? x - m : (x - m) * esc); };
  auto apply_mask = [&](f32x16& sc, int key0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = key0 + 8 * (r / 4) + 4 * hh + (r % 4);
      const bool vis = (key < a_end) | ((key >= b_start) & (key <= i_loc));   // branch-free
      sc[r] = vis ? sc[r] : -INFINITY;
    }
  };
  // p rounded to bf16 once; the row sum is taken over the rounded values (v_dot2c with a pair of
  // ones), so that O is an exact convex combination of V rows with the weights the MFMA sees
  auto probs = [&](const f32x16& sc, float m, unsigned (&pw)[8]) {
    float rs = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pw[e] = pack_bf16(prob(sc[2 * e], m), prob(sc[2 * e + 1], m));
      rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[e]),
                                           __builtin_bit_cast(bf16x2, 0x3f803f80u), rs, false);
    }
    return rs;
  };
  auto out_of_window = [&](float rs) { return !(rs >= 0x1p-40f && rs <= 0x1p40f); };
  // One exact online-softmax step of row block b for the whole wave: taken when a partial row sum
  // is outside [2^-40, 2^40] (also catches inf/NaN/0).  Rare: first steps of a row, masked steps
  // with no visible key, or scores drifting by more than 40 octaves.  The reference moves to this
  // step's row maximum, but never so far down that the history (l, O) would leave fp32 range:
  // delta >= log2(l) - 20.  Both half-waves of a row take identical decisions.
  auto recentre = [&](int b, const f32x16& sc, unsigned (&pw)[8]) {
    float mx = sc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
    mx = pair_max(mx) - mref[b];                // relative to the current reference
    const float l_tot = pair_sum(l_run[b]);
    if (mx > -INFINITY && mx < INFINITY) {      // rows with no visible key keep their reference
      float delta = mx, alpha = 0.0f;           // empty history: nothing to rescale
      if (l_tot > 0.0f) {
        delta = fmaxf(mx, (__builtin_amdgcn_logf(l_tot) - 20.0f) / esc);
        alpha = __builtin_amdgcn_exp2f(-delta * esc);
      }
      mref[b] += delta;
      l_run[b] *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][db][r] *= alpha;
    }
    return probs(sc, mref[b], pw);
  };
  auto qk_both = [&](f32x16 (&acc)[2]) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[0][t], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[1][t], acc[1], 0, 0, 0);
    }
  };

  // ---- Q tile (and its cos/sin rows) through LDS.  A lane needs 16-byte pieces of 32 different
  // rows, which as direct global loads is one cache line per lane; instead the four waves copy
  // whole rows with global->LDS loads (swizzled like K) into stages 3.. that the K/V pipeline does
  // not need yet, while stages 0..2 are being filled.
  constexpr unsigned Q_AREA = 3 * STAGE_BYTES;
  constexpr unsigned CS_AREA = (KS == 2) ? (NSG + 3) * STAGE_BYTES : Q_AREA + G * 32 * 256;
  {
    const int rows_m1 = tile.rows - 1;
    const int64_t tok0 = (int64_t)tile.tok_base + tile.t0;
    // Q: G*32 rows of 16 chunks; one instruction = 64 chunks = 4 rows; 8*G instructions in all
#pragma unroll
    for (int n = 0; n < 2 * G; ++n) {
      const int P = (wave + 4 * n) * 64 + lane;
      const int r = P >> 4, pos = P & 15;
      const int hl = r >> 5, tok = min(r & 31, rows_m1);
      const uint16_t* src = q + ((tok0 + tok) * hq + kvh * G + hl) * D + ((pos ^ (r & 15)) << 3);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)src,
          (__attribute__((address_space(3))) void*)(uintptr_t)(smem_base + Q_AREA + (wave + 4 * n) * 1024),
          16, 0, 0);
    }
    if (FOLD) {   // rotary table rows: 32 tokens x 32 chunks (64 float2)
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const int P = (wave + 4 * n) * 64 + lane;
        const int tok = P >> 5, pos = P & 31;
        const float2* src = cs + (tok0 + min(tok, rows_m1)) * (D / 2) + ((pos ^ (tok & 15)) << 1);
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)src,
            (__attribute__((address_space(3))) void*)(uintptr_t)(smem_base + CS_AREA + (wave + 4 * n) * 1024),
            16, 0, 0);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 3; ++i) stage(i, i);
  // own Q / table loads have landed (they are older than the 3 stages just issued, if all 3 exist)
  if (n_i >= 3) __builtin_amdgcn_s_waitcnt(vmcnt_imm(3 * LPS));
  else __builtin_amdgcn_s_waitcnt(0x0f70);
  __builtin_amdgcn_s_barrier();                          // ... and everyone else's
  {
    const uint4* q_lds = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(&smem[0][0][0][0]) + Q_AREA);
    const uint4* cs_lds = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(&smem[0][0][0][0]) + CS_AREA);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      float x[KT][8];
      const int r = (2 * hp + b) * 32 + qrow;
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        const uint4 raw = q_lds[(r << 4) + ((2 * t + hh) ^ (r & 15))];
        const unsigned* pr = reinterpret_cast<const unsigned*>(&raw);
#pragma unroll
        for (int e = 0; e < 4; ++e) { x[t][2 * e] = bf16_lo(pr[e]); x[t][2 * e + 1] = bf16_hi(pr[e]); }
      }
      if (FOLD) {          // FOLD <=> rotary embedding on: pair (c, c + D/2), c = 16 t + 8 hh + e
#pragma unroll
        for (int t = 0; t < KT / 2; ++t) {
#pragma unroll
          for (int k2 = 0; k2 < 4; ++k2) {
            const uint4 w = cs_lds[(qrow << 5) + ((8 * t + 4 * hh + k2) ^ (qrow & 15))];
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
        qf[b][t] = as_bf16x8(pk);
      }
    }
  }
  __syncthreads();                                       // the Q area may now be overwritten
#pragma unroll
  for (int i = 3; i < NSG; ++i) stage(i, i);
  if (n_i >= NSG) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSG - 3) * LPS));  // stages 0..2 have landed
  else __builtin_amdgcn_s_waitcnt(0x0f70);
  __builtin_amdgcn_s_barrier();

  // ---- pipeline prologue: P(0), S(1), K operand of step 2, V^T operand of step 0
  static_for<0, KT>([&](auto x) { read_k1(x, 0); });
  wait_all();
  f32x16 s0[2], s1[2];
  qk_both(s0);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, KT>([&](auto x) { read_k1(x, min(1, last) % NSG); });
  if (step_key0(0) >= tile.n_full * 64) { apply_mask(s0[0], step_key0(0)); apply_mask(s0[1], step_key0(0)); }
  unsigned p0[2][8];
  float rs0[2];
  rs0[0] = probs(s0[0], mref[0], p0[0]);
  rs0[1] = probs(s0[1], mref[1], p0[1]);
  wait_all();
  qk_both(s1);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, KT>([&](auto x) { read_v1(x, 0); });
  static_for<0, KT>([&](auto x) { read_k1(x, min(2, last) % NSG); });
  if (__builtin_amdgcn_ballot_w64(out_of_window(rs0[0]) | out_of_window(rs0[1])) != 0) {
    rs0[0] = recentre(0, s0[0], p0[0]);
    rs0[1] = recentre(1, s0[1], p0[1]);
  }
  l_run[0] += rs0[0];
  l_run[1] += rs0[1];
  // LDS stage of step i+1 (b1), of step i+3 (b3) and the stage freed by step i (bs = i % NSG)
  int b1 = min(1, last) % NSG, b3 = min(3, last) % NSG, bs = 0;

  for (int i = 0; i < n_i; ++i) {
    // After the barrier stage i % NSG is free (its reads were issued in earlier iterations and
    // are waited for inside the previous block) and steps <= i+3 must be visible: up to NSG-4
    // newer stages may stay in flight.
    {
      const int newer = min(i + NSG - 1, last) - (i + 3);
      if (newer >= NSG - 4) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSG - 4) * LPS));
      else __builtin_amdgcn_s_waitcnt(0x0f70);
    }
    // the V^T reads of step i (the older 8 of the 16 outstanding) must have left the stage that
    // is refilled below; the younger K reads touch other stages
    asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    stage(i + NSG, bs);
    const bool have1 = i + 1 <= last;
    if (have1) {
      const int key0 = step_key0(i + 1);
      if (key0 >= tile.n_full * 64) { apply_mask(s1[0], key0); apply_mask(s1[1], key0); }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- one block of 32 MFMAs: O^T += V^T P^T of step i and S^T of step i+2, both row blocks;
    // probabilities of step i+1 on the VALU; operand reads for the next iteration in between.
    f32x16 s2[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) s2[b][r] = 0.0f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      pf[b][0] = as_bf16x8(make_uint4(p0[b][0], p0[b][1], p0[b][2], p0[b][3]));
      pf[b][1] = as_bf16x8(make_uint4(p0[b][4], p0[b][5], p0[b][6], p0[b][7]));
    }
    unsigned p1[2][8];
    float rs1[2] = {0.0f, 0.0f};
    // first half: the 16 P V MFMAs; each V^T register is refilled (step i+1) once consumed; the
    // probabilities of row block 0 are formed meanwhile
    static_for<0, KT>([&](auto x) {
      constexpr int uu = decltype(x)::value / DB, db = decltype(x)::value % DB;
      PV_WAIT_ONE(15, vf[x]);
      o[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[x], pf[0][uu], o[0][db], 0, 0, 0);
      o[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[x], pf[1][uu], o[1][db], 0, 0, 0);
      read_v1(x, b1);
      p1[0][x] = pack_bf16(prob(s1[0][2 * x], mref[0]), prob(s1[0][2 * x + 1], mref[0]));
      rs1[0] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p1[0][x]),
                                               __builtin_bit_cast(bf16x2, 0x3f803f80u), rs1[0], false);
    });
    // second half: the 16 Q K^T MFMAs (two alternating accumulator chains); K registers are
    // refilled (step i+3); probabilities of row block 1
    static_for<0, KT>([&](auto x) {
      PV_WAIT_ONE(15, kf[x]);
      s2[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[x], qf[0][x], s2[0], 0, 0, 0);
      s2[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[x], qf[1][x], s2[1], 0, 0, 0);
      read_k1(x, b3);
      p1[1][x] = pack_bf16(prob(s1[1][2 * x], mref[1]), prob(s1[1][2 * x + 1], mref[1]));
      rs1[1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p1[1][x]),
                                               __builtin_bit_cast(bf16x2, 0x3f803f80u), rs1[1], false);
    });
    __builtin_amdgcn_sched_barrier(0);
    if (have1) {
      if (__builtin_amdgcn_ballot_w64(out_of_window(rs1[0]) | out_of_window(rs1[1])) != 0) {
        rs1[0] = recentre(0, s1[0], p1[0]);
        rs1[1] = recentre(1, s1[1], p1[1]);
      }
      l_run[0] += rs1[0];
      l_run[1] += rs1[1];
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      s1[b] = s2[b];
#pragma unroll
      for (int e = 0; e < 8; ++e) p0[b][e] = p1[b][e];
    }
    bs = bs + 1 == NSG ? 0 : bs + 1;
    b1 = (i + 2 <= last) ? (b1 + 1 == NSG ? 0 : b1 + 1) : b1;
    b3 = (i + 4 <= last) ? (b3 + 1 == NSG ? 0 : b3 + 1) : b3;
  }
  wait_all();

  // ---- merge the key groups (KS == 2): group 1 hands (O, mref, l) to group 0 through LDS
  float l_tot[2] = {pair_sum(l_run[0]), pair_sum(l_run[1])};
  if constexpr (KS == 2) {
    __syncthreads();                                   // every wave is done with the stages
    float* xch = reinterpret_cast<float*>(&smem[0][0][0][0]) + (size_t)hp * (2 * (DB * 16 + 2) * 64);
    if (ks == 1) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float* dst = xch + b * (DB * 16 + 2) * 64 + lane;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[(db * 16 + r) * 64] = o[b][db][r];
        dst[(DB * 16) * 64] = mref[b];
        dst[(DB * 16 + 1) * 64] = l_tot[b];
      }
    }
    __syncthreads();
    if (ks == 1) return;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const float* src = xch + b * (DB * 16 + 2) * 64 + lane;
      const float m1 = src[(DB * 16) * 64], l1 = src[(DB * 16 + 1) * 64];
      // weights relative to the larger reference; an empty side (l = 0) gets weight 0
      const float ma = l_tot[b] > 0.0f ? mref[b] : -INFINITY;
      const float mb = l1 > 0.0f ? m1 : -INFINITY;
      const float m = fmaxf(ma, mb);
      const float wa = l_tot[b] > 0.0f ? __builtin_amdgcn_exp2f((ma - m) * esc) : 0.0f;
      const float wb = l1 > 0.0f ? __builtin_amdgcn_exp2f((mb - m) * esc) : 0.0f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][db][r] = o[b][db][r] * wa + src[(db * 16 + r) * 64] * wb;
      l_tot[b] = l_tot[b] * wa + l1 * wb;
      mref[b] = m;
    }
  }

  // ---- epilogue: normalise, then transpose each row block through LDS so that every output
  // row leaves as one contiguous 256-byte (bf16) or 512-byte (fp32) run
  if constexpr (KS == 1) __syncthreads();              // every wave is done with the stages
  // per-wave transposition area (32 rows x 528 B); with the key split it sits above the merge area
  char* tr = reinterpret_cast<char*>(&smem[0][0][0][0]) + (KS == 2 ? 96 * 1024 : 0) + (size_t)wave * (32 * 528);
  const int64_t tok0 = (int64_t)tile.tok_base + tile.t0;
  // rows with few visible keys are produced in fp32 by the preparation kernel: not stored here
  auto stored = [&](int row) {
    if (row >= tile.rows) return false;
    const int64_t gg = tok0 + row;
    const int cnt = plan[h.off_aend + gg] + (tile.t0 + row) - plan[h.off_bstart + gg] + 1;
    return cnt > PV_SHORT_ROW_KEYS;
  };
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const float inv = 1.0f / l_tot[b];
    const int head = head0 + b;
    if (out_f32) {
      // row stride 528 B (512 + 16): the 32 lanes of a half-wave hit distinct banks
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const float4 w = make_float4(o[b][db][4 * gq] * inv, o[b][db][4 * gq + 1] * inv,
                                       o[b][db][4 * gq + 2] * inv, o[b][db][4 * gq + 3] * inv);
          *reinterpret_cast<float4*>(tr + qrow * 528 + (db * 32 + 8 * gq + 4 * hh) * 4) = w;
        }
      float* op = reinterpret_cast<float*>(out);
#pragma unroll
      for (int it = 0; it < 16; ++it) {                // 2 rows per instruction, 32 lanes x 16 B per row
        const int row = 2 * it + (lane >> 5), c = lane & 31;
        const float4 w = *reinterpret_cast<const float4*>(tr + row * 528 + c * 16);
        if (stored(row)) *reinterpret_cast<float4*>(op + ((tok0 + row) * hq + head) * D + c * 4) = w;
      }
    } else {
      // row stride 264 B (256 + 8)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          uint2 w;
          w.x = pack_bf16(o[b][db][4 * gq] * inv, o[b][db][4 * gq + 1] * inv);
          w.y = pack_bf16(o[b][db][4 * gq + 2] * inv, o[b][db][4 * gq + 3] * inv);
          *reinterpret_cast<uint2*>(tr + qrow * 264 + (db * 32 + 8 * gq + 4 * hh) * 2) = w;
        }
      uint16_t* op = reinterpret_cast<uint16_t*>(out);
#pragma unroll
      for (int it = 0; it < 8; ++it) {                 // 4 rows per instruction, 16 lanes x 16 B per row
        const int row = 4 * it + (lane >> 4), c = lane & 15;
        // 264-byte rows are only 8-byte aligned: read the 16 bytes as two 8-byte halves
        const uint2 w0 = *reinterpret_cast<const uint2*>(tr + row * 264 + c * 16);
        const uint2 w1 = *reinterpret_cast<const uint2*>(tr + row * 264 + c * 16 + 8);
        if (stored(row))
          *reinterpret_cast<uint4*>(op + ((tok0 + row) * hq + head) * D + c * 8) = make_uint4(w0.x, w0.y, w1.x, w1.y);
      }
    }
    if (lse && hh == 0 && valid && a_end + i_loc - b_start + 1 > PV_SHORT_ROW_KEYS)
      lse[(int64_t)head * h.total_tokens + g] = (mref[b] * esc + log2f(l_tot[b])) * 0.6931471805599453f;
  }
}

template <int HP, int KS>
hipError_t launch(const int32_t* plan, const PlanHeader& h, const uint16_t* q, const uint16_t* krot,
                  const uint16_t* vt, const float2* cs, void* out, float* lse, int hq, int hkv,
                  float qscale, bool rope, bool out_f32, hipStream_t s) {
  const dim3 grid((unsigned)((int64_t)h.n_q_tiles * hkv));
  if (rope)
    k_attn_m64<HP, KS, true><<<grid, dim3(256), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                        qscale, out_f32);
  else
    k_attn_m64<HP, KS, false><<<grid, dim3(256), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                         qscale, out_f32);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_m64(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                           const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                           float* lse, int hq, int hkv, int d, float qscale, bool rope,
                           bool out_f32, hipStream_t s) {
  if (d != 128) return hipErrorNotSupported;
  const int group = hq / hkv;
  if (group == 4) return launch<2, 2>(plan, h, q, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, s);
  if (group == 8) return launch<4, 1>(plan, h, q, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, s);
  return hipErrorNotSupported;
}

}  // namespace pv
