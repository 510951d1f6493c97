// bf16 MFMA path of pv_masked_attention for gfx950.
//
// Three launches on the caller's stream:
//   k_rope_table_bf16  cos/sin of every token's rotary angle (fp64 angle, fp32 result)
//   k_prep_kv          K rotated and written head-major in key tiles; V written transposed in
//                      16-key slabs whose element order is the MFMA operand order, so the main
//                      kernel stages both with plain 16-byte copies
//   k_attn_bf16        flash-style fused Q K^T / online softmax / P V.  One workgroup = one query
//                      tile (32 tokens) x one kv head; wave w owns query head kvh*G + w, so the
//                      G query heads of a GQA group share every K/V tile staged in LDS.
//
// The product S^T = K Q^T is formed (keys x queries) so that a lane owns one query column:
// row max / row sum are in-lane reductions plus one half-wave exchange, and the rescale factor
// of the online softmax is a per-lane scalar.  O^T = V^T P^T then takes P^T straight from the
// accumulator registers of S^T (the key order inside a slab is chosen to make that a pure
// register repack).
#include <type_traits>

#include "pv_internal.h"

namespace pv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);   // round to nearest even
  return __builtin_bit_cast(unsigned, r);
}
__device__ __forceinline__ float bf16_lo(unsigned u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// Value held by the lane 32 away (both halves get the other's value via max/sum of the pair).
__device__ __forceinline__ float pair_max(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16-byte LDS read issued as inline assembly: the compiler neither tracks it nor orders it against
// the global->LDS staging loads (its own LDS reads would wait for every outstanding staging load).
// The caller must execute LDS_WAIT on the destination registers before using them.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  bf16x8 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// s_waitcnt lgkmcnt(n) tied to the registers it makes valid, so no consumer can be moved above it.
#define LDS_WAIT4(n, a, b, c, d) \
  asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+v"(a), "+v"(b), "+v"(c), "+v"(d))

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// s_waitcnt immediate (gfx9 encoding) that waits for vmcnt <= n only.
__host__ __device__ constexpr int vmcnt_imm(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }

// ---------------------------------------------------------------- rotary table
__global__ __launch_bounds__(256) void k_rope_table_bf16(const int32_t* plan, PlanHeader h,
                                                         RopeFreq f, int half, float2* cs) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)h.total_tokens * half) return;
  const int g = (int)(idx / half), c = (int)(idx % half);
  const double phi = (double)plan[h.off_pos + g] * f.inv_freq[c];
  double sn, cn;
  sincos(phi, &sn, &cn);
  cs[idx] = make_float2((float)cn, (float)sn);
}

// ---------------------------------------------------------------- K/V preparation
// grid = (padded_keys / 64, Hkv), 256 threads.  Pad rows (beyond the request) are written as 0 so
// that masked probabilities (exactly 0) never meet a non-finite value.
template <int D>
__global__ __launch_bounds__(256) void k_prep_kv(const int32_t* __restrict__ plan, PlanHeader h,
                                                 const uint16_t* __restrict__ k,
                                                 const uint16_t* __restrict__ v,
                                                 const float2* __restrict__ cs, int hkv, bool rope,
                                                 uint16_t* __restrict__ krot,
                                                 uint16_t* __restrict__ vt) {
  constexpr int HALF = D / 2;
  const int tile_row = blockIdx.x * 64;      // first padded key row of this tile
  const int kvh = blockIdx.y;
  // owner request of the tile
  const int32_t* kp = plan + h.off_kpad_start;
  int lo = 0, hi = h.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (kp[mid] <= tile_row) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int tok_base = plan[h.off_tok_start + b];
  const int n_b = plan[h.off_tok_start + b + 1] - tok_base;
  const int key0 = tile_row - kp[b];         // first local key of the tile
  const int64_t out_base = ((int64_t)kvh * h.padded_keys + tile_row) * D;

  // K: thread = (key, group of 8 rotation pairs)
  for (int item = threadIdx.x; item < 64 * (HALF / 8); item += 256) {
    const int key = item / (HALF / 8), c0 = (item % (HALF / 8)) * 8;
    uint4 lo4 = make_uint4(0, 0, 0, 0), hi4 = make_uint4(0, 0, 0, 0);
    if (key0 + key < n_b) {
      const int64_t g = tok_base + key0 + key;
      const uint16_t* src = k + (g * hkv + kvh) * D;
      lo4 = *reinterpret_cast<const uint4*>(src + c0);
      hi4 = *reinterpret_cast<const uint4*>(src + c0 + HALF);
      if (rope) {
        const float2* t = cs + g * HALF + c0;
        unsigned* pl = reinterpret_cast<unsigned*>(&lo4);
        unsigned* ph = reinterpret_cast<unsigned*>(&hi4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float2 t0 = t[2 * e], t1 = t[2 * e + 1];
          const float l0 = bf16_lo(pl[e]), l1 = bf16_hi(pl[e]);
          const float h0 = bf16_lo(ph[e]), h1 = bf16_hi(ph[e]);
          pl[e] = pack_bf16(l0 * t0.x - h0 * t0.y, l1 * t1.x - h1 * t1.y);
          ph[e] = pack_bf16(h0 * t0.x + l0 * t0.y, h1 * t1.x + l1 * t1.y);
        }
      }
    }
    uint16_t* dst = krot + out_base + (int64_t)key * D;
    *reinterpret_cast<uint4*>(dst + c0) = lo4;
    *reinterpret_cast<uint4*>(dst + c0 + HALF) = hi4;
  }

  // V^T: slab s (16 keys) is [2][D][8]; element (hh, d, m) is key 8*(m/4) + 4*hh + (m%4) of the
  // slab at feature d.  Thread = one 16-byte chunk (s, hh, d).
  for (int item = threadIdx.x; item < 4 * 2 * D; item += 256) {
    const int d = item % D, hh = (item / D) % 2, s = item / (2 * D);
    unsigned short e[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int key = key0 + s * 16 + 8 * (m / 4) + 4 * hh + (m % 4);
      e[m] = (key < n_b) ? v[((int64_t)(tok_base + key) * hkv + kvh) * D + d] : (unsigned short)0;
    }
    uint4 o;
    o.x = e[0] | ((unsigned)e[1] << 16); o.y = e[2] | ((unsigned)e[3] << 16);
    o.z = e[4] | ((unsigned)e[5] << 16); o.w = e[6] | ((unsigned)e[7] << 16);
    reinterpret_cast<uint4*>(vt + out_base)[item] = o;
  }
}

// ---------------------------------------------------------------- main kernel
// FOLD: the softmax scale (times log2 e) is folded into Q before its single bf16 rounding, which
// is free when Q is rotated anyway.  Without rotation Q enters the MFMA exactly as given and the
// scale multiplies the fp32 score inside the exponent instead.
template <int D, int G, bool FOLD>
__global__ __launch_bounds__(G * 64, 2) void k_attn_bf16(
    const int32_t* __restrict__ plan, PlanHeader h, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ krot, const uint16_t* __restrict__ vt,
    const float2* __restrict__ cs, void* __restrict__ out, float* __restrict__ lse, int hq, int hkv,
    float qscale, bool rope, bool out_f32) {
  constexpr int NT = G * 64;
  constexpr int KT = D / 16;            // MFMA steps along the feature dim for S^T
  constexpr int DB = D / 32;            // 32-feature blocks of O^T
  constexpr int CH32 = 32 * D / 8;      // 16-byte chunks per 32-key K (or V^T) stage
  constexpr int CPR = D / 8;            // chunks per key row
  constexpr int NS = (D == 128) ? 5 : 8;                 // LDS stages of 32 keys (K and V^T each)
  constexpr int LPS = 2 * ((CH32 / 64) / G);             // staging loads every wave issues per stage
  // One LDS array on purpose: with several LDS variables the compiler attaches alias scopes and
  // then makes every LDS read wait for all outstanding global->LDS loads, which would serialise
  // the staging pipeline.  Ordering is enforced here with explicit vmcnt waits and barriers.
  __shared__ uint4 smem[NS][2][CH32];
#define sK(buf) smem[buf][0]
#define sV(buf) smem[buf][1]

  const int kvh = blockIdx.x % hkv;
  const QTile tile = reinterpret_cast<const QTile*>(plan + h.off_work)[blockIdx.x / hkv];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int qrow = lane & 31, hh = lane >> 5;
  const int head = kvh * G + wave;
  const bool valid = qrow < tile.rows;
  const int64_t g = (int64_t)tile.tok_base + tile.t0 + qrow;
  const int i_loc = valid ? tile.t0 + qrow : -1;
  int a_end = 0, b_start = 0;
  if (valid) { a_end = plan[h.off_aend + g]; b_start = plan[h.off_bstart + g]; }

  // ---- Q fragments: rotate, (FOLD) multiply by softmax scale * log2(e), round to bf16 once
  bf16x8 qf[KT];
  {
    float x[KT][8];
    const uint16_t* qp = q + (g * hq + head) * D + 8 * hh;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (valid) raw = *reinterpret_cast<const uint4*>(qp + 16 * t);
      const unsigned* pr = reinterpret_cast<const unsigned*>(&raw);
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[t][2 * e] = bf16_lo(pr[e]); x[t][2 * e + 1] = bf16_hi(pr[e]); }
    }
    if (rope && valid) {
      const float2* tb = cs + g * (D / 2) + 8 * hh;
#pragma unroll
      for (int t = 0; t < KT / 2; ++t) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float2 cs1 = tb[16 * t + e];
          const float lo = x[t][e], hi = x[t + KT / 2][e];
          x[t][e] = lo * cs1.x - hi * cs1.y;
          x[t + KT / 2][e] = hi * cs1.x + lo * cs1.y;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      uint4 pk;
      const float f = FOLD ? qscale : 1.0f;
      pk.x = pack_bf16(x[t][0] * f, x[t][1] * f);
      pk.y = pack_bf16(x[t][2] * f, x[t][3] * f);
      pk.z = pack_bf16(x[t][4] * f, x[t][5] * f);
      pk.w = pack_bf16(x[t][6] * f, x[t][7] * f);
      qf[t] = as_bf16x8(pk);
    }
  }

  // ---- key steps.  A key tile of the plan (64 keys) is two steps of 32 keys; tiles run over
  // [0, n_a) then [jb0, jb1).  Step j lives in LDS stage j % NS.
  const int n_tiles = tile.n_a + (tile.jb1 - tile.jb0);
  const int n_steps = 2 * n_tiles;
  const int64_t head_base = ((int64_t)kvh * h.padded_keys + tile.kpad_base) * D;   // elements
  auto step_key0 = [&](int j) {           // first key (request-local) of step j
    const int idx = j >> 1;
    const int jt = idx < tile.n_a ? idx : tile.jb0 + (idx - tile.n_a);
    return jt * 64 + (j & 1) * 32;
  };
  // Direct global->LDS staging: a wave instruction moves 64 consecutive 16-byte chunks, lane l
  // landing at chunk (base + l).  The K bank swizzle (chunk pos ^ row within each 256-byte row)
  // is applied by choosing which global chunk a lane fetches.
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);      // wave index as a scalar
  constexpr int NREP = (CH32 / 64 + G - 1) / G;                  // staging instructions per wave
  unsigned gk_off[NREP], gv_off[NREP];                           // per-lane byte offsets in a stage
#pragma unroll
  for (int n = 0; n < NREP; ++n) {
    const int P = (wave_s + n * G) * 64 + lane;
    const int R = P >> 4, pos = P & 15;
    gk_off[n] = (unsigned)(((R << 4) + (pos ^ (R & 15))) * 16);
    gv_off[n] = (unsigned)(P * 16);
  }
  const unsigned smem_base =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)(char*)&smem[0][0][0];
  constexpr unsigned STAGE_BYTES = 2 * CH32 * 16;
  const char* krot_b = reinterpret_cast<const char*>(krot) + head_base * 2;
  const char* vt_b = reinterpret_cast<const char*>(vt) + head_base * 2;
  // stage step j into LDS stage `buf` (scalar bases + per-lane offsets: a few scalar ops per step)
  auto stage = [&](int j, int buf) {
    if (j >= n_steps) return;
    const int64_t off = (int64_t)step_key0(j) * (D * 2);
    const char* gk = krot_b + off;
    const char* gv = vt_b + off;
    const unsigned lds0 = smem_base + (unsigned)buf * STAGE_BYTES;
#pragma unroll
    for (int n = 0; n < NREP; ++n) {
      const int c = wave_s + n * G;
      if ((CH32 / 64) % G != 0 && c >= CH32 / 64) break;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(gk + gk_off[n]),
          (__attribute__((address_space(3))) void*)(uintptr_t)(lds0 + c * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(gv + gv_off[n]),
          (__attribute__((address_space(3))) void*)(uintptr_t)(lds0 + CH32 * 16 + c * 1024), 16, 0, 0);
    }
  };
  bf16x8 kf[KT];          // K operand of the next S^T
  bf16x8 vf[2][DB];       // V^T operands of the current step
  // per-lane LDS byte offsets inside a stage (the K swizzle makes them lane dependent per k-step)
  unsigned k_off[KT];
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const int L = qrow * CPR + 2 * t + hh;
    const int R = L >> 4, pos = L & 15;
    k_off[t] = smem_base + (unsigned)(((R << 4) + (pos ^ (R & 15))) * 16);
  }
  const unsigned v_off = smem_base + (unsigned)((CH32 + hh * D + qrow) * 16);
  auto load_k = [&](int buf) {
    const unsigned sb = (unsigned)buf * STAGE_BYTES;
    static_for<0, KT>([&](auto t) { kf[t] = lds_read_b128<0>(k_off[t] + sb); });
  };
  auto load_v = [&](int buf) {
    const unsigned a = v_off + (unsigned)buf * STAGE_BYTES;
    static_for<0, 2>([&](auto uu) {
      static_for<0, DB>([&](auto db) { vf[uu][db] = lds_read_b128<(uu * 2 * D + db * 32) * 16>(a); });
    });
  };
  auto wait_k = [&]() {   // K operands valid; the DB*2 newer V reads may still be in flight
    if constexpr (D == 128) {
      asm volatile("s_waitcnt lgkmcnt(8)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]),
                   "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]));
    }
  };
  auto wait_k_only = [&]() {   // nothing newer in flight
    if constexpr (D == 128) {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]),
                   "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]));
    }
  };
  auto wait_v = [&]() {
    if constexpr (D == 128) {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vf[0][0]), "+v"(vf[0][1]), "+v"(vf[0][2]),
                   "+v"(vf[0][3]), "+v"(vf[1][0]), "+v"(vf[1][1]), "+v"(vf[1][2]), "+v"(vf[1][3]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vf[0][0]), "+v"(vf[0][1]), "+v"(vf[1][0]), "+v"(vf[1][1]));
    }
  };

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.0f;
  // Scores are accumulated on top of cinit = -mref (log2 units), so the MFMA result is already
  // s - mref and the probability is a bare exp2.  mref is only re-centred when a row sum leaves
  // a safe window (see the re-centre block below); l_run and o are relative to mref.
  float mref = 0.0f, l_run = 0.0f;       // mref in score units (log2 units when FOLD)
  const float esc = FOLD ? 1.0f : qscale;   // exponent scale: p = 2^(esc * (s - mref))
  auto prob = [&](float x) { return __builtin_amdgcn_exp2f(FOLD ? x : x * esc); };
  f32x16 cinit;
#pragma unroll
  for (int r = 0; r < 16; ++r) cinit[r] = 0.0f;

#pragma unroll
  for (int j = 0; j < NS - 1; ++j) stage(j, j);
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __syncthreads();
  load_k(0);
  wait_k_only();
  f32x16 s_cur = cinit;
#pragma unroll
  for (int t = 0; t < KT; ++t) s_cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], s_cur, 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  load_k(n_steps > 1 ? 1 : 0);
  // LDS stage of step j (bv), of step j+2 (bk) and the stage freed by step j-1 (bs)
  int bv = 0, bk = 2 % NS, bs = NS - 1;

  for (int j = 0; j < n_steps; ++j) {
    // Steps <= j+2 must have landed before this iteration's reads; stage j-1's buffer is free once
    // every wave has passed the barrier.  Up to NS-4 newer stages may stay in flight.
    {
      const int newer = min(j + NS - 2, n_steps - 1) - (j + 2);
      if (newer >= NS - 4 && NS > 4) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 4) * LPS));
      else __builtin_amdgcn_s_waitcnt(0x0f70);
    }
    __syncthreads();
    stage(j + NS - 1, bs);
    load_v(bv);

    const int key0 = step_key0(j);
    if (key0 >= tile.n_full * 64) {               // step not fully visible: apply the row predicate
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 8 * (r / 4) + 4 * hh + (r % 4);
        const bool vis = (key < a_end) | ((key >= b_start) & (key <= i_loc));   // branch-free
        s_cur[r] = vis ? s_cur[r] : -INFINITY;
      }
    }
    wait_k();
    __builtin_amdgcn_sched_barrier(0);

    // ---- S^T of step j+1 (MFMA) while the probabilities of step j are formed (VALU)
    asm volatile("" : "+v"(cinit));
    f32x16 s_next = cinit;
#pragma unroll
    for (int t = 0; t < KT; ++t) s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], s_next, 0, 0, 0);

    // p rounded to bf16 once; the row sum is taken over the rounded values (v_dot2c with a pair
    // of ones), so that O is an exact convex combination of V rows with the weights the MFMA sees
    unsigned pw[8];
    float rs = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pw[e] = pack_bf16(prob(s_cur[2 * e]), prob(s_cur[2 * e + 1]));
      rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[e]),
                                           __builtin_bit_cast(bf16x2, 0x3f803f80u), rs, false);
    }
    // interleave: after each MFMA of the dependent chain, a share of the softmax VALU work
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 32 / KT + 1, 0);
    }
    // Re-centre when a partial row sum is outside [2^-40, 2^40] (also catches inf/NaN/0): one
    // exact online-softmax step for the whole wave.  Rare: first steps of a row, masked steps
    // with no visible key, or scores drifting by more than 40 octaves.  The reference moves to
    // this step's row maximum, but never so far down that the history (l, O) would leave fp32
    // range: delta >= log2(l) - 20.  Both half-waves of a row take identical decisions.
    if (__builtin_amdgcn_ballot_w64(!(rs >= 0x1p-40f && rs <= 0x1p40f)) != 0) {
      float mx = s_cur[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_cur[r]);
      mx = pair_max(mx);
      const float l_tot = pair_sum(l_run);
      if (mx > -INFINITY && mx < INFINITY) {      // rows with no visible key keep their reference
        float delta = mx, alpha = 0.0f;           // empty history: nothing to rescale
        if (l_tot > 0.0f) {
          delta = fmaxf(mx, (__builtin_amdgcn_logf(l_tot) - 20.0f) / esc);
          alpha = __builtin_amdgcn_exp2f(-delta * esc);
        }
        mref += delta;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s_cur[r] -= delta; s_next[r] -= delta; cinit[r] = -mref; }
      }
      rs = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pw[e] = pack_bf16(prob(s_cur[2 * e]), prob(s_cur[2 * e + 1]));
        rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[e]),
                                             __builtin_bit_cast(bf16x2, 0x3f803f80u), rs, false);
      }
    }
    l_run += rs;

    // ---- O^T += V^T P^T for step j, while the K operand of step j+2 is fetched from LDS
    __builtin_amdgcn_sched_barrier(0);
    wait_v();
    load_k(j + 2 < n_steps ? bk : bv);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int uu = 0; uu < 2; ++uu) {
      const bf16x8 pf = as_bf16x8(make_uint4(pw[4 * uu], pw[4 * uu + 1], pw[4 * uu + 2], pw[4 * uu + 3]));
#pragma unroll
      for (int db = 0; db < DB; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[uu][db], pf, o[db], 0, 0, 0);
    }
    s_cur = s_next;
    bv = bv + 1 == NS ? 0 : bv + 1;
    bk = bk + 1 == NS ? 0 : bk + 1;
    bs = bs + 1 == NS ? 0 : bs + 1;
  }

#undef sK
#undef sV
  // ---- epilogue
  const float l_tot = pair_sum(l_run);
  if (valid) {
    const float inv = 1.0f / l_tot;
    const int64_t row = (g * hq + head) * D;
    if (out_f32) {
      float* op = reinterpret_cast<float*>(out) + row;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float4 w = make_float4(o[db][4 * gq] * inv, o[db][4 * gq + 1] * inv,
                                 o[db][4 * gq + 2] * inv, o[db][4 * gq + 3] * inv);
          *reinterpret_cast<float4*>(op + db * 32 + 8 * gq + 4 * hh) = w;
        }
    } else {
      uint16_t* op = reinterpret_cast<uint16_t*>(out) + row;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          uint2 w;
          w.x = pack_bf16(o[db][4 * gq] * inv, o[db][4 * gq + 1] * inv);
          w.y = pack_bf16(o[db][4 * gq + 2] * inv, o[db][4 * gq + 3] * inv);
          *reinterpret_cast<uint2*>(op + db * 32 + 8 * gq + 4 * hh) = w;
        }
    }
    if (lse && hh == 0)
      lse[(int64_t)head * h.total_tokens + g] = (mref * esc + log2f(l_tot)) * 0.6931471805599453f;
  }
}

template <int D, int G>
static hipError_t launch_main(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                              const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                              float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                              hipStream_t s) {
  const dim3 grid((unsigned)((int64_t)h.n_q_tiles * hkv));
  if (rope)
    k_attn_bf16<D, G, true><<<grid, dim3(G * 64), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                          qscale, rope, out_f32);
  else
    k_attn_bf16<D, G, false><<<grid, dim3(G * 64), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
                                                           qscale, rope, out_f32);
  return hipGetLastError();
}

template <int D>
static hipError_t dispatch_g(int G, const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                             const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                             float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                             hipStream_t s) {
  switch (G) {
#define PV_CASE(GG) case GG: return launch_main<D, GG>(plan, h, q, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, s);
    PV_CASE(1) PV_CASE(2) PV_CASE(3) PV_CASE(4) PV_CASE(5) PV_CASE(6) PV_CASE(7) PV_CASE(8)
#undef PV_CASE
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attn_bf16(const int32_t* plan_dev, const PlanHeader& h, const void* q,
                            const void* k, const void* v, void* out, float* lse, int hq, int hkv,
                            int d, int out_dtype, float scale, const RopeFreq& freq, bool rope,
                            char* ws, const AttnWorkspace& wl, hipEvent_t ev0, hipEvent_t ev1,
                            hipStream_t s) {
  float2* cs = reinterpret_cast<float2*>(ws + wl.off_cs);
  uint16_t* krot = reinterpret_cast<uint16_t*>(ws + wl.off_krot);
  uint16_t* vt = reinterpret_cast<uint16_t*>(ws + wl.off_vt);
  const uint16_t* kq = reinterpret_cast<const uint16_t*>(q);
  const uint16_t* kk = reinterpret_cast<const uint16_t*>(k);
  const uint16_t* kv = reinterpret_cast<const uint16_t*>(v);
  hipError_t e;
  if (rope) {
    const int64_t n = (int64_t)h.total_tokens * (d / 2);
    k_rope_table_bf16<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(plan_dev, h, freq, d / 2, cs);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    const dim3 grid((unsigned)(h.padded_keys / 64), (unsigned)hkv);
    if (d == 64) k_prep_kv<64><<<grid, dim3(256), 0, s>>>(plan_dev, h, kk, kv, cs, hkv, rope, krot, vt);
    else k_prep_kv<128><<<grid, dim3(256), 0, s>>>(plan_dev, h, kk, kv, cs, hkv, rope, krot, vt);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const float qscale = scale * 1.4426950408889634f;
  const bool out_f32 = out_dtype == PV_F32;
  if (ev0) { e = hipEventRecord(ev0, s); if (e != hipSuccess) return e; }
  if (d == 64) e = dispatch_g<64>(hq / hkv, plan_dev, h, kq, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, s);
  else e = dispatch_g<128>(hq / hkv, plan_dev, h, kq, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, s);
  if (e != hipSuccess) return e;
  if (ev1) { e = hipEventRecord(ev1, s); if (e != hipSuccess) return e; }
  return hipSuccess;
}

}  // namespace pv
