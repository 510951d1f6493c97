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
template <int D, int G>
__global__ __launch_bounds__(G * 64, 2) void k_attn_bf16(
    const int32_t* __restrict__ plan, PlanHeader h, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ krot, const uint16_t* __restrict__ vt,
    const float2* __restrict__ cs, void* __restrict__ out, float* __restrict__ lse, int hq, int hkv,
    float qscale, bool rope, bool out_f32) {
  constexpr int NT = G * 64;
  constexpr int KT = D / 16;            // MFMA steps along the feature dim for S^T
  constexpr int DB = D / 32;            // 32-feature blocks of O^T
  constexpr int CH = 64 * D / 8;        // 16-byte chunks per K (or V^T) tile
  constexpr int CPR = D / 8;            // chunks per key row
  __shared__ uint4 sK[2][CH];
  __shared__ uint4 sV[2][CH];

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

  // ---- Q fragments: rotate and round to bf16 once.  The softmax scale (times log2 e) is applied
  // to the fp32 scores inside the exponent's fma, so un-rotated inputs enter the MFMA exactly.
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
      pk.x = pack_bf16(x[t][0], x[t][1]);
      pk.y = pack_bf16(x[t][2], x[t][3]);
      pk.z = pack_bf16(x[t][4], x[t][5]);
      pk.w = pack_bf16(x[t][6], x[t][7]);
      qf[t] = as_bf16x8(pk);
    }
  }

  // ---- key tile sequence: [0, n_a) then [jb0, jb1)
  const int n_tiles = tile.n_a + (tile.jb1 - tile.jb0);
  const int64_t head_base = ((int64_t)kvh * h.padded_keys + tile.kpad_base) * D;   // elements
  auto tile_index = [&](int idx) { return idx < tile.n_a ? idx : tile.jb0 + (idx - tile.n_a); };
  // Stage one K tile and one V^T tile with direct global->LDS loads: a wave instruction moves 64
  // consecutive 16-byte chunks, lane l landing at chunk (base + l).  The K bank swizzle (chunk
  // pos ^ row within each 256-byte row) is applied by choosing which global chunk a lane fetches.
  auto stage = [&](int jt, int buf) {
    const uint4* gk = reinterpret_cast<const uint4*>(krot + head_base + (int64_t)jt * 64 * D);
    const uint4* gv = reinterpret_cast<const uint4*>(vt + head_base + (int64_t)jt * 64 * D);
    for (int c = wave; c < CH / 64; c += G) {
      const int P = c * 64 + lane;
      const int R = P >> 4, pos = P & 15;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(gk + (R << 4) + (pos ^ (R & 15))),
          (__attribute__((address_space(3))) void*)(&sK[buf][c * 64]), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(gv + P),
          (__attribute__((address_space(3))) void*)(&sV[buf][c * 64]), 16, 0, 0);
    }
  };

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.0f;
  float m_run = -1e30f, l_run = 0.0f;

  stage(tile_index(0), 0);

  for (int idx = 0; idx < n_tiles; ++idx) {
    const int cur = idx & 1;
    const int jt = tile_index(idx);
    // tile idx has landed (own loads: vmcnt(0); other waves': barrier); the barrier also means
    // every wave is done reading the other buffer, which the next stage() overwrites
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
    if (idx + 1 < n_tiles) stage(tile_index(idx + 1), cur ^ 1);

    // ---- S^T = K Q^T for two blocks of 32 keys
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.0f;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int L = (kb * 32 + qrow) * CPR + 2 * t + hh;
        const int R = L >> 4, pos = L & 15;
        const bf16x8 a = as_bf16x8(sK[cur][(R << 4) + (pos ^ (R & 15))]);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[t], s[kb], 0, 0, 0);
      }
    }

    // ---- mask (only tiles that are not fully visible)
    if (jt >= tile.n_full) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = jt * 64 + kb * 32 + 8 * (r / 4) + 4 * hh + (r % 4);
          const bool vis = (key < a_end) | ((key >= b_start) & (key <= i_loc));   // branch-free
          s[kb][r] = vis ? s[kb][r] : -INFINITY;
        }
    }

    // ---- online softmax on raw scores; p = 2^(qscale * (s - m))
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    mx = pair_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * qscale);
    const float neg_mc = -m_new * qscale;
    // p rounded to bf16 once; the row sum is taken over the rounded values (v_dot2c with a pair
    // of ones), so that O is an exact convex combination of V rows with the weights the MFMA sees
    uint4 pp[4];
    float rs = 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      unsigned w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = 8 * (u & 1) + 2 * e;
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[u >> 1][r], qscale, neg_mc));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[u >> 1][r + 1], qscale, neg_mc));
        w[e] = pack_bf16(p0, p1);
        rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e]),
                                             __builtin_bit_cast(bf16x2, 0x3f803f80u), rs, false);
      }
      pp[u] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    l_run = l_run * alpha + rs;
    if (__any(m_new > m_run)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    m_run = m_new;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bf16x8 pf = as_bf16x8(pp[u]);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 a = as_bf16x8(sV[cur][(u * 2 + hh) * D + db * 32 + qrow]);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, o[db], 0, 0, 0);
      }
    }

  }

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
      lse[(int64_t)head * h.total_tokens + g] = (m_run * qscale + log2f(l_tot)) * 0.6931471805599453f;
  }
}

template <int D, int G>
static hipError_t launch_main(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                              const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                              float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                              hipStream_t s) {
  const dim3 grid((unsigned)((int64_t)h.n_q_tiles * hkv));
  k_attn_bf16<D, G><<<grid, dim3(G * 64), 0, s>>>(plan, h, q, krot, vt, cs, out, lse, hq, hkv,
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
