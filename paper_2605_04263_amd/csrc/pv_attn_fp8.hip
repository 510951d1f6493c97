// FP8 K/V path of the masked attention for gfx950: K and V arrive as OCP FP8 E4M3 codes with one
// fp32 scale per kv head (the storage format of an FP8 serving stack; the keys are what a KV cache
// holds, i.e. already rotated), Q arrives in bf16 and is rotated here.  Both products run on the
// FP8 matrix instruction v_mfma_f32_32x32x64_f8f6f4 (64-deep, twice the bf16 rate), fp32 accumulate:
//   k_prep_fp8   K and V^T of every 64-key tile re-laid-out in MFMA operand order (plain byte moves,
//                no arithmetic on the codes), and the cos/sin table for Q
//   (rows that see at most PV_SHORT_ROW_KEYS keys are evaluated in plain fp32 by extra workgroups at the
//   end of k_attn_fp8's grid, one wave per row and query head)
//   k_attn_fp8   flash-style pass: one workgroup = one 32-token query tile x one kv head, wave w =
//                query head kvh*G + w; a step is one 64-key tile.  Q is rotated, scaled by a per-row
//                power of two and split into two E4M3 terms (the rounded value and 16 x the rounding
//                residual, the second product scaled by 2^-4 inside the instruction), which carries Q
//                at about bf16 precision through the FP8 pipe; probabilities are formed against a running
//                reference, scaled by 2^8 and rounded to E4M3; the row sum comes out of the matrix
//                pipe (a tile of ones as the fifth V^T block), so the output is an exact convex
//                combination of V rows with the rounded weights.
// Operand layout of the instruction (checked on the device): lane l holds row (or column) l % 32 and
// the 32 consecutive depth indices 32 * (l / 32) .. + 31, byte j of its 32 bytes = depth offset j;
// the accumulator is laid out like the other 32x32 products (lane: column l % 32, register r: row
// 8 (r / 4) + 4 (l / 32) + r % 4).
#include "pv_attn_common.h"

namespace pv {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kStepKeys = 64;            // keys per step = depth of the second product

__device__ __forceinline__ f32x16 mfma_fp8(const i32x8& a, const i32x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);   // both operands E4M3, no block scales
}
// The same product with the B operand scaled by 2^-4 in the instruction (block scales are E8M0
// exponents, 0x7f = 1; checked on the device): used for the low part of Q.
__device__ __forceinline__ f32x16 mfma_fp8_b_sixteenth(const i32x8& a, const i32x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0x7f, 0, 0x7b);
}
__device__ __forceinline__ float fp8_byte(unsigned word, int byte) {
  switch (byte) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8((int)word, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8((int)word, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8((int)word, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8((int)word, 3);
  }
}
// four floats -> four E4M3 codes in one dword (round to nearest even; callers keep |x| <= 448)
__device__ __forceinline__ unsigned pack_fp8x4(float a, float b, float c, float d) {
  int w = 0;
  w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
  return (unsigned)w;
}

// ---------------------------------------------------------------- preparation
// One workgroup per (64-key tile, kv head).  Workspace per kv head and tile (8 KB each for D = 128):
//   K:    16-byte chunk ((u * 2 + t) * 2 + c) * 64 + l  = features 64 t + 32 (l / 32) + 16 c .. + 15
//         of key 32 u + l % 32           (u: 32-key half, t: 64-feature half)
//   V^T:  16-byte chunk (db * 2 + c) * 64 + l            = feature 32 db + l % 32 at the 16 keys
//         32 c + 8 i + 4 (l / 32) + e, byte 4 i + e      (the key order in which the accumulator
//         registers of S^T hold keys, so probabilities go into the second product in place)
// Pad keys (beyond the request) are zero codes.
template <int D>
__global__ __launch_bounds__(256) void k_prep_fp8(const int32_t* __restrict__ plan, PlanHeader h,
                                                  const uint8_t* __restrict__ k8,
                                                  const uint8_t* __restrict__ v8, RopeFreq f,
                                                  float2* __restrict__ cs, int hkv, bool rope,
                                                  uint8_t* __restrict__ kw, uint8_t* __restrict__ vw) {
  static_assert(D == 128, "the FP8 path is built for head_dim 128");
  constexpr int CPR = D / 16;                              // 16-byte chunks per key row
  __shared__ uint4 v_s[kStepKeys][CPR + 1];                // V rows of the tile, padded
  const int tile = (int)blockIdx.x / hkv, kvh = (int)blockIdx.x % hkv;
  const int row0 = tile * kStepKeys;                       // first padded key row
  const int32_t* kp = plan + h.off_kpad_start;
  int lo = 0, hi = h.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (kp[mid] <= row0) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int tok_base = plan[h.off_tok_start + b];
  const int n_b = plan[h.off_tok_start + b + 1] - tok_base;
  const int key0 = row0 - kp[b];
  const int tid = threadIdx.x;
  uint8_t* k_out = kw + ((int64_t)kvh * h.padded_keys + row0) * D;
  uint8_t* v_out = vw + ((int64_t)kvh * h.padded_keys + row0) * D;
#pragma unroll
  for (int it = 0; it < kStepKeys * CPR / 256; ++it) {
    const int ch = tid + it * 256, key = ch / CPR, c16 = ch % CPR;
    uint4 kx = make_uint4(0, 0, 0, 0), vx = make_uint4(0, 0, 0, 0);
    if (key0 + key < n_b) {
      const int64_t src = (caller_row(plan, h, tok_base + key0 + key) * hkv + kvh) * D + c16 * 16;
      kx = *reinterpret_cast<const uint4*>(k8 + src);
      vx = *reinterpret_cast<const uint4*>(v8 + src);
    }
    const int u = key >> 5, t = c16 >> 2, hh = (c16 >> 1) & 1, c = c16 & 1;
    reinterpret_cast<uint4*>(k_out)[((u * 2 + t) * 2 + c) * 64 + hh * 32 + (key & 31)] = kx;
    v_s[key][c16] = vx;
  }
  __syncthreads();
  const uint8_t* vb = reinterpret_cast<const uint8_t*>(&v_s[0][0]);
  constexpr int VROW = (CPR + 1) * 16;
#pragma unroll
  for (int it = 0; it < (D / 32) * 2 * 64 / 256; ++it) {
    const int ch = tid + it * 256, l = ch & 63, c = (ch >> 6) & 1, db = ch >> 7;
    const int feat = 32 * db + (l & 31), hh = l >> 5;
    unsigned w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[i] = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        w[i] |= (unsigned)vb[(32 * c + 8 * i + 4 * hh + e) * VROW + feat] << (8 * e);
    }
    reinterpret_cast<uint4*>(v_out)[(db * 2 + c) * 64 + l] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  if (rope && kvh == 0) {
    for (int item = tid; item < kStepKeys * (D / 2); item += 256) {
      const int key = item / (D / 2), c = item % (D / 2);
      if (key0 + key < n_b) {
        const int64_t g = tok_base + key0 + key;
        cs[g * (D / 2) + c] = rotary_cos_sin(plan[h.off_pos + g], f.inv_freq[c]);
      }
    }
  }
}

// ---------------------------------------------------------------- rows with few keys, fp32
// One wave per (short row, query head); lane c owns the rotation pair (c, c + D/2).
template <int D>
__device__ void short_unit_fp8(const int32_t* __restrict__ plan, const PlanHeader& h,
                               const uint16_t* __restrict__ q, const uint8_t* __restrict__ k8,
                               const uint8_t* __restrict__ v8, const float* __restrict__ k_scale,
                               const float* __restrict__ v_scale, const float2* __restrict__ table,
                               int hq, int hkv, bool rope, float scale, void* __restrict__ out,
                               float* __restrict__ lse, bool out_f32, int unit, int lane) {
  constexpr int HALF = D / 2;
  const int4 desc = reinterpret_cast<const int4*>(plan + h.off_short)[unit / hq];
  const int head = unit % hq, kvh = head / (hq / hkv);
  const int g = desc.x, base = desc.y, i = g - base, a_end = desc.z, b_start = desc.w;
  const int n_a = min(a_end, (int)PV_SHORT_ROW_KEYS);
  const int b0 = max(b_start, a_end);
  const int n = min(n_a + max(i - b0 + 1, 0), (int)PV_SHORT_ROW_KEYS);
  const int c = lane;                                      // HALF == 64 lanes for D = 128
  const int64_t g_row = caller_row(plan, h, g);
  const uint16_t* qr = q + (g_row * hq + head) * D;
  const float xl = __uint_as_float((unsigned)qr[c] << 16), xh = __uint_as_float((unsigned)qr[c + HALF] << 16);
  float ql = xl, qh = xh;
  if (rope) {
    const float2 t = table[(int64_t)g * HALF + c];
    ql = xl * t.x - xh * t.y;
    qh = xh * t.x + xl * t.y;
  }
  const float ks = k_scale[kvh], vs = v_scale[kvh];
  float sc[PV_SHORT_ROW_KEYS], vl[PV_SHORT_ROW_KEYS], vh[PV_SHORT_ROW_KEYS];
  float m = -INFINITY;
#pragma unroll
  for (int e = 0; e < PV_SHORT_ROW_KEYS; ++e) {
    const int key = e < n_a ? e : b0 + (e - n_a);
    const int64_t row = (caller_row(plan, h, base + (e < n ? key : i)) * hkv + kvh) * D;
    const float kl = fp8_byte(k8[row + c], 0), kh = fp8_byte(k8[row + c + HALF], 0);
    vl[e] = fp8_byte(v8[row + c], 0);
    vh[e] = fp8_byte(v8[row + c + HALF], 0);
    float part = e < n ? ql * kl + qh * kh : 0.0f;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    sc[e] = e < n ? part * (scale * ks) : -INFINITY;
    m = fmaxf(m, sc[e]);
  }
  float l = 0.0f, ol = 0.0f, oh = 0.0f;
#pragma unroll
  for (int e = 0; e < PV_SHORT_ROW_KEYS; ++e) {
    const float p = expf(sc[e] - m);
    l += p;
    if (e < n) { ol = fmaf(p, vl[e], ol); oh = fmaf(p, vh[e], oh); }
  }
  const int64_t orow = (g_row * hq + head) * D;
  const float rl = ol * vs / l, rh = oh * vs / l;
  if (out_f32) {
    float* op = reinterpret_cast<float*>(out) + orow;
    op[c] = rl; op[c + HALF] = rh;
  } else {
    uint16_t* op = reinterpret_cast<uint16_t*>(out) + orow;
    op[c] = (uint16_t)(pack_bf16(rl, 0.0f) & 0xffffu);
    op[c + HALF] = (uint16_t)(pack_bf16(rh, 0.0f) & 0xffffu);
  }
  if (lse && lane == 0) lse[(int64_t)head * h.total_tokens + g_row] = m + logf(l);
}

// ---------------------------------------------------------------- main kernel
// Staging of one step's K and V^T tiles (2 x 512 chunks of 16 bytes) through registers.  Free functions
// on purpose: a private array captured by a lambda is not kept in registers by the compiler.
template <int G, int CPT>
__device__ __forceinline__ void fp8_fetch(uint4 (&st)[CPT], const uint8_t* __restrict__ kw,
                                          const uint8_t* __restrict__ vw, int64_t off, int tid) {
  constexpr int CH = kStepKeys * 128 / 16;
#pragma unroll
  for (int n = 0; n < CPT; ++n) {
    // (threads beyond the last chunk repeat it: every register is loaded unconditionally)
    const int x = min(tid + n * (G * 64), 2 * CH - 1);
    st[n] = x < CH ? reinterpret_cast<const uint4*>(kw + off)[x] : reinterpret_cast<const uint4*>(vw + off)[x - CH];
  }
}
template <int G, int CPT>
__device__ __forceinline__ void fp8_commit(const uint4 (&st)[CPT], uint4* __restrict__ buf, int tid) {
  constexpr int CH = kStepKeys * 128 / 16;
#pragma unroll
  for (int n = 0; n < CPT; ++n) {
    const int x = tid + n * (G * 64);
    if ((2 * CH) % (G * 64) == 0 || x < 2 * CH) buf[x] = st[n];
  }
}

template <int D, int G>
__global__ __launch_bounds__(G * 64, 2) void k_attn_fp8(
    const int32_t* __restrict__ plan, PlanHeader h, const uint16_t* __restrict__ q,
    const uint8_t* __restrict__ kw, const uint8_t* __restrict__ vw, const float2* __restrict__ cs,
    const float* __restrict__ k_scale, const float* __restrict__ v_scale, void* __restrict__ out,
    float* __restrict__ lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
    const uint8_t* __restrict__ k8, const uint8_t* __restrict__ v8, float scale, int n_short_blocks) {
  static_assert(D == 128, "the FP8 path is built for head_dim 128");
  // The last n_short_blocks workgroups evaluate the rows with very few keys in fp32, one (row, query
  // head) per wave, from the caller's codes and the table of rotary angles: light work that starts
  // when every item of the grid has been taken, in the tail of the launch.
  if (n_short_blocks > 0 && blockIdx.x >= gridDim.x - (unsigned)n_short_blocks) {
    const int unit = (int)(blockIdx.x - (gridDim.x - (unsigned)n_short_blocks)) * G + ((int)threadIdx.x >> 6);
    if (unit < h.n_short_rows * hq)                        // whole waves leave together
      short_unit_fp8<D>(plan, h, q, k8, v8, k_scale, v_scale, cs, hq, hkv, rope, scale, out, lse, out_f32,
                        unit, (int)threadIdx.x & 63);
    return;
  }
  constexpr int TILE_BYTES = kStepKeys * D;               // 8 KB of K, the same of V^T
  constexpr int TILE_CHUNKS = TILE_BYTES / 16;            // 512
  constexpr int CPT = (2 * TILE_CHUNKS + G * 64 - 1) / (G * 64);   // staging chunks per thread and step
  __shared__ uint4 smem[2][2 * TILE_CHUNKS];              // [buffer][K chunks, then V^T chunks]

  const int item = (int)blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int qrow = lane & 31, hh = lane >> 5;
  const int kvh = item % hkv, head = kvh * G + wave;
  const QTile tile = reinterpret_cast<const QTile*>(plan + h.off_work)[item / hkv];
  const bool valid = qrow < tile.rows;
  const int row_l = tile.t0 + min(qrow, tile.rows - 1);    // pad lanes repeat the last row (never stored)
  const int64_t g = (int64_t)tile.tok_base + row_l;
  const int i_loc = valid ? tile.t0 + qrow : -1;
  int a_end = 0, b_start = 0;
  if (valid) { a_end = plan[h.off_aend + g]; b_start = plan[h.off_bstart + g]; }

  // ---- Q: features 32 hh .. + 31 and 64 + 32 hh .. + 31 of this lane's row (the rotation pairs
  // (c, c + 64) sit in one lane), rotated, scaled by a power of two that brings the row's largest
  // magnitude into [128, 256), rounded to E4M3.
  i32x8 qf[2], qlo[2];                                     // Q = qf + qlo / 16, both E4M3
  float c_row;                                             // exponent argument per unit of S
  {
    const uint16_t* qr = q + (caller_row(plan, h, g) * hq + head) * D;
    float lo[32], hi[32];
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
      const uint4 a = reinterpret_cast<const uint4*>(qr + 32 * hh)[v4];
      const uint4 b = reinterpret_cast<const uint4*>(qr + 64 + 32 * hh)[v4];
      const unsigned aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        lo[8 * v4 + 2 * e] = bf16_lo(aw[e]); lo[8 * v4 + 2 * e + 1] = bf16_hi(aw[e]);
        hi[8 * v4 + 2 * e] = bf16_lo(bw[e]); hi[8 * v4 + 2 * e + 1] = bf16_hi(bw[e]);
      }
    }
    if (rope) {
      const float2* t = cs + g * (D / 2) + 32 * hh;
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const float2 w = t[j];
        const float l0 = lo[j], h0 = hi[j];
        lo[j] = l0 * w.x - h0 * w.y;
        hi[j] = h0 * w.x + l0 * w.y;
      }
    }
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < 32; ++j) amax = fmaxf(amax, fmaxf(fabsf(lo[j]), fabsf(hi[j])));
    amax = pair_max(amax);
    // power of two f with 128 <= amax * f < 256 (exact scaling; 1 for an all-zero row)
    int e2 = (int)((__float_as_uint(amax) >> 23) & 255u) - 127;
    e2 = max(e2, -100);
    const float fac = amax > 0.0f ? __uint_as_float((unsigned)(127 + 7 - e2) << 23) : 1.0f;
    const float inv_fac = amax > 0.0f ? __uint_as_float((unsigned)(127 - 7 + e2) << 23) : 1.0f;
    auto split4 = [&](const float* x, int& top, int& rest) {   // four values -> rounded codes and residual codes
      const float x0 = x[0] * fac, x1 = x[1] * fac, x2 = x[2] * fac, x3 = x[3] * fac;
      const unsigned w = pack_fp8x4(x0, x1, x2, x3);
      top = (int)w;
      rest = (int)pack_fp8x4((x0 - fp8_byte(w, 0)) * 16.0f, (x1 - fp8_byte(w, 1)) * 16.0f,
                             (x2 - fp8_byte(w, 2)) * 16.0f, (x3 - fp8_byte(w, 3)) * 16.0f);
    };
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      int top, rest;
      split4(&lo[4 * w], top, rest);
      qf[0][w] = top; qlo[0][w] = rest;
      split4(&hi[4 * w], top, rest);
      qf[1][w] = top; qlo[1][w] = rest;
    }
    c_row = qscale * k_scale[kvh] * inv_fac;               // qscale = softmax scale * log2(e)
  }

  f32x16 o[4], lacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) { o[0][r] = 0.0f; o[1][r] = 0.0f; o[2][r] = 0.0f; o[3][r] = 0.0f; lacc[r] = 0.0f; }
  i32x8 ones;
#pragma unroll
  for (int w = 0; w < 8; ++w) ones[w] = 0x38383838;       // 1.0 in E4M3
  float mref = -INFINITY;                                  // reference of the exponent, log2 units

  const int n_steps = tile.n_a + (tile.jb1 - tile.jb0);
  const int64_t head_base = ((int64_t)kvh * h.padded_keys + tile.kpad_base) * D;     // bytes
  auto step_tile = [&](int j) { return j < tile.n_a ? j : tile.jb0 + (j - tile.n_a); };
  // staging through registers: chunk x of the 2 * TILE_CHUNKS of a step (K first, then V^T)
  uint4 st[CPT];
  fp8_fetch<G, CPT>(st, kw, vw, head_base + (int64_t)step_tile(0) * TILE_BYTES, tid);
  fp8_commit<G, CPT>(st, &smem[0][0], tid);
  __syncthreads();

  for (int j = 0; j < n_steps; ++j) {
    const int buf = j & 1;
    // (the last step fetches its own tile once more instead of branching: a conditional fetch makes
    // the compiler keep the staging registers in scratch memory)
    fp8_fetch<G, CPT>(st, kw, vw, head_base + (int64_t)step_tile(min(j + 1, n_steps - 1)) * TILE_BYTES, tid);
    const uint4* kt = &smem[buf][0];
    const uint4* vt = &smem[buf][TILE_CHUNKS];
    // S^T of the two 32-key halves
    f32x16 s[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[u][r] = 0.0f;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4 a0 = kt[((u * 2 + t) * 2 + 0) * 64 + lane], a1 = kt[((u * 2 + t) * 2 + 1) * 64 + lane];
        i32x8 a;
        a[0] = (int)a0.x; a[1] = (int)a0.y; a[2] = (int)a0.z; a[3] = (int)a0.w;
        a[4] = (int)a1.x; a[5] = (int)a1.y; a[6] = (int)a1.z; a[7] = (int)a1.w;
        s[u] = mfma_fp8(a, qf[t], s[u]);
        s[u] = mfma_fp8_b_sixteenth(a, qlo[t], s[u]);
      }
    }
    const int jt = step_tile(j);
    const int key0 = jt * kStepKeys;
    if (jt >= tile.n_full) {
      // Row predicate: the keys of half u that this lane holds are key0 + 32 u + 4 hh + c,
      // c = 8 (r / 4) + r % 4; the row's visible ones among the 32 become a bit mask, and a score
      // is kept or replaced by -inf with one bit-field extract and one bit-field insert.
      auto low_bits = [](int n) {                          // bits [0, n) of 32, n clamped to [0, 32]
        const unsigned m = (1u << (n & 31)) - 1u;
        return n <= 0 ? 0u : n >= 32 ? 0xffffffffu : m;
      };
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int base = key0 + 32 * u + 4 * hh;
        const unsigned vis = low_bits(a_end - base) | (low_bits(i_loc - base + 1) & ~low_bits(b_start - base));
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned keep = (unsigned)__builtin_amdgcn_sbfe((int)vis, 8 * (r / 4) + (r % 4), 1);
          s[u][r] = __uint_as_float((__float_as_uint(s[u][r]) & keep) | (0xff800000u & ~keep));
        }
      }
    }
    // running reference: moved up when this step's largest exponent exceeds it by more than 0.75
    // octave (probabilities scaled by 2^8 then stay below 2^8.75 = 431 < 448, the largest E4M3 value)
    float mx = s[0][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
    mx = pair_max(mx) * c_row;                              // c_row > 0
    const bool raise = mx > mref + 0.75f || (mref == -INFINITY && mx > -INFINITY);
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
      const float m_new = raise ? mx : mref;
      const float alpha = mref == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(mref - m_new);   // 1 when unchanged
      mref = m_new;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o[0][r] *= alpha; o[1][r] *= alpha; o[2][r] *= alpha; o[3][r] *= alpha; lacc[r] *= alpha;
      }
    }
    // probabilities: 2^(S c - mref + 8), rounded to E4M3, in accumulator key order
    const float bias = mref == -INFINITY ? 0.0f : 8.0f - mref;   // no key seen yet: every S is -inf, p = 0
    i32x8 pb;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float p[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[u][4 * i + e], c_row, bias));
        pb[4 * u + i] = (int)pack_fp8x4(p[0], p[1], p[2], p[3]);
      }
    // O^T += V^T P^T, and the row sums through a tile of ones
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const uint4 a0 = vt[(db * 2 + 0) * 64 + lane], a1 = vt[(db * 2 + 1) * 64 + lane];
      i32x8 a;
      a[0] = (int)a0.x; a[1] = (int)a0.y; a[2] = (int)a0.z; a[3] = (int)a0.w;
      a[4] = (int)a1.x; a[5] = (int)a1.y; a[6] = (int)a1.z; a[7] = (int)a1.w;
      o[db] = mfma_fp8(a, pb, o[db]);
    }
    lacc = mfma_fp8(ones, pb, lacc);
    fp8_commit<G, CPT>(st, &smem[buf ^ 1][0], tid);
    __syncthreads();
  }

  // ---- epilogue: every register of lacc holds the row sum of this lane's query column
  const float l_tot = lacc[0];
  const bool stored = valid && a_end + i_loc - b_start + 1 > PV_SHORT_ROW_KEYS;   // short rows: the extra workgroups
  if (stored) {
    const float inv = v_scale[kvh] / l_tot;
    const int64_t orow = (caller_row(plan, h, g) * hq + head) * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int feat = 32 * db + 8 * i + 4 * hh;
        const float x0 = o[db][4 * i] * inv, x1 = o[db][4 * i + 1] * inv, x2 = o[db][4 * i + 2] * inv, x3 = o[db][4 * i + 3] * inv;
        if (out_f32) {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + orow + feat) = make_float4(x0, x1, x2, x3);
        } else {
          uint2 w;
          w.x = pack_bf16(x0, x1); w.y = pack_bf16(x2, x3);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + orow + feat) = w;
        }
      }
    if (lse && hh == 0)
      lse[(int64_t)head * h.total_tokens + caller_row(plan, h, g)] = (log2f(l_tot) - 8.0f + mref) * 0.6931471805599453f;
  }
}

template <int G>
static hipError_t launch_main_fp8(const int32_t* plan, const PlanHeader& h, const uint16_t* q, const uint8_t* kw,
                                  const uint8_t* vw, const float2* cs, const float* ks, const float* vs, void* out,
                                  float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                                  const uint8_t* k8, const uint8_t* v8, float scale, hipStream_t s) {
  dim3 grid;
  // one wave per (short row, query head), G of them to a workgroup, behind the items of the grid
  const int64_t n_short = ((int64_t)h.n_short_rows * hq + G - 1) / G;
  if (n_short > 0x7fffffff || !grid_1d((int64_t)h.n_q_tiles * hkv + n_short, G * 64, &grid))
    return hipErrorInvalidConfiguration;
  k_attn_fp8<128, G><<<grid, dim3(G * 64), 0, s>>>(plan, h, q, kw, vw, cs, ks, vs, out, lse, hq, hkv, qscale, rope,
                                                   out_f32, k8, v8, scale, (int)n_short);
  return hipGetLastError();
}

hipError_t launch_attn_fp8(const int32_t* plan_dev, const PlanHeader& h, const void* q, const void* k8,
                           const void* v8, const float* k_scale, const float* v_scale, void* out, float* lse,
                           int hq, int hkv, int d, int out_dtype, float scale, const RopeFreq& freq, bool rope,
                           char* ws, const AttnWorkspace& wl, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s) {
  if (d != 128) return hipErrorInvalidValue;
  float2* cs = reinterpret_cast<float2*>(ws + wl.off_cs);
  uint8_t* kw = reinterpret_cast<uint8_t*>(ws + wl.off_krot);
  uint8_t* vw = reinterpret_cast<uint8_t*>(ws + wl.off_vt);
  const uint16_t* kq = reinterpret_cast<const uint16_t*>(q);
  const bool out_f32 = out_dtype == PV_F32;
  dim3 grid;
  if (!grid_1d((int64_t)(h.padded_keys / kStepKeys) * hkv, 256, &grid)) return hipErrorInvalidConfiguration;
  k_prep_fp8<128><<<grid, dim3(256), 0, s>>>(plan_dev, h, (const uint8_t*)k8, (const uint8_t*)v8, freq, cs, hkv, rope, kw, vw);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const float qscale = scale * 1.4426950408889634f;
  if (ev0) { e = hipEventRecord(ev0, s); if (e != hipSuccess) return e; }
  switch (hq / hkv) {
#define PV_CASE(GG) case GG: e = launch_main_fp8<GG>(plan_dev, h, kq, kw, vw, cs, k_scale, v_scale, out, lse, hq, hkv, qscale, rope, out_f32, (const uint8_t*)k8, (const uint8_t*)v8, scale, s); break;
    PV_CASE(1) PV_CASE(2) PV_CASE(3) PV_CASE(4) PV_CASE(5) PV_CASE(6) PV_CASE(7) PV_CASE(8)
#undef PV_CASE
    default: e = hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  if (ev1) { e = hipEventRecord(ev1, s); if (e != hipSuccess) return e; }
  return hipSuccess;
}

}  // namespace pv
