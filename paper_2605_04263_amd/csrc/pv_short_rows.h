// The caller's K/V tensors as the kernels see them, and the fp32 evaluation of the rows with very few
// visible keys.  Used by the K/V preparation kernel (segment-only and prepared-key calls) and by the
// main kernel, whose whole-pass launches carry these rows as extra workgroups at the end of the grid.
#ifndef PV_SHORT_ROWS_H_
#define PV_SHORT_ROWS_H_

#include "pv_attn_common.h"

namespace pv {

// Where the caller's K and V rows are: one dense tensor each, or (block_table != nullptr) a pool of
// pages of page_size tokens, token row r of the packed batch living at row
// block_table[r / page_size] * page_size + r % page_size of the pool.
struct KvSource {
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* block_table;
  int page_size;
  __device__ __forceinline__ int64_t row(int64_t r) const {
    return block_table ? (int64_t)block_table[r / page_size] * page_size + r % page_size : r;
  }
};

struct ShortRowArgs {          // what the fp32 evaluation of the short rows needs beyond k, v, cs
  const uint16_t* q;
  void* out;
  float* lse;
  int hq;
  float scale;
  bool out_f32;
  bool seg_only;       // segment-only call: rows of prompt and draft tokens are left alone
  const float2* table; // (cos, sin) of every packed row's rotary angles, [row][D/2], if already written;
                       // nullptr: the angles are computed here from the frequencies
};

// Rows with at most PV_SHORT_ROW_KEYS visible keys, in plain fp32 (the main kernel does not store
// them).  One workgroup per (row, kv head): all threads first rotate the row's visible keys into
// LDS (one rotary angle per thread and pass instead of one per key and lane), then wave w
// evaluates query head kvh*G + w (+NW, ...), lane c owning the rotation pair (c, c + D/2).
// NW = waves of the workgroup (at least 4; the first four move the keys).  `f` may be null when
// a.table is given.
template <int D, int NW = 4>
__device__ void short_row_block(const int32_t* __restrict__ plan, const PlanHeader& h,
                                const KvSource& src, const RopeFreq* f, int hkv, bool rope, const ShortRowArgs& a,
                                int4 desc, int kvh, float (*ks)[D], float (*vs)[D]) {
  static_assert(NW >= 4, "four waves move the keys");
  constexpr int HALF = D / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool mover = tid < 256;
  const int G = a.hq / hkv;
  // desc = (packed row, first row of its request, a_end, b_start), written by the host
  const int g = desc.x, base = desc.y, i = g - base;
  const int a_end = desc.z, b_start = desc.w;
  if (a.seg_only && b_start == 0) return;      // a prompt or draft row (uniform over the workgroup)
  // Visible keys: [0, a_end) then [max(b_start, a_end), i]; at most PV_SHORT_ROW_KEYS of them.
  const int n_a = min(a_end, (int)PV_SHORT_ROW_KEYS);
  const int b0 = max(b_start, a_end);
  const int n = min(n_a + max(i - b0 + 1, 0), (int)PV_SHORT_ROW_KEYS);
  // the query pair of this wave's first head and the row's position are requested up front as well
  const bool on = lane < HALF;
  const int c = on ? lane : 0;
  const int64_t g_row = caller_row(plan, h, g);        // this row in q / out / lse
  const uint16_t* q_first = a.q + (g_row * a.hq + kvh * G + min(wave, G - 1)) * D;
  const unsigned short q_lo0 = q_first[c], q_hi0 = q_first[c + HALF];
  const int pos_g = (rope && !a.table) ? plan[h.off_pos + g] : 0;
  // all loads of the pass are issued before any of them is used (fixed trip count, predicated)
  constexpr int IT = PV_SHORT_ROW_KEYS * HALF / 256;
  static_assert(IT * 256 == PV_SHORT_ROW_KEYS * HALF, "whole passes");
  unsigned short k_lo[IT], k_hi[IT], v_lo[IT], v_hi[IT];
  int pos_k[IT];
  float2 tab_k[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int item = (tid & 255) + it * 256;
    const int e = item / HALF, c = item % HALF;
    const int key = e < n_a ? e : b0 + (e - n_a);
    const int tok = base + (e < n ? key : i);             // clamp to a valid row when predicated off
    const int64_t tok_row = src.row(caller_row(plan, h, tok));
    const uint16_t* kr = src.k + (tok_row * hkv + kvh) * D;
    const uint16_t* vr = src.v + (tok_row * hkv + kvh) * D;
    k_lo[it] = kr[c]; k_hi[it] = kr[c + HALF];
    v_lo[it] = vr[c]; v_hi[it] = vr[c + HALF];
    pos_k[it] = 0;
    tab_k[it] = make_float2(1.0f, 0.0f);
    if (rope) {
      if (a.table) tab_k[it] = a.table[(int64_t)tok * HALF + c];
      else pos_k[it] = plan[h.off_pos + tok];
    }
  }
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int item = (tid & 255) + it * 256;
    const int e = item / HALF, c = item % HALF;
    if (mover && e < n) {
      const float xl = __uint_as_float((unsigned)k_lo[it] << 16), xh = __uint_as_float((unsigned)k_hi[it] << 16);
      float rl = xl, rh = xh;
      if (rope) {
        const float2 t = a.table ? tab_k[it] : rotary_cos_sin(pos_k[it], f->inv_freq[c]);
        rl = xl * t.x - xh * t.y;
        rh = xh * t.x + xl * t.y;
      }
      ks[e][c] = rl; ks[e][c + HALF] = rh;
      vs[e][c] = __uint_as_float((unsigned)v_lo[it] << 16);
      vs[e][c + HALF] = __uint_as_float((unsigned)v_hi[it] << 16);
    }
  }
  __syncthreads();
  const float2 t_g = !rope ? make_float2(1.0f, 0.0f)
                     : a.table ? a.table[(int64_t)g * HALF + c] : rotary_cos_sin(pos_g, f->inv_freq[c]);
  for (int hl = wave; hl < G; hl += NW) {
    const int head = kvh * G + hl;
    const uint16_t* qr = a.q + (g_row * a.hq + head) * D;
    const unsigned short q_lo = hl == wave ? q_lo0 : qr[c], q_hi = hl == wave ? q_hi0 : qr[c + HALF];
    const float xl = __uint_as_float((unsigned)q_lo << 16), xh = __uint_as_float((unsigned)q_hi << 16);
    const float ql = xl * t_g.x - xh * t_g.y, qh = xh * t_g.x + xl * t_g.y;
    float sc[PV_SHORT_ROW_KEYS];
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < PV_SHORT_ROW_KEYS; ++e) {
      float part = (on && e < n) ? ql * ks[e][c] + qh * ks[e][c + HALF] : 0.0f;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
      sc[e] = e < n ? part * a.scale : -INFINITY;
      m = fmaxf(m, sc[e]);
    }
    float l = 0.0f, ol = 0.0f, oh = 0.0f;
#pragma unroll
    for (int e = 0; e < PV_SHORT_ROW_KEYS; ++e) {
      const float p = expf(sc[e] - m);                  // exp(-inf) = 0 for the unused slots
      l += p;
      if (e < n) {
        ol = fmaf(p, vs[e][c], ol);
        oh = fmaf(p, vs[e][c + HALF], oh);
      }
    }
    if (on) {
      const int64_t row = (g_row * a.hq + head) * D;
      if (a.out_f32) {
        float* op = reinterpret_cast<float*>(a.out) + row;
        op[c] = ol / l; op[c + HALF] = oh / l;
      } else {
        uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + row;
        op[c] = (uint16_t)(pack_bf16(ol / l, 0.0f) & 0xffffu);
        op[c + HALF] = (uint16_t)(pack_bf16(oh / l, 0.0f) & 0xffffu);
      }
      if (a.lse && lane == 0) a.lse[(int64_t)head * h.total_tokens + g_row] = m + logf(l);
    }
  }
}

}  // namespace pv
#endif
