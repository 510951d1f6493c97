// fp32 debug path of pv_masked_attention: plain FMA arithmetic, one thread per (row, q head),
// no tiling.  It exists to check the mask, the positions and the rotary embedding at tight
// tolerance; it is not tuned.
#include "pv_internal.h"

namespace pv {

// cos/sin of pos * inv_freq[c], angle formed and reduced in fp64.
__global__ __launch_bounds__(256) void k_rope_table(const int32_t* plan, PlanHeader h, RopeFreq f,
                                                    int half, float2* cs) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)h.total_tokens * half) return;
  const int g = (int)(idx / half), c = (int)(idx % half);
  const double phi = (double)plan[h.off_pos + g] * f.inv_freq[c];
  double sn, cn;
  sincos(phi, &sn, &cn);
  cs[idx] = make_float2((float)cn, (float)sn);
}

// k_rot is indexed by virtual row (the appended order); k by the caller's row.
__global__ __launch_bounds__(256) void k_rotate_k_f32(const int32_t* plan, PlanHeader h, const float* k,
                                                      const float2* cs, int hkv, int d, int64_t total,
                                                      float* k_rot, bool rope) {
  const int half = d / 2;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (g, head, c)
  if (idx >= total * hkv * half) return;
  const int c = (int)(idx % half);
  const int64_t gh = idx / half;
  const int64_t g = gh / hkv;
  const int64_t src = (caller_row(plan, h, g) * hkv + gh % hkv) * d;
  const float lo = k[src + c], hi = k[src + c + half];
  float2 t = rope ? cs[g * half + c] : make_float2(1.0f, 0.0f);
  k_rot[gh * d + c] = lo * t.x - hi * t.y;
  k_rot[gh * d + c + half] = hi * t.x + lo * t.y;
}

template <int D>
__global__ __launch_bounds__(64) void k_attn_f32(const int32_t* plan, PlanHeader h, const float* q,
                                                 const float* k_rot, const float* v, float* out,
                                                 float* lse, int hq, int hkv, float scale,
                                                 const float2* cs, bool rope) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (g, head)
  if (idx >= (int64_t)h.total_tokens * hq) return;
  const int g = (int)(idx / hq), head = (int)(idx % hq);
  const int kvh = head / (hq / hkv);
  constexpr int HALF = D / 2;

  // request of this row (linear scan is fine for a debug path)
  int b = 0;
  while (plan[h.off_tok_start + b + 1] <= g) ++b;
  const int base = plan[h.off_tok_start + b];
  const int i = g - base;
  const int a_end = plan[h.off_aend + g], b_start = plan[h.off_bstart + g];

  float qr[D];
  const int64_t g_row = caller_row(plan, h, g);        // this row in q / v / out / lse
  const float* qp = q + (g_row * hq + head) * D;
#pragma unroll
  for (int c = 0; c < HALF; ++c) {
    const float lo = qp[c], hi = qp[c + HALF];
    const float2 t = rope ? cs[(int64_t)g * HALF + c] : make_float2(1.0f, 0.0f);
    qr[c] = lo * t.x - hi * t.y;
    qr[c + HALF] = hi * t.x + lo * t.y;
  }
  float acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.0f;
  float m = -INFINITY, l = 0.0f;

  for (int range = 0; range < 2; ++range) {
    const int j0 = range == 0 ? 0 : max(b_start, a_end);
    const int j1 = range == 0 ? a_end : i + 1;
    for (int j = j0; j < j1; ++j) {
      const float* kp = k_rot + ((int64_t)(base + j) * hkv + kvh) * D;
      float s = 0.0f;
#pragma unroll
      for (int c = 0; c < D; ++c) s = fmaf(qr[c], kp[c], s);
      s *= scale;
      const float m_new = fmaxf(m, s);
      const float alpha = expf(m - m_new);      // exp(-inf) = 0 on the first key
      const float p = expf(s - m_new);
      l = l * alpha + p;
      const float* vp = v + (caller_row(plan, h, base + j) * hkv + kvh) * D;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(p, vp[c], acc[c] * alpha);
      m = m_new;
    }
  }
  const float inv = 1.0f / l;
  float* op = out + (g_row * hq + head) * D;
#pragma unroll
  for (int c = 0; c < D; ++c) op[c] = acc[c] * inv;
  if (lse) lse[(int64_t)head * h.total_tokens + g_row] = m + logf(l);
}

hipError_t launch_attn_f32(const int32_t* plan_dev, const PlanHeader& h, const float* q,
                           const float* k, const float* v, float* out, float* lse, int hq,
                           int hkv, int d, float scale, const RopeFreq& freq, bool rope, char* ws,
                           const AttnWorkspace& wl, hipStream_t s) {
  float2* cs = reinterpret_cast<float2*>(ws + wl.off_cs);
  float* k_rot = reinterpret_cast<float*>(ws + wl.off_krot);
  const int half = d / 2;
  hipError_t e;
  dim3 grid;
  if (rope) {
    const int64_t n = (int64_t)h.total_tokens * half;
    if (!grid_1d((n + 255) / 256, 256, &grid)) return hipErrorInvalidConfiguration;
    k_rope_table<<<grid, dim3(256), 0, s>>>(plan_dev, h, freq, half, cs);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    const int64_t n = (int64_t)h.total_tokens * hkv * half;
    if (!grid_1d((n + 255) / 256, 256, &grid)) return hipErrorInvalidConfiguration;
    k_rotate_k_f32<<<grid, dim3(256), 0, s>>>(plan_dev, h, k, cs, hkv, d, h.total_tokens, k_rot, rope);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int64_t n = (int64_t)h.total_tokens * hq;
  if (!grid_1d((n + 63) / 64, 64, &grid)) return hipErrorInvalidConfiguration;
  if (d == 64)
    k_attn_f32<64><<<grid, dim3(64), 0, s>>>(plan_dev, h, q, k_rot, v, out, lse, hq, hkv, scale, cs, rope);
  else
    k_attn_f32<128><<<grid, dim3(64), 0, s>>>(plan_dev, h, q, k_rot, v, out, lse, hq, hkv, scale, cs, rope);
  return hipGetLastError();
}

}  // namespace pv
