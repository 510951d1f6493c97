// bf16 MFMA path of pv_masked_attention for gfx950.
//
// This file: the K/V preparation kernel, the merge kernel and the dispatch; the main kernel itself
// is in pv_attn_bf16_main.h.
//
// Two launches on the caller's stream for the whole pass:
//   k_prep_kv          cos/sin of every token's rotary angle (reduced in fp64, fp32 result), K rotated
//                      and written head-major in MFMA operand order, V written transposed in 16-key
//                      slabs in MFMA operand order, so the main kernel stages both with plain
//                      16-byte copies; extra blocks evaluate the rows with very few keys in fp32
//   k_attn_bf16        flash-style fused Q K^T / online softmax / P V.  One workgroup = one query
//                      tile (32 tokens) x one kv head; wave w owns query head kvh*G + w, so the
//                      G query heads of a GQA group share every K/V tile staged in LDS.
// The segment-only call launches the same kernel over the tiles that hold segment rows, each cut
// along the keys into pieces, and then
//   k_merge_pieces     combines the pieces' unnormalised results.
//
// The product S^T = K Q^T is formed (keys x queries) so that a lane owns one query column:
// row max / row sum are in-lane reductions plus one half-wave exchange, and the rescale factor
// of the online softmax is a per-lane scalar.  O^T = V^T P^T then takes P^T straight from the
// accumulator registers of S^T (the key order inside a slab is chosen to make that a pure
// register repack).
#include "pv_attn_common.h"
#include "pv_short_rows.h"

namespace pv {

// ---------------------------------------------------------------- K/V preparation
// grid = one block per (short row, kv head) first (they take longest, so they start first), then
// blocks of 16 keys x 2 kv heads.  Pad rows (beyond the request) are written as 0 so that masked
// probabilities (exactly 0) never meet a non-finite value.
//   n_short_blocks  short-row blocks in this launch (0: none)
//   key_blocks      whether the launch has key blocks at all (a launch of short rows only has none)
//   tok_first/last  key blocks that hold no token of the packed range [tok_first, tok_last) leave
//                   their part of the workspace as it is (keys prepared by an earlier call)
template <int D>
__global__ __launch_bounds__(256) void k_prep_kv(const int32_t* __restrict__ plan, PlanHeader h,
                                                 KvSource src, RopeFreq f,
                                                 float2* __restrict__ cs, int hkv, bool rope,
                                                 uint16_t* __restrict__ krot,
                                                 uint16_t* __restrict__ vt, ShortRowArgs sr,
                                                 int n_short_blocks, int tok_first, int tok_last) {
  constexpr int HALF = D / 2;
  constexpr int KB = 16;                       // keys per block
  constexpr int HG = 2;                        // kv heads per block
  // one LDS area, used either by a short-row block or by a key block
  constexpr int CS_BYTES = KB * HALF * 8, VS_BYTES = HG * KB * (D / 8 + 1) * 16;
  static_assert(2 * PV_SHORT_ROW_KEYS * D * 4 <= CS_BYTES + VS_BYTES, "short-row tiles must fit");
  __shared__ uint4 lds[(CS_BYTES + VS_BYTES) / 16];
  if ((int)blockIdx.x < n_short_blocks) {      // one (short row, kv head) each
    const int idx = (int)blockIdx.x;
    const int4 desc = reinterpret_cast<const int4*>(plan + h.off_short)[idx / hkv];
    const int kvh = idx % hkv;
    float (*ks)[D] = reinterpret_cast<float (*)[D]>(&lds[0]);
    short_row_block<D, 4>(plan, h, src, &f, hkv, rope, sr, desc, kvh, ks, ks + PV_SHORT_ROW_KEYS);
    return;
  }
  float2 (*cs_s)[HALF] = reinterpret_cast<float2 (*)[HALF]>(&lds[0]);                       // cos/sin of the block's tokens
  uint4 (*v_s)[KB][D / 8 + 1] = reinterpret_cast<uint4 (*)[KB][D / 8 + 1]>(&lds[CS_BYTES / 16]);   // V rows of one pass, padded
  const int n_hg = (hkv + HG - 1) / HG;        // head groups
  const int mb = (int)blockIdx.x - n_short_blocks;
  const int row0 = (mb / n_hg) * KB;           // first padded key row of this block
  const int h0 = (mb % n_hg) * HG;             // first kv head of this block
  const int nh = min(HG, hkv - h0);
  // owner request of the block (requests are padded to multiples of 64 keys)
  const int32_t* kp = plan + h.off_kpad_start;
  int lo = 0, hi = h.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (kp[mid] <= row0) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int tok_base = plan[h.off_tok_start + b];
  const int n_b = plan[h.off_tok_start + b + 1] - tok_base;
  const int key0 = row0 - kp[b];               // first local key of the block
  const int tid = threadIdx.x;
  // Uniform over the workgroup: rows beyond the request's padding (a head stride larger than this
  // plan's key count) are never read; a block with tokens runs if one of them is in the requested
  // range; a block of padding only (zeros, see above) goes with the request's last token.
  if (row0 >= kp[b + 1]) return;
  const int first_tok = tok_base + min(key0, n_b - 1), end_tok = tok_base + min(key0 + KB, n_b);
  if (first_tok >= tok_last || end_tok <= tok_first) return;

  // The K and V rows of the block are requested first, so that their latency overlaps the rotary
  // angles below.  V item = (key, head, 16-byte piece); K item = (key, head, group of 8 rotation
  // pairs): consecutive threads read consecutive 16-byte pieces of a token's row.
  constexpr int VIT = (HG * KB * (D / 8) + 255) / 256, KIT = (HG * KB * (HALF / 8) + 255) / 256;
  uint4 v_reg[VIT], k_lo[KIT], k_hi[KIT];
#pragma unroll
  for (int it = 0; it < VIT; ++it) {
    const int item = tid + it * 256;
    const int ch = item % (D / 8), hl = (item / (D / 8)) % nh, key = item / ((D / 8) * nh);
    v_reg[it] = make_uint4(0, 0, 0, 0);
    if (item < nh * KB * (D / 8) && key0 + key < n_b)
      v_reg[it] = *reinterpret_cast<const uint4*>(
          src.v + (src.row(caller_row(plan, h, tok_base + key0 + key)) * hkv + h0 + hl) * D + ch * 8);
  }
#pragma unroll
  for (int it = 0; it < KIT; ++it) {
    const int item = tid + it * 256;
    const int c0 = (item % (HALF / 8)) * 8, hl = (item / (HALF / 8)) % nh, key = item / ((HALF / 8) * nh);
    k_lo[it] = make_uint4(0, 0, 0, 0);
    k_hi[it] = make_uint4(0, 0, 0, 0);
    if (item < nh * KB * (HALF / 8) && key0 + key < n_b) {
      const uint16_t* kr = src.k + (src.row(caller_row(plan, h, tok_base + key0 + key)) * hkv + h0 + hl) * D;
      k_lo[it] = *reinterpret_cast<const uint4*>(kr + c0);
      k_hi[it] = *reinterpret_cast<const uint4*>(kr + c0 + HALF);
    }
  }
  // cos/sin of the rotary angles (fp64 angle reduced to a fraction of a turn, fp32 result), also
  // written to the table that the main kernel rotates Q with
  if (rope) {
    for (int item = tid; item < KB * HALF; item += 256) {
      const int key = item / HALF, c = item % HALF;
      float2 t = make_float2(1.0f, 0.0f);
      if (key0 + key < n_b) {
        const int64_t g = tok_base + key0 + key;
        t = rotary_cos_sin(plan[h.off_pos + g], f.inv_freq[c]);
        if (h0 == 0) cs[g * HALF + c] = t;
      }
      cs_s[key][c] = t;
    }
  }
  {
#pragma unroll
    for (int it = 0; it < VIT; ++it) {         // V rows into LDS
      const int item = tid + it * 256;
      const int ch = item % (D / 8), hl = (item / (D / 8)) % nh, key = item / ((D / 8) * nh);
      if (item < nh * KB * (D / 8)) v_s[hl][key][ch] = v_reg[it];
    }
    __syncthreads();                           // cs_s and v_s ready
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int item = tid + it * 256;
      if (item >= nh * KB * (HALF / 8)) break;
      const int c0 = (item % (HALF / 8)) * 8, hl = (item / (HALF / 8)) % nh, key = item / ((HALF / 8) * nh);
      uint4 lo4 = k_lo[it], hi4 = k_hi[it];
      if (rope && key0 + key < n_b) {
        const float2* t = &cs_s[key][c0];
        unsigned* pl = reinterpret_cast<unsigned*>(&lo4);
        unsigned* ph = reinterpret_cast<unsigned*>(&hi4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float2 t0 = t[2 * e], t1 = t[2 * e + 1];
          const float l0 = bf16_lo(pl[e]), l1 = bf16_hi(pl[e]);
          const float h0f = bf16_lo(ph[e]), h1f = bf16_hi(ph[e]);
          pl[e] = pack_bf16(l0 * t0.x - h0f * t0.y, l1 * t1.x - h1f * t1.y);
          ph[e] = pack_bf16(h0f * t0.x + l0 * t0.y, h1f * t1.x + l1 * t1.y);
        }
      }
      // operand order: inside a block of 32 keys, chunk (t, hh, row) = features 16 t + 8 hh .. + 7
      // of key `row` sits at chunk index t * 64 + hh * 32 + row
      const int prow = row0 + key;             // padded key row
      uint4* dst = reinterpret_cast<uint4*>(krot + ((int64_t)(h0 + hl) * h.padded_keys + (prow & ~31)) * D) + (prow & 31);
      const int ci = c0 >> 3;                  // chunk of the low half; the high one is D/16 later
      dst[(ci >> 1) * 64 + (ci & 1) * 32] = lo4;
      dst[((ci + D / 16) >> 1) * 64 + ((ci + D / 16) & 1) * 32] = hi4;
    }
    // V^T: a slab (16 keys) is [2][D][8]; element (hh, d, m) is key 8*(m/4) + 4*hh + (m%4) of the
    // slab at feature d.  Item = one 16-byte chunk (head, hh, d).
    constexpr int VROW = (D / 8 + 1) * 8;      // padded row length in elements
    for (int item = tid; item < nh * 2 * D; item += 256) {
      const int d = item % D, hh = (item / D) % 2, hl = item / (2 * D);
      const uint16_t* vs16 = reinterpret_cast<const uint16_t*>(&v_s[hl][0][0]);
      unsigned short e[8];
#pragma unroll
      for (int m = 0; m < 8; ++m) e[m] = vs16[(8 * (m / 4) + 4 * hh + (m % 4)) * VROW + d];
      uint4 o;
      o.x = e[0] | ((unsigned)e[1] << 16); o.y = e[2] | ((unsigned)e[3] << 16);
      o.z = e[4] | ((unsigned)e[5] << 16); o.w = e[6] | ((unsigned)e[7] << 16);
      reinterpret_cast<uint4*>(vt + ((int64_t)(h0 + hl) * h.padded_keys + row0) * D)[hh * D + d] = o;
    }
  }
}

// Merge of the key pieces of the segment-only call.  One workgroup per (tile holding segment rows,
// query head); 8 threads per row, each D/8 features.  Piece c holds, relative to its own reference
// mref_c = -nmref_c (log2 units), the unnormalised O_c and the row sum l_c; with M = max mref_c over
// the pieces that saw a key, O = sum_c 2^(mref_c - M) O_c / sum_c 2^(mref_c - M) l_c.
template <int D>
__global__ __launch_bounds__(256) void k_merge_pieces(const int32_t* __restrict__ plan, PlanHeader h,
                                                      const float* __restrict__ part, int split,
                                                      void* __restrict__ out, float* __restrict__ lse,
                                                      int hq, int hkv, bool out_f32) {
  constexpr int MAXSPLIT = 8, FPT = D / 8;           // features per thread
  const int G = hq / hkv;
  const int item = (int)blockIdx.x / G, hl = (int)blockIdx.x % G;     // (tile, kv head), head of group
  const int kvh = item % hkv, head = kvh * G + hl;
  const QTile tile = reinterpret_cast<const QTile*>(plan + h.off_segwork)[item / hkv];
  const int row = threadIdx.x >> 3, sub = threadIdx.x & 7;
  if (row >= tile.rows) return;
  const int64_t g = (int64_t)tile.tok_base + tile.t0 + row;
  const int a_end = plan[h.off_aend + g], b_start = plan[h.off_bstart + g];
  const int i_loc = tile.t0 + row;
  // segment rows only; rows with few keys come from the preparation kernel
  if (b_start == 0 || a_end + i_loc - b_start + 1 <= PV_SHORT_ROW_KEYS) return;
  float mref[MAXSPLIT], lsum[MAXSPLIT];
  float M = -INFINITY;
#pragma unroll
  for (int c = 0; c < MAXSPLIT; ++c) {
    mref[c] = 0.0f; lsum[c] = 0.0f;
    if (c < split) {
      const float* p = part + ((int64_t)((int64_t)item * split + c) * G + hl) * (32 * (D + 2));
      const float2 ml = reinterpret_cast<const float2*>(p + 32 * D)[row];
      mref[c] = -ml.x; lsum[c] = ml.y;
      if (ml.y > 0.0f) M = fmaxf(M, mref[c]);
    }
  }
  float acc[FPT];
#pragma unroll
  for (int e = 0; e < FPT; ++e) acc[e] = 0.0f;
  float L = 0.0f;
#pragma unroll
  for (int c = 0; c < MAXSPLIT; ++c) {
    if (c < split && lsum[c] > 0.0f) {               // a piece without a visible key holds nothing
      const float w = exp2f(mref[c] - M);
      L = fmaf(w, lsum[c], L);
      const float* p = part + ((int64_t)((int64_t)item * split + c) * G + hl) * (32 * (D + 2)) +
                       row * D + sub * FPT;
#pragma unroll
      for (int e = 0; e < FPT; e += 4) {
        const float4 x = *reinterpret_cast<const float4*>(p + e);
        acc[e] = fmaf(w, x.x, acc[e]); acc[e + 1] = fmaf(w, x.y, acc[e + 1]);
        acc[e + 2] = fmaf(w, x.z, acc[e + 2]); acc[e + 3] = fmaf(w, x.w, acc[e + 3]);
      }
    }
  }
  const float inv = 1.0f / L;
  const int64_t orow = (caller_row(plan, h, g) * hq + head) * D + sub * FPT;
  if (out_f32) {
    float* op = reinterpret_cast<float*>(out) + orow;
#pragma unroll
    for (int e = 0; e < FPT; e += 4)
      *reinterpret_cast<float4*>(op + e) =
          make_float4(acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv);
  } else {
    uint16_t* op = reinterpret_cast<uint16_t*>(out) + orow;
#pragma unroll
    for (int e = 0; e < FPT; e += 4) {
      uint2 w;
      w.x = pack_bf16(acc[e] * inv, acc[e + 1] * inv);
      w.y = pack_bf16(acc[e + 2] * inv, acc[e + 3] * inv);
      *reinterpret_cast<uint2*>(op + e) = w;
    }
  }
  if (lse && sub == 0)
    lse[(int64_t)head * h.total_tokens + caller_row(plan, h, g)] = (log2f(L) + M) * 0.6931471805599453f;
}

// The main kernel's launchers: defined in pv_attn_bf16_main.h, instantiated in the translation units
// built from pv_attn_bf16_inst.hip.
template <int D, int G>
hipError_t launch_main(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                       const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                       float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                       int split, float* part, const KvSource& raw_kv, float scale, int n_short,
                       hipStream_t s);
template <int D>
hipError_t launch_query_tiles(const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                              const uint16_t* krot, const uint16_t* vt, const float2* cs,
                              void* out, float* lse, int hq, int hkv, float qscale, bool rope,
                              bool out_f32, const KvSource& raw_kv, float scale, int n_short,
                              hipStream_t s);

template <int D>
static hipError_t dispatch_g(int G, const int32_t* plan, const PlanHeader& h, const uint16_t* q,
                             const uint16_t* krot, const uint16_t* vt, const float2* cs, void* out,
                             float* lse, int hq, int hkv, float qscale, bool rope, bool out_f32,
                             int split, float* part, const KvSource& raw_kv, float scale, int n_short,
                             hipStream_t s) {
  if (split == 0 && group_uses_query_tiles(G) && h.n_quads > 0)
    return launch_query_tiles<D>(plan, h, q, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, raw_kv,
                                 scale, n_short, s);
  switch (G) {
#define PV_CASE(GG) case GG: return launch_main<D, GG>(plan, h, q, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, split, part, raw_kv, scale, n_short, s);
    PV_CASE(1) PV_CASE(2) PV_CASE(3) PV_CASE(4) PV_CASE(5) PV_CASE(6) PV_CASE(7) PV_CASE(8)
#undef PV_CASE
  }
  return hipErrorInvalidValue;
}

// K/V preparation (key blocks of the token range, and the short rows unless sr.q is null).
hipError_t launch_prep_bf16(const int32_t* plan_dev, const PlanHeader& h, const KvArgs& kv, int hkv, int d,
                            const RopeFreq& freq, bool rope, char* ws, const AttnWorkspace& wl,
                            bool key_blocks, int64_t tok_first, int64_t tok_last, const void* q, void* out,
                            float* lse, int hq, float scale, bool out_f32, bool segments_only,
                            hipStream_t s) {
  float2* cs = reinterpret_cast<float2*>(ws + wl.off_cs);
  uint16_t* krot = reinterpret_cast<uint16_t*>(ws + wl.off_krot);
  uint16_t* vt = reinterpret_cast<uint16_t*>(ws + wl.off_vt);
  KvSource src;
  src.k = reinterpret_cast<const uint16_t*>(kv.k);
  src.v = reinterpret_cast<const uint16_t*>(kv.v);
  src.block_table = kv.block_table;
  src.page_size = kv.page_size;
  ShortRowArgs sr;
  sr.q = reinterpret_cast<const uint16_t*>(q); sr.out = out; sr.lse = lse; sr.hq = hq; sr.scale = scale;
  sr.out_f32 = out_f32; sr.seg_only = segments_only; sr.table = nullptr;
  const int64_t n_short = q ? (int64_t)h.n_short_rows * hkv : 0;
  const int64_t n_key = key_blocks ? (int64_t)(h.padded_keys / 16) * ((hkv + 1) / 2) : 0;
  if (n_short + n_key == 0) return hipSuccess;
  dim3 grid;
  if (!grid_1d(n_short + n_key, 256, &grid) || n_short > 0x7fffffff) return hipErrorInvalidConfiguration;
  const int t0 = (int)tok_first, t1 = (int)tok_last;
  if (d == 64) k_prep_kv<64><<<grid, dim3(256), 0, s>>>(plan_dev, h, src, freq, cs, hkv, rope, krot, vt, sr, (int)n_short, t0, t1);
  else k_prep_kv<128><<<grid, dim3(256), 0, s>>>(plan_dev, h, src, freq, cs, hkv, rope, krot, vt, sr, (int)n_short, t0, t1);
  return hipGetLastError();
}

// True when the main kernel's launch can carry the rows with few keys itself (as extra workgroups of
// at least four waves at the end of a whole-pass grid).
bool main_kernel_takes_short_rows(const PlanHeader& h, int hq, int hkv, bool segments_only) {
  const int G = hq / hkv;
  if (segments_only || h.n_short_rows == 0) return false;
  return (group_uses_query_tiles(G) && h.n_quads > 0) || G >= 4;
}

// The main kernel over prepared keys (and the merge of the key pieces of the segment-only call).
// short_rows_kv != nullptr: the launch also evaluates the rows with few keys from these K/V tensors.
hipError_t launch_main_bf16(const int32_t* plan_dev, const PlanHeader& h, const void* q, void* out,
                            float* lse, int hq, int hkv, int d, int out_dtype, float scale, bool rope,
                            char* ws, const AttnWorkspace& wl, bool segments_only,
                            const KvArgs* short_rows_kv, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s) {
  if (segments_only && h.n_seg_tiles == 0) return hipSuccess;          // no segment anywhere
  float2* cs = reinterpret_cast<float2*>(ws + wl.off_cs);
  uint16_t* krot = reinterpret_cast<uint16_t*>(ws + wl.off_krot);
  uint16_t* vt = reinterpret_cast<uint16_t*>(ws + wl.off_vt);
  float* part = reinterpret_cast<float*>(ws + wl.off_part);
  const uint16_t* kq = reinterpret_cast<const uint16_t*>(q);
  const bool out_f32 = out_dtype == PV_F32;
  hipError_t e;
  const float qscale = scale * 1.4426950408889634f;
  const int split = segments_only ? wl.split : 0;
  KvSource raw_kv = {nullptr, nullptr, nullptr, 1};
  int64_t n_short = 0;
  if (short_rows_kv) {
    raw_kv.k = reinterpret_cast<const uint16_t*>(short_rows_kv->k);
    raw_kv.v = reinterpret_cast<const uint16_t*>(short_rows_kv->v);
    raw_kv.block_table = short_rows_kv->block_table;
    raw_kv.page_size = short_rows_kv->page_size;
    n_short = (int64_t)h.n_short_rows * hkv;
    if (n_short > 0x7fffffff) return hipErrorInvalidConfiguration;
  }
  if (ev0) { e = hipEventRecord(ev0, s); if (e != hipSuccess) return e; }
  if (d == 64) e = dispatch_g<64>(hq / hkv, plan_dev, h, kq, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, split, part, raw_kv, scale, (int)n_short, s);
  else e = dispatch_g<128>(hq / hkv, plan_dev, h, kq, krot, vt, cs, out, lse, hq, hkv, qscale, rope, out_f32, split, part, raw_kv, scale, (int)n_short, s);
  if (e != hipSuccess) return e;
  if (ev1) { e = hipEventRecord(ev1, s); if (e != hipSuccess) return e; }
  if (split > 1) {
    dim3 grid;
    if (!grid_1d((int64_t)h.n_seg_tiles * hq, 256, &grid)) return hipErrorInvalidConfiguration;
    if (d == 64) k_merge_pieces<64><<<grid, dim3(256), 0, s>>>(plan_dev, h, part, split, out, lse, hq, hkv, out_f32);
    else k_merge_pieces<128><<<grid, dim3(256), 0, s>>>(plan_dev, h, part, split, out, lse, hq, hkv, out_f32);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace pv
