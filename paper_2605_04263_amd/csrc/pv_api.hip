// C ABI of the library: argument validation on the host, then kernel launches on the caller's
// stream.  Nothing here allocates device memory or synchronises (pv_profile_read excepted).
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "pv_internal.h"

namespace pv {

static thread_local int32_t g_last_hip = 0;
// Profiling state, all of it under g_profile_lock.
static std::mutex g_profile_lock;
static bool g_profile = false;
static hipEvent_t g_ev[PV_PROFILE_RING][2];     // created on first use, destroyed when profiling is switched off
static int64_t g_ev_calls = 0;                  // calls recorded since profiling was enabled

// Workspace of pv_masked_attention_static: part of the library's device image, one copy per GPU at an
// address of its own.  In host code this name is only a handle for hipGetSymbolAddress; the address
// looked up there (per device) is what kernels and host calls are given.
static __device__ __align__(256) unsigned char scratch[PV_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void* g_scratch_ptr[kMaxDevices];        // per device, filled on first use with that device current

static inline pv_status hip_fail(hipError_t e) {
  g_last_hip = (int32_t)e;
  return PV_ERR_HIP;
}

static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

void plan_layout(int batch, int64_t total_tokens, int64_t total_segments, int64_t n_q_tiles,
                 int64_t padded_keys, int64_t n_short_rows, int layout, int64_t n_seg_tiles,
                 int64_t n_quads, PlanHeader* h) {
  std::memset(h, 0, sizeof(*h));
  h->magic = kPlanMagic;
  h->batch = batch;
  h->total_tokens = (int32_t)total_tokens;
  h->total_segments = (int32_t)total_segments;
  h->n_q_tiles = (int32_t)n_q_tiles;
  h->tile_m = kTileM;
  h->tile_n = kTileN;
  h->padded_keys = (int32_t)padded_keys;
  h->n_short_rows = (int32_t)n_short_rows;
  h->layout = layout;
  h->n_seg_tiles = (int32_t)n_seg_tiles;
  h->n_quads = (int32_t)n_quads;
  int64_t o = sizeof(PlanHeader) / 4;
  auto take = [&](int64_t n) { int64_t r = o; o = align_up(o + n, 4); return (int32_t)r; };
  h->off_prompt = take(batch);
  h->off_draft = take(batch);
  h->off_nseg = take(batch);
  h->off_seglen = take(batch);
  h->off_tok_start = take(batch + 1);
  h->off_seg_start = take(batch + 1);
  h->off_qtile_start = take(batch + 1);
  h->off_kpad_start = take(batch + 1);
  h->off_mask_start = take(2 * (int64_t)(batch + 1));
  h->off_bounds = take(total_segments);
  h->off_short = take(4 * n_short_rows);
  h->off_segtile_start = take(batch + 1);
  h->off_quad_start = take(batch + 1);
  h->off_device_begin = (int32_t)o;
  h->off_pos = take(total_tokens);
  h->off_aend = take(total_tokens);
  h->off_bstart = take(total_tokens);
  h->off_judge = take(total_segments);
  h->off_tiles = take(n_q_tiles * 8);
  h->off_work = take(n_q_tiles * 8);
  h->off_map = layout == PV_LAYOUT_INTERLEAVED ? take(total_tokens) : 0;
  h->off_segwork = take(n_seg_tiles * 8);
  h->off_quadwork = take(n_quads * 8);
  h->total_ints = (int32_t)o;
}

// Pieces per work item of the segment-only call: enough to give every workgroup slot of the chip
// (256 compute units x 2) an item, at most 8.
static int segment_split(int64_t n_seg_tiles, int hkv) {
  const int64_t items = n_seg_tiles * hkv;
  if (items <= 0) return 1;
  int64_t c = (512 + items - 1) / items;
  return (int)(c < 1 ? 1 : (c > 8 ? 8 : c));
}

AttnWorkspace attn_workspace_layout(int64_t total_tokens, int64_t padded_keys, int64_t n_seg_tiles,
                                    int hq, int hkv, int d, int in_dtype) {
  AttnWorkspace w;
  w.off_part = 0;
  w.split = 1;
  int64_t o = 0;
  w.off_cs = o;
  o = align_up(o + total_tokens * (d / 2) * 8, 256);
  w.off_krot = o;
  if (in_dtype == PV_BF16) {
    o = align_up(o + (int64_t)hkv * padded_keys * d * 2, 256);
    w.off_vt = o;
    o = align_up(o + (int64_t)hkv * padded_keys * d * 2, 256);
    w.split = segment_split(n_seg_tiles, hkv);
    w.off_part = o;
    w.total_full = o;
    if (w.split > 1) o = align_up(o + n_seg_tiles * hq * w.split * 32 * (d + 2) * 4, 256);
  } else {
    o = align_up(o + total_tokens * hkv * d * 4, 256);
    w.off_vt = o;
    w.total_full = o;
  }
  w.total = o;
  return w;
}

struct Totals {
  int64_t tokens = 0, segments = 0, max_len = 0, q_tiles = 0, padded_keys = 0, mask_bytes = 0;
  int64_t short_rows = 0, short_seg_rows = 0, seg_tiles = 0, quads = 0;
};

// Rows of request (P, T, S, boundaries) that see at most PV_SHORT_ROW_KEYS keys: the first causal
// rows, and rows of segments whose visible prefix is nearly empty.  Calls f(local_row).
template <typename F>
static void for_each_short_row(int64_t P, int64_t T, int64_t K, int64_t S, const int32_t* bounds, F f) {
  const int64_t c = P + T;
  for (int64_t i = 0; i < c && i + 1 <= PV_SHORT_ROW_KEYS; ++i) f(i);
  for (int64_t k = 0; k < K; ++k)
    for (int64_t a = 0; a < S && P + bounds[k] + a + 1 <= PV_SHORT_ROW_KEYS; ++a) f(c + k * S + a);
}

// Validates the problem; fills totals.  Limits keep every index inside int32.
static pv_status validate_problem(const pv_problem* p, Totals* t) {
  if (!p) return PV_ERR_NULL;
  if (p->batch < 1 || p->batch > (1 << 20)) return PV_ERR_SHAPE;
  if (p->layout != PV_LAYOUT_APPENDED && p->layout != PV_LAYOUT_INTERLEAVED) return PV_ERR_SHAPE;
  if (!p->prompt_len || !p->draft_len || !p->num_segments || !p->segment_len) return PV_ERR_NULL;
  int64_t nseg = 0;
  for (int b = 0; b < p->batch; ++b) {
    if (p->num_segments[b] < 0) return PV_ERR_SHAPE;
    nseg += p->num_segments[b];
  }
  if (nseg > 0 && !p->boundaries) return PV_ERR_NULL;
  int64_t seg = 0;
  for (int b = 0; b < p->batch; ++b) {
    const int64_t P = p->prompt_len[b], T = p->draft_len[b], K = p->num_segments[b],
                  S = p->segment_len[b];
    if (P < 0 || T < 1 || S < 1) return PV_ERR_SHAPE;
    const int64_t n = P + T + K * S;
    if (n > (1 << 24)) return PV_ERR_SHAPE;
    int64_t prev = 0;
    for (int64_t k = 0; k < K; ++k) {
      const int64_t pk = p->boundaries[seg + k];
      if (pk < prev || pk > T) return PV_ERR_BOUNDARY;
      prev = pk;
    }
    for_each_short_row(P, T, K, S, p->boundaries + seg, [&](int64_t i) {
      t->short_rows++;
      if (i >= P + T) t->short_seg_rows++;
    });
    seg += K;
    t->tokens += n;
    t->max_len = n > t->max_len ? n : t->max_len;
    t->q_tiles += (n + kTileM - 1) / kTileM;
    t->quads += ((n + kTileM - 1) / kTileM + 3) / 4;
    if (K > 0) t->seg_tiles += (n + kTileM - 1) / kTileM - (P + T) / kTileM;
    t->padded_keys += align_up(n, kTileN);
    t->mask_bytes += n * n;
  }
  t->segments = nseg;
  if (t->tokens > (1ll << 27) || t->padded_keys > (1ll << 27)) return PV_ERR_SHAPE;
  return PV_OK;
}

static pv_status validate_heads(int hq, int hkv, int d, int in_dtype) {
  if (in_dtype != PV_BF16 && in_dtype != PV_F32) return PV_ERR_DTYPE;
  if (hq < 1 || hkv < 1 || hq % hkv != 0 || hq / hkv > 8 || hq > 1024) return PV_ERR_SHAPE;
  if (d != 64 && d != 128) return PV_ERR_SHAPE;
  return PV_OK;
}

static void fill_sizes(const pv_problem* p, const Totals& t, int hq, int hkv, int d, int in_dtype,
                       pv_sizes* s) {
  std::memset(s, 0, sizeof(*s));
  s->batch = p->batch;
  s->total_tokens = t.tokens;
  s->total_segments = t.segments;
  s->max_seq_len = t.max_len;
  s->n_q_tiles = t.q_tiles;
  s->padded_keys = t.padded_keys;
  PlanHeader h;
  plan_layout(p->batch, t.tokens, t.segments, t.q_tiles, t.padded_keys, t.short_rows, p->layout,
              t.seg_tiles, group_uses_query_tiles(hq / hkv) ? t.quads : 0, &h);
  s->n_seg_tiles = (int32_t)t.seg_tiles;
  s->n_quads = h.n_quads;
  s->n_short_rows = (int32_t)t.short_rows;
  s->n_short_seg_rows = (int32_t)t.short_seg_rows;
  s->layout = p->layout;
  s->plan_bytes = (int64_t)h.total_ints * 4;
  s->dense_mask_bytes = t.mask_bytes;
  s->attn_workspace_bytes =
      attn_workspace_layout(t.tokens, t.padded_keys, t.seg_tiles, hq, hkv, d, in_dtype).total;
  s->n_q_heads = hq;
  s->n_kv_heads = hkv;
  s->head_dim = d;
  s->in_dtype = in_dtype;
  s->tile_m = kTileM;
  s->tile_n = kTileN;
}

// A pv_sizes is trusted only if it is self-consistent with the layout functions.
static pv_status check_sizes(const pv_sizes* s, PlanHeader* h) {
  if (!s) return PV_ERR_NULL;
  if (s->batch < 1 || s->total_tokens < 1 || s->total_segments < 0 || s->n_q_tiles < 1 ||
      s->tile_m != kTileM || s->tile_n != kTileN || s->padded_keys < s->total_tokens ||
      s->n_short_rows < 0 || s->n_short_rows > s->total_tokens || s->n_short_seg_rows < 0 ||
      s->n_short_seg_rows > s->n_short_rows)
    return PV_ERR_SHAPE;
  // the limits pv_query_sizes enforces: every index and offset of the plan stays inside int32
  if (s->batch > (1 << 20) || s->total_tokens > (1ll << 27) || s->padded_keys > (1ll << 27) ||
      s->total_segments > s->total_tokens || s->n_q_tiles > s->total_tokens || s->n_seg_tiles < 0 ||
      s->n_seg_tiles > s->n_q_tiles || s->n_quads < 0 || s->n_quads > s->n_q_tiles)
    return PV_ERR_SHAPE;
  if (validate_heads(s->n_q_heads, s->n_kv_heads, s->head_dim, s->in_dtype) != PV_OK)
    return PV_ERR_SHAPE;
  if (s->layout != PV_LAYOUT_APPENDED && s->layout != PV_LAYOUT_INTERLEAVED) return PV_ERR_SHAPE;
  plan_layout((int)s->batch, s->total_tokens, s->total_segments, s->n_q_tiles, s->padded_keys,
              s->n_short_rows, s->layout, s->n_seg_tiles, s->n_quads, h);
  if (s->plan_bytes != (int64_t)h->total_ints * 4) return PV_ERR_SHAPE;
  return PV_OK;
}

static inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

static pv_status check_arch() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return hip_fail(e);
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return PV_ERR_ARCH;
  return PV_OK;
}

static pv_status arch_ok_cached() {
  static thread_local int cached_dev = -1;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev == cached_dev) return PV_OK;
  pv_status st = check_arch();
  if (st == PV_OK) cached_dev = dev;
  return st;
}

}  // namespace pv

using namespace pv;

extern "C" {

pv_status pv_query_sizes(const pv_problem* problem, int32_t n_q_heads, int32_t n_kv_heads,
                         int32_t head_dim, int32_t in_dtype, pv_sizes* out) {
  if (!out) return PV_ERR_NULL;
  Totals t;
  pv_status st = validate_problem(problem, &t);
  if (st != PV_OK) return st;
  st = validate_heads(n_q_heads, n_kv_heads, head_dim, in_dtype);
  if (st != PV_OK) return st;
  fill_sizes(problem, t, n_q_heads, n_kv_heads, head_dim, in_dtype, out);
  return PV_OK;
}

pv_status pv_build_mask(const pv_problem* problem, const pv_sizes* sizes, void* plan_dev,
                        int64_t plan_bytes, uint8_t* dense_mask_dev, int64_t dense_mask_bytes,
                        void* stream) {
  Totals t;
  pv_status st = validate_problem(problem, &t);
  if (st != PV_OK) return st;
  PlanHeader h;
  st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (sizes->batch != problem->batch || sizes->total_tokens != t.tokens ||
      sizes->total_segments != t.segments || sizes->n_q_tiles != t.q_tiles ||
      sizes->padded_keys != t.padded_keys || sizes->dense_mask_bytes != t.mask_bytes ||
      sizes->n_short_rows != t.short_rows || sizes->n_short_seg_rows != t.short_seg_rows ||
      sizes->layout != problem->layout ||
      sizes->n_seg_tiles != t.seg_tiles ||
      sizes->n_quads != (group_uses_query_tiles(sizes->n_q_heads / sizes->n_kv_heads) ? t.quads : 0))
    return PV_ERR_SHAPE;
  if (!plan_dev) return PV_ERR_NULL;
  if (plan_bytes < sizes->plan_bytes) return PV_ERR_WORKSPACE;
  if (dense_mask_dev && dense_mask_bytes < sizes->dense_mask_bytes) return PV_ERR_WORKSPACE;
  if (misaligned(plan_dev)) return PV_ERR_ALIGN;

  // Host image of the uploaded part of the plan: header, per-request arrays, boundaries.
  std::vector<int32_t> img;
  try {
    img.assign((size_t)h.off_device_begin, 0);
  } catch (const std::bad_alloc&) {               // no exception may cross the C boundary
    return PV_ERR_WORKSPACE;
  }
  std::memcpy(img.data(), &h, sizeof(h));
  const int B = problem->batch;
  int64_t tok = 0, seg = 0, qt = 0, kp = 0, mk = 0, ns = 0, sgt = 0, qd = 0;
  int64_t* mask_start = reinterpret_cast<int64_t*>(img.data() + h.off_mask_start);
  for (int b = 0; b <= B; ++b) {
    img[h.off_tok_start + b] = (int32_t)tok;
    img[h.off_seg_start + b] = (int32_t)seg;
    img[h.off_qtile_start + b] = (int32_t)qt;
    img[h.off_kpad_start + b] = (int32_t)kp;
    mask_start[b] = mk;
    img[h.off_segtile_start + b] = (int32_t)sgt;
    img[h.off_quad_start + b] = (int32_t)qd;
    if (b == B) break;
    const int64_t P = problem->prompt_len[b], T = problem->draft_len[b],
                  K = problem->num_segments[b], S = problem->segment_len[b];
    const int64_t n = P + T + K * S;
    img[h.off_prompt + b] = (int32_t)P;
    img[h.off_draft + b] = (int32_t)T;
    img[h.off_nseg + b] = (int32_t)K;
    img[h.off_seglen + b] = (int32_t)S;
    for (int64_t k = 0; k < K; ++k) img[h.off_bounds + seg + k] = problem->boundaries[seg + k];
    // A short row carries its descriptor with it (the same values the plan kernels write for the
    // row), so that the blocks evaluating it start from one load instead of a chain of three.
    for_each_short_row(P, T, K, S, problem->boundaries + seg, [&](int64_t i) {
      int32_t* e = &img[h.off_short + 4 * ns++];
      const int64_t c = P + T;
      const int64_t k = i < c ? 0 : (i - c) / S;
      e[0] = (int32_t)(tok + i);
      e[1] = (int32_t)tok;
      e[2] = i < c ? 0 : (int32_t)(P + problem->boundaries[seg + k]);
      e[3] = i < c ? 0 : (int32_t)(c + k * S);
    });
    tok += n;
    seg += K;
    qt += (n + kTileM - 1) / kTileM;
    qd += ((n + kTileM - 1) / kTileM + 3) / 4;
    if (K > 0) sgt += (n + kTileM - 1) / kTileM - (P + T) / kTileM;
    kp += align_up(n, kTileN);
    mk += n * n;
  }

  st = arch_ok_cached();
  if (st != PV_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = launch_plan_kernels((int32_t*)plan_dev, h, img.data(), (int)img.size(),
                                     dense_mask_dev, s);
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

// What an attention call does: prepare the keys (rotary table, rotated K, transposed V in the
// workspace), run the main kernel over prepared keys (with the fp32 evaluation of the short rows), or
// both.
enum { kPhasePrepare = 1, kPhaseAttend = 2 };

static pv_status attention_call(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                const void* k, const void* v, void* out, float* lse,
                                int32_t out_dtype, float softmax_scale, float rope_theta,
                                void* workspace, int64_t workspace_bytes, void* stream,
                                bool segments_only, bool library_workspace = false,
                                int phases = kPhasePrepare | kPhaseAttend,
                                const int32_t* block_table = nullptr, int32_t page_size = 0,
                                int64_t tok_first = 0, int64_t tok_last = -1,
                                int64_t key_capacity = 0) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  // Prepared keys shared by calls under different plans: the per-head stride of the workspace is
  // the caller's capacity instead of this plan's padded key count.
  // (an explicit capacity always selects the capacity-based layout, so that every pass that names the
  // same capacity finds the same offsets, also the pass whose own key count equals it)
  const bool own_stride = key_capacity != 0;
  if (key_capacity == 0) key_capacity = sizes->padded_keys;
  if (key_capacity < sizes->padded_keys || key_capacity % kTileN != 0 || key_capacity > (1ll << 27))
    return PV_ERR_SHAPE;
  const bool attend = (phases & kPhaseAttend) != 0, prepare = (phases & kPhasePrepare) != 0;
  if (!plan_dev || !k || !v || !workspace) return PV_ERR_NULL;
  if (attend && (!q || !out)) return PV_ERR_NULL;
  if (out_dtype != PV_BF16 && out_dtype != PV_F32) return PV_ERR_DTYPE;
  if (sizes->in_dtype == PV_F32 && out_dtype != PV_F32) return PV_ERR_DTYPE;
  if ((segments_only || phases != (kPhasePrepare | kPhaseAttend)) && sizes->in_dtype != PV_BF16)
    return PV_ERR_DTYPE;
  if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return PV_ERR_SHAPE;
  if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return PV_ERR_SHAPE;
  if (block_table && page_size < 1) return PV_ERR_SHAPE;
  if (tok_last < 0) tok_last = sizes->total_tokens;
  if (tok_first < 0 || tok_first > tok_last || tok_last > sizes->total_tokens) return PV_ERR_SHAPE;
  const int hq = sizes->n_q_heads, hkv = sizes->n_kv_heads, d = sizes->head_dim;
  const AttnWorkspace wl =
      attn_workspace_layout(own_stride ? key_capacity : sizes->total_tokens, key_capacity,
                            sizes->n_seg_tiles, hq, hkv, d, sizes->in_dtype);
  h.padded_keys = (int32_t)key_capacity;          // the kernels take the head stride from their copy of the header
  // a caller's workspace must have the size pv_query_sizes reports (which also covers the
  // segment-only call); the library's own fixed array only has to hold what the whole pass uses
  if (workspace_bytes < (library_workspace ? wl.total_full : wl.total)) return PV_ERR_WORKSPACE;
  if (misaligned(plan_dev) || misaligned(q) || misaligned(k) || misaligned(v) ||
      misaligned(out) || misaligned(workspace) || ((uintptr_t)lse & 3u) || ((uintptr_t)block_table & 3u))
    return PV_ERR_ALIGN;
  st = arch_ok_cached();
  if (st != PV_OK) return st;

  const float scale = softmax_scale == 0.0f ? (float)(1.0 / std::sqrt((double)d)) : softmax_scale;
  RopeFreq freq;
  const bool rope = rope_theta > 0.0f;
  for (int c = 0; c < 64; ++c)
    freq.inv_freq[c] =
        (rope && c < d / 2) ? std::pow((double)rope_theta, -2.0 * (double)c / (double)d) : 0.0;

  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  if (sizes->in_dtype == PV_F32) {
    e = launch_attn_f32((const int32_t*)plan_dev, h, (const float*)q, (const float*)k,
                        (const float*)v, (float*)out, lse, hq, hkv, d, scale, freq, rope,
                        (char*)workspace, wl, s);
  } else {
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    std::unique_lock<std::mutex> guard(g_profile_lock);
    const bool profiling = g_profile && attend;
    if (profiling) {
      hipEvent_t* pair = g_ev[g_ev_calls % PV_PROFILE_RING];
      if (!pair[0]) {
        e = hipEventCreate(&pair[0]);
        if (e != hipSuccess) { pair[0] = nullptr; return hip_fail(e); }
      }
      if (!pair[1]) {
        e = hipEventCreate(&pair[1]);
        if (e != hipSuccess) { pair[1] = nullptr; return hip_fail(e); }
      }
      ev0 = pair[0];
      ev1 = pair[1];
    } else {
      guard.unlock();                               // the ordinary path holds no lock while launching
    }
    // One preparation launch: the key blocks (if asked for) and, when the main kernel follows and
    // cannot take them itself, the rows with few keys in fp32.  A whole pass that prepares all its
    // keys in this call (so that the table of rotary angles is complete) leaves them to the main
    // kernel, where they run as extra workgroups in the tail of the launch.
    KvArgs kv;
    kv.k = k; kv.v = v; kv.block_table = block_table; kv.page_size = page_size;
    const bool short_in_main = attend && prepare && tok_first == 0 && tok_last == sizes->total_tokens &&
                               main_kernel_takes_short_rows(h, hq, hkv, segments_only);
    e = launch_prep_bf16((const int32_t*)plan_dev, h, kv, hkv, d, freq, rope, (char*)workspace, wl,
                         prepare, tok_first, tok_last,
                         // a segment-only pass has no short rows to do unless a segment sees almost nothing
                         attend && !short_in_main && (!segments_only || sizes->n_short_seg_rows > 0) ? q : nullptr,
                         out, lse, hq, scale, out_dtype == PV_F32, segments_only, s);
    if (e == hipSuccess && attend)
      e = launch_main_bf16((const int32_t*)plan_dev, h, q, out, lse, hq, hkv, d, out_dtype, scale, rope,
                           (char*)workspace, wl, segments_only, short_in_main ? &kv : nullptr, ev0, ev1, s);
    if (e == hipSuccess && profiling) ++g_ev_calls;
  }
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_masked_attention(const pv_sizes* sizes, const void* plan_dev, const void* q,
                              const void* k, const void* v, void* out, float* lse,
                              int32_t out_dtype, float softmax_scale, float rope_theta,
                              void* workspace, int64_t workspace_bytes, void* stream) {
  return attention_call(sizes, plan_dev, q, k, v, out, lse, out_dtype, softmax_scale, rope_theta,
                        workspace, workspace_bytes, stream, false);
}

// Address of this device's copy of `scratch` (looked up once per device, with that device current).
static pv_status static_workspace(void** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return PV_ERR_SHAPE;
  std::lock_guard<std::mutex> guard(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!p) return hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return PV_OK;
}

pv_status pv_masked_attention_static(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                     const void* k, const void* v, void* out, float* lse,
                                     int32_t out_dtype, float softmax_scale, float rope_theta,
                                     void* stream) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (!plan_dev || !q || !k || !v || !out) return PV_ERR_NULL;
  // refused before anything touches the GPU: the fixed array cannot hold this problem
  int64_t need = 0;
  st = pv_static_workspace_needed(sizes, &need);
  if (st != PV_OK) return st;
  if (need > (int64_t)PV_STATIC_WORKSPACE_BYTES) return PV_ERR_WORKSPACE;
  st = arch_ok_cached();
  if (st != PV_OK) return st;
  void* ws = nullptr;
  st = static_workspace(&ws);
  if (st != PV_OK) return st;
  return attention_call(sizes, plan_dev, q, k, v, out, lse, out_dtype, softmax_scale, rope_theta,
                        ws, PV_STATIC_WORKSPACE_BYTES, stream, false, true);
}

pv_status pv_static_workspace_needed(const pv_sizes* sizes, int64_t* bytes_out) {
  if (!bytes_out) return PV_ERR_NULL;
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  *bytes_out = attn_workspace_layout(sizes->total_tokens, sizes->padded_keys, sizes->n_seg_tiles,
                                     sizes->n_q_heads, sizes->n_kv_heads, sizes->head_dim,
                                     sizes->in_dtype).total_full;
  return PV_OK;
}

pv_status pv_segment_attention(const pv_sizes* sizes, const void* plan_dev, const void* q,
                               const void* k, const void* v, void* out, float* lse,
                               int32_t out_dtype, float softmax_scale, float rope_theta,
                               void* workspace, int64_t workspace_bytes, void* stream) {
  return attention_call(sizes, plan_dev, q, k, v, out, lse, out_dtype, softmax_scale, rope_theta,
                        workspace, workspace_bytes, stream, true);
}

pv_status pv_masked_attention_fp8kv(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                    const void* k_fp8, const void* v_fp8, const float* k_scale_dev,
                                    const float* v_scale_dev, void* out, float* lse, int32_t out_dtype,
                                    float softmax_scale, float rope_theta, void* workspace,
                                    int64_t workspace_bytes, void* stream) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (!plan_dev || !q || !k_fp8 || !v_fp8 || !k_scale_dev || !v_scale_dev || !out || !workspace)
    return PV_ERR_NULL;
  if (sizes->in_dtype != PV_BF16) return PV_ERR_DTYPE;          // Q is bf16
  if (out_dtype != PV_BF16 && out_dtype != PV_F32) return PV_ERR_DTYPE;
  if (sizes->head_dim != 128) return PV_ERR_SHAPE;
  if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return PV_ERR_SHAPE;
  if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return PV_ERR_SHAPE;
  const int hq = sizes->n_q_heads, hkv = sizes->n_kv_heads, d = sizes->head_dim;
  const AttnWorkspace wl = attn_workspace_layout(sizes->total_tokens, sizes->padded_keys,
                                                 sizes->n_seg_tiles, hq, hkv, d, PV_BF16);
  if (workspace_bytes < wl.total) return PV_ERR_WORKSPACE;
  if (misaligned(plan_dev) || misaligned(q) || misaligned(k_fp8) || misaligned(v_fp8) || misaligned(out) ||
      misaligned(workspace) || ((uintptr_t)lse & 3u) || ((uintptr_t)k_scale_dev & 3u) ||
      ((uintptr_t)v_scale_dev & 3u))
    return PV_ERR_ALIGN;
  st = arch_ok_cached();
  if (st != PV_OK) return st;
  const float scale = softmax_scale == 0.0f ? (float)(1.0 / std::sqrt((double)d)) : softmax_scale;
  RopeFreq freq;
  const bool rope = rope_theta > 0.0f;
  for (int c = 0; c < 64; ++c)
    freq.inv_freq[c] = rope ? std::pow((double)rope_theta, -2.0 * (double)c / (double)d) : 0.0;
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  std::unique_lock<std::mutex> guard(g_profile_lock);
  const bool profiling = g_profile;
  hipError_t e;
  if (profiling) {
    hipEvent_t* pair = g_ev[g_ev_calls % PV_PROFILE_RING];
    for (int i = 0; i < 2; ++i)
      if (!pair[i]) {
        e = hipEventCreate(&pair[i]);
        if (e != hipSuccess) { pair[i] = nullptr; return hip_fail(e); }
      }
    ev0 = pair[0];
    ev1 = pair[1];
  } else {
    guard.unlock();
  }
  e = launch_attn_fp8((const int32_t*)plan_dev, h, q, k_fp8, v_fp8, k_scale_dev, v_scale_dev, out, lse, hq,
                      hkv, d, out_dtype, scale, freq, rope, (char*)workspace, wl, ev0, ev1,
                      (hipStream_t)stream);
  if (e == hipSuccess && profiling) ++g_ev_calls;
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_prepare_kv(const pv_sizes* sizes, const void* plan_dev, const void* k, const void* v,
                        const int32_t* block_table_dev, int32_t page_size, int64_t first_token,
                        int64_t last_token, int64_t key_capacity, float rope_theta,
                        void* workspace, int64_t workspace_bytes, void* stream) {
  if (last_token < 0 || key_capacity < 0) return PV_ERR_SHAPE;
  return attention_call(sizes, plan_dev, nullptr, k, v, nullptr, nullptr, PV_BF16, 0.0f, rope_theta,
                        workspace, workspace_bytes, stream, true, false, kPhasePrepare,
                        block_table_dev, page_size, first_token, last_token, key_capacity);
}

pv_status pv_prepared_workspace_bytes(const pv_sizes* sizes, int64_t key_capacity, int64_t* bytes_out) {
  if (!bytes_out) return PV_ERR_NULL;
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  const bool own_stride = key_capacity != 0;
  if (key_capacity == 0) key_capacity = sizes->padded_keys;
  if (key_capacity < sizes->padded_keys || key_capacity % kTileN != 0 || key_capacity > (1ll << 27))
    return PV_ERR_SHAPE;
  *bytes_out = attn_workspace_layout(own_stride ? key_capacity : sizes->total_tokens, key_capacity,
                                     sizes->n_seg_tiles, sizes->n_q_heads, sizes->n_kv_heads,
                                     sizes->head_dim, sizes->in_dtype).total;
  return PV_OK;
}

pv_status pv_segment_attention_prepared(const pv_sizes* sizes, const void* plan_dev, const void* q,
                                        const void* k, const void* v,
                                        const int32_t* block_table_dev, int32_t page_size,
                                        int64_t key_capacity, void* out, float* lse,
                                        int32_t out_dtype, float softmax_scale, float rope_theta,
                                        void* workspace, int64_t workspace_bytes, void* stream) {
  if (key_capacity < 0) return PV_ERR_SHAPE;
  return attention_call(sizes, plan_dev, q, k, v, out, lse, out_dtype, softmax_scale, rope_theta,
                        workspace, workspace_bytes, stream, true, false, kPhaseAttend,
                        block_table_dev, page_size, 0, -1, key_capacity);
}

pv_status pv_first_reject(const pv_sizes* sizes, const void* plan_dev, const float* logits_dev,
                          double margin_threshold, int32_t mode, int32_t* out_dev, void* stream) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (!plan_dev || !out_dev) return PV_ERR_NULL;
  if (sizes->total_segments > 0 && !logits_dev) return PV_ERR_NULL;
  if (mode != 0 && mode != 1) return PV_ERR_SHAPE;
  if (std::isnan(margin_threshold)) return PV_ERR_SHAPE;
  if (misaligned(plan_dev) || ((uintptr_t)logits_dev & 7u) || ((uintptr_t)out_dev & 15u))
    return PV_ERR_ALIGN;
  st = arch_ok_cached();
  if (st != PV_OK) return st;
  hipError_t e = launch_first_reject((const int32_t*)plan_dev, h, logits_dev, margin_threshold,
                                     mode, out_dev, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_judge_logits(const pv_sizes* sizes, const void* plan_dev, const void* hidden_dev,
                          const void* w2_dev, int32_t hidden_size, float* logits_dev,
                          void* stream) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (!plan_dev) return PV_ERR_NULL;
  if (hidden_size < 8 || hidden_size > 65536 || hidden_size % 8 != 0) return PV_ERR_SHAPE;
  if (sizes->total_segments > 0 && (!hidden_dev || !w2_dev || !logits_dev)) return PV_ERR_NULL;
  if (misaligned(plan_dev) || misaligned(hidden_dev) || misaligned(w2_dev) ||
      ((uintptr_t)logits_dev & 7u))
    return PV_ERR_ALIGN;
  st = arch_ok_cached();
  if (st != PV_OK) return st;
  hipError_t e = launch_judge_logits((const int32_t*)plan_dev, h, hidden_dev, w2_dev, hidden_size,
                                     logits_dev, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_decide(const pv_sizes* sizes, const void* plan_dev, const float* logits_dev,
                    const float* full_logits_dev, const pv_policy* policy, int32_t* out_dev,
                    void* stream) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (!plan_dev || !out_dev || !policy) return PV_ERR_NULL;
  if (sizes->total_segments > 0 && !logits_dev) return PV_ERR_NULL;
  if (policy->premature != 0 && policy->premature != 1) return PV_ERR_SHAPE;
  if (!policy->premature && !full_logits_dev) return PV_ERR_NULL;
  if (policy->n_short < 0 || policy->n_short > PV_MAX_SHORT_CHUNKS || policy->kappa < 0 ||
      policy->relaxed_count_min < 0)
    return PV_ERR_SHAPE;
  if (!(policy->eta >= 0.0) || !std::isfinite(policy->eta) || !(policy->rho >= 0.0) ||
      std::isnan(policy->margin_chunk) || std::isnan(policy->margin_chunk_relaxed) ||
      std::isnan(policy->margin_full) || std::isnan(policy->margin_full_relaxed))
    return PV_ERR_SHAPE;
  for (int i = 0; i < policy->n_short; ++i)
    if (std::isnan(policy->margin_short[i])) return PV_ERR_SHAPE;
  if (misaligned(plan_dev) || ((uintptr_t)logits_dev & 7u) || ((uintptr_t)full_logits_dev & 7u) ||
      ((uintptr_t)out_dev & 15u))
    return PV_ERR_ALIGN;
  st = arch_ok_cached();
  if (st != PV_OK) return st;
  hipError_t e = launch_decide((const int32_t*)plan_dev, h, logits_dev, full_logits_dev, *policy,
                               out_dev, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_plan_export(const pv_sizes* sizes, const void* plan_dev, int32_t* positions_dev,
                         int32_t* a_end_dev, int32_t* b_start_dev, int32_t* judge_row_dev,
                         void* stream) {
  PlanHeader h;
  pv_status st = check_sizes(sizes, &h);
  if (st != PV_OK) return st;
  if (!plan_dev) return PV_ERR_NULL;
  st = arch_ok_cached();
  if (st != PV_OK) return st;
  hipError_t e = launch_plan_export((const int32_t*)plan_dev, h, positions_dev, a_end_dev,
                                    b_start_dev, judge_row_dev, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> guard(g_profile_lock);
  g_profile = on != 0;
  g_ev_calls = 0;
  hipError_t first = hipSuccess;
  if (!g_profile) {                                 // switched off: give the events back
    for (auto& pair : g_ev)
      for (hipEvent_t& ev : pair)
        if (ev) {
          const hipError_t e = hipEventDestroy(ev);
          if (e != hipSuccess && first == hipSuccess) first = e;
          ev = nullptr;
        }
  }
  return first == hipSuccess ? PV_OK : hip_fail(first);
}

static pv_status profile_pair_ms(int64_t call, float* ms) {
  hipEvent_t* pair = g_ev[call % PV_PROFILE_RING];
  hipError_t e = hipEventSynchronize(pair[1]);
  if (e != hipSuccess) return hip_fail(e);
  e = hipEventElapsedTime(ms, pair[0], pair[1]);
  if (e != hipSuccess) return hip_fail(e);
  return PV_OK;
}

pv_status pv_profile_read(float* main_kernel_ms) {
  if (!main_kernel_ms) return PV_ERR_NULL;
  std::lock_guard<std::mutex> guard(g_profile_lock);
  if (!g_profile || g_ev_calls == 0) return PV_ERR_SHAPE;
  return profile_pair_ms(g_ev_calls - 1, main_kernel_ms);
}

pv_status pv_profile_read_all(float* ms_host, int32_t capacity, int32_t* n_out) {
  if (!ms_host || !n_out) return PV_ERR_NULL;
  if (capacity < 0) return PV_ERR_SHAPE;
  *n_out = 0;
  std::lock_guard<std::mutex> guard(g_profile_lock);
  if (!g_profile) return PV_ERR_SHAPE;
  int64_t n = g_ev_calls < PV_PROFILE_RING ? g_ev_calls : PV_PROFILE_RING;
  if (n > capacity) n = capacity;
  for (int64_t i = 0; i < n; ++i) {
    pv_status st = profile_pair_ms(g_ev_calls - n + i, &ms_host[i]);
    if (st != PV_OK) return st;
  }
  *n_out = (int32_t)n;
  return PV_OK;
}

pv_status pv_margin_from_tau(double tau, double* margin_out) {
  if (!margin_out) return PV_ERR_NULL;
  if (!(tau > 0.0 && tau < 1.0)) return PV_ERR_SHAPE;
  *margin_out = std::log(tau / (1.0 - tau));
  return PV_OK;
}

const char* pv_strerror(pv_status status) {
  switch (status) {
    case PV_OK: return "ok";
    case PV_ERR_NULL: return "required pointer is NULL";
    case PV_ERR_SHAPE: return "unsupported or inconsistent shape";
    case PV_ERR_BOUNDARY: return "boundaries must be non-decreasing and within [0, draft_len]";
    case PV_ERR_WORKSPACE: return "buffer smaller than pv_query_sizes reported";
    case PV_ERR_ALIGN: return "device pointer not sufficiently aligned";
    case PV_ERR_DTYPE: return "unsupported dtype combination";
    case PV_ERR_ARCH: return "current device is not gfx950";
    case PV_ERR_HIP: return "HIP runtime error (see pv_last_hip_error)";
    default: return "unknown status";
  }
}

int32_t pv_last_hip_error(void) { return g_last_hip; }

const char* pv_version(void) { return "pv 0.1 (gfx950)"; }

}  // extern "C"
