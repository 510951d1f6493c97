// Integer kernels: plan construction (row descriptors, positions, judge rows, tile work list),
// the optional dense mask, plan export and the readout.
#include "pv_internal.h"

namespace pv {

// ---------------------------------------------------------------- upload of the host image
constexpr int kUploadInts = 896;   // 3584 bytes of kernel arguments per launch
struct UploadChunk { int32_t v[kUploadInts]; };

__global__ __launch_bounds__(256) void k_upload(int32_t* dst, UploadChunk c, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = c.v[i];
}

static hipError_t launch_upload(int32_t* plan_dev, const int32_t* host_ints, int n, hipStream_t s) {
  // The image travels in kernel arguments: they are captured at launch, so the host buffer can
  // be released immediately and no pageable-memory copy semantics are involved.
  for (int o = 0; o < n; o += kUploadInts) {
    UploadChunk c;
    const int m = (n - o) < kUploadInts ? (n - o) : kUploadInts;
    for (int i = 0; i < m; ++i) c.v[i] = host_ints[o + i];
    for (int i = m; i < kUploadInts; ++i) c.v[i] = 0;
    k_upload<<<dim3((m + 255) / 256), dim3(256), 0, s>>>(plan_dev + o, c, m);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------------------- row descriptors
struct Req {
  int P, T, K, S, N;
  const int32_t* bounds;
};

__device__ inline Req load_req(const int32_t* plan, const PlanHeader& h, int b) {
  Req r;
  r.P = plan[h.off_prompt + b];
  r.T = plan[h.off_draft + b];
  r.K = plan[h.off_nseg + b];
  r.S = plan[h.off_seglen + b];
  r.N = r.P + r.T + r.K * r.S;
  r.bounds = plan + h.off_bounds + plan[h.off_seg_start + b];
  return r;
}

// Visible keys of local row i are [0, a_end) and [b_start, i].  Prompt and draft rows are plain
// causal (a_end = b_start = 0).  A row of segment k sees the prompt and the first p_k draft
// tokens (a_end = P + p_k) and its own segment up to itself (b_start = first row of the
// segment); its rotary position continues from the end of that prefix.
__device__ inline void row_desc(const Req& r, int i, int* pos, int* a_end, int* b_start) {
  const int c = r.P + r.T;
  if (i < c) {
    *pos = i; *a_end = 0; *b_start = 0;
  } else {
    const int k = (i - c) / r.S;
    const int a = (i - c) - k * r.S;
    *a_end = r.P + r.bounds[k];
    *b_start = c + k * r.S;
    *pos = *a_end + a;
  }
}

// Interleaved packing ("Parallel partial verify"): where local token i of the appended order
// [prompt | draft | segments] sits when every segment follows the draft tokens it judges.  A draft
// token is pushed back by the segments whose boundary does not exceed it; segment k comes after
// its p_k draft tokens and the k segments before it.
__device__ inline int interleaved_row(const Req& r, int i) {
  const int c = r.P + r.T;
  if (i < r.P) return i;
  if (i < c) {
    const int t = i - r.P;
    int lo = 0, hi = r.K;          // number of boundaries <= t
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (r.bounds[mid] <= t) lo = mid + 1; else hi = mid;
    }
    return i + lo * r.S;
  }
  const int k = (i - c) / r.S;
  const int a = (i - c) - k * r.S;
  return r.P + r.bounds[k] + k * r.S + a;
}

// Largest b with start[b] <= x, for a non-decreasing start[0..n] with start[0] = 0 <= x < start[n].
__device__ inline int find_owner(const int32_t* start, int n, int x) {
  int lo = 0, hi = n;            // invariant: start[lo] <= x < start[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (start[mid] <= x) lo = mid; else hi = mid;
  }
  // skip empty owners (start[lo] == start[lo+1]) cannot happen for lo returned here because
  // start[lo] <= x < start[lo+1] after the loop.
  return lo;
}

// Row g of the packed batch (and, for g < total_segments, judge row g).  `img` is where the
// uploaded part of the plan is read from (the plan itself, or a copy in LDS).
__device__ inline void plan_token(int32_t* plan, const int32_t* img, const PlanHeader& h, int g) {
  if (g < h.total_tokens) {
    const int b = find_owner(img + h.off_tok_start, h.batch, g);
    const Req r = load_req(img, h, b);
    int pos, ae, bs;
    row_desc(r, g - img[h.off_tok_start + b], &pos, &ae, &bs);
    plan[h.off_pos + g] = pos;
    plan[h.off_aend + g] = ae;
    plan[h.off_bstart + g] = bs;
    if (h.layout == PV_LAYOUT_INTERLEAVED)
      plan[h.off_map + g] = img[h.off_tok_start + b] + interleaved_row(r, g - img[h.off_tok_start + b]);
  }
  if (g < h.total_segments) {
    const int b = find_owner(img + h.off_seg_start, h.batch, g);
    const Req r = load_req(img, h, b);
    const int k = g - img[h.off_seg_start + b];
    // the verdict of segment k is read at its last token (a row of the caller's tensors)
    const int last = r.P + r.T + (k + 1) * r.S - 1;
    plan[h.off_judge + g] = img[h.off_tok_start + b] +
                            (h.layout == PV_LAYOUT_INTERLEAVED ? interleaved_row(r, last) : last);
  }
}

__global__ __launch_bounds__(256) void k_plan_tokens(int32_t* plan, PlanHeader h) {
  plan_token(plan, plan, h, blockIdx.x * blockDim.x + threadIdx.x);
}

// Query tile t: the union of its rows' visible key sets, in key-tile units.  *seg_slot is the
// tile's place in the list of tiles that hold segment rows (request after request), -1 if it
// holds none.
__device__ inline QTile plan_tile(const int32_t* plan, const PlanHeader& h, int t, int* seg_slot) {
  const int b = find_owner(plan + h.off_qtile_start, h.batch, t);
  const Req r = load_req(plan, h, b);
  const int t0 = (t - plan[h.off_qtile_start + b]) * h.tile_m;
  const int rows = min(h.tile_m, r.N - t0);
  const int bn = h.tile_n;
  int min_prefix = 0x7fffffff;   // min over rows of the length of the fully visible key prefix
  int max_low = 0;               // max over rows of the end of the low range
  int min_b = 0x7fffffff, max_i = -1;
  // The rows of a tile are consecutive, causal rows first.  Their low range ends at i + 1, which
  // grows with i; a segment row's ends at P + p_k and its second range starts at the segment's
  // first row, both non-decreasing in k because the boundaries are sorted.  The extremes over the
  // tile therefore sit at the first and last row of each kind.
  const int c = r.P + r.T, last = t0 + rows - 1;
  *seg_slot = last >= c ? plan[h.off_segtile_start + b] + (t0 - c / h.tile_m * h.tile_m) / h.tile_m : -1;
  if (t0 < c) {
    min_prefix = t0 + 1;
    max_low = min(last, c - 1) + 1;
  }
  if (last >= c) {
    int pos, ae0, bs0, ae1, bs1;
    row_desc(r, max(t0, c), &pos, &ae0, &bs0);
    row_desc(r, last, &pos, &ae1, &bs1);
    min_prefix = min(min_prefix, ae0);
    max_low = max(max_low, ae1);
    min_b = bs0;
    max_i = last;
  }
  QTile q;
  q.tok_base = plan[h.off_tok_start + b];
  q.t0 = t0;
  q.rows = rows;
  q.n_full = min_prefix / bn;
  q.n_a = (max_low + bn - 1) / bn;
  if (max_i >= 0) {
    q.jb0 = max(q.n_a, min_b / bn);
    q.jb1 = max(q.jb0, max_i / bn + 1);
  } else {
    q.jb0 = q.n_a; q.jb1 = q.n_a;
  }
  q.kpad_base = plan[h.off_kpad_start + b];
  return q;
}

// Group qd of four consecutive query tiles of a request (the last group of a request may hold
// fewer): the union of their key-tile lists, for the launch whose workgroups take four query tiles
// of one head.  Every wave of such a workgroup masks with its own tile's descriptor, so key tiles
// that only some of the four need are simply fully masked for the others.  `n_full` of the result
// carries the index of the group's first tile in the tile list instead.  *slot: the groups of a
// request are listed last first (the last group has the longest key list).
__device__ inline QTile plan_quad(const int32_t* plan, const PlanHeader& h, int qd, int* slot) {
  const int b = find_owner(plan + h.off_quad_start, h.batch, qd);
  const int q0 = plan[h.off_quad_start + b], nq = plan[h.off_quad_start + b + 1] - q0;
  const int ql = qd - q0;
  const int t_first = plan[h.off_qtile_start + b] + 4 * ql;
  const int t_end = min(t_first + 4, plan[h.off_qtile_start + b + 1]);
  int unused;
  QTile u = plan_tile(plan, h, t_first, &unused);
  for (int t = t_first + 1; t < t_end; ++t) {
    const QTile q = plan_tile(plan, h, t, &unused);
    u.rows += q.rows;
    u.n_a = max(u.n_a, q.n_a);
    if (q.jb1 > q.jb0) {
      if (u.jb1 > u.jb0) { u.jb0 = min(u.jb0, q.jb0); u.jb1 = max(u.jb1, q.jb1); }
      else { u.jb0 = q.jb0; u.jb1 = q.jb1; }
    }
  }
  if (u.jb1 > u.jb0) { u.jb0 = max(u.jb0, u.n_a); u.jb1 = max(u.jb1, u.jb0); }
  else { u.jb0 = u.n_a; u.jb1 = u.n_a; }
  u.n_full = t_first;
  *slot = q0 + (nq - 1 - ql);
  return u;
}

__global__ __launch_bounds__(256) void k_plan_tiles(int32_t* plan, PlanHeader h) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < h.n_q_tiles) {
    int seg_slot;
    const QTile q = plan_tile(plan, h, t, &seg_slot);
    reinterpret_cast<QTile*>(plan + h.off_tiles)[t] = q;
    if (seg_slot >= 0) reinterpret_cast<QTile*>(plan + h.off_segwork)[seg_slot] = q;
  }
  if (t < h.n_quads) {
    int slot;
    const QTile u = plan_quad(plan, h, t, &slot);
    reinterpret_cast<QTile*>(plan + h.off_quadwork)[slot] = u;
  }
}

// Small problems: the whole plan in one launch.  The host image arrives in the kernel arguments, so
// every workgroup has it without waiting for another: workgroup 0 writes it to the plan and builds the
// tile lists (phases separated by workgroup barriers), the other workgroups share the per-token
// arrays among them.  Nothing written by one workgroup is read by another inside the launch.
constexpr int kSmallTokens = 8192, kSmallTiles = 1024;
__global__ __launch_bounds__(1024) void k_plan_small(int32_t* plan, PlanHeader h, UploadChunk c,
                                                     int n_img) {
  __shared__ int cost_s[kSmallTiles];
  __shared__ int32_t img_s[kUploadInts];       // the request data is read from here, not from HBM
  const int tid = threadIdx.x;
  const bool first = blockIdx.x == 0;
  for (int i = tid; i < n_img; i += 1024) {
    const int32_t x = c.v[i];
    if (first) plan[i] = x;
    img_s[i] = x;
  }
  __syncthreads();
  const int n1 = h.total_tokens > h.total_segments ? h.total_tokens : h.total_segments;
  if (gridDim.x == 1 || !first) {              // tokens: all workgroups but the first, if there are others
    const int nb = gridDim.x == 1 ? 1 : (int)gridDim.x - 1, me = gridDim.x == 1 ? 0 : (int)blockIdx.x - 1;
    for (int g = me * 1024 + tid; g < n1; g += nb * 1024) plan_token(plan, img_s, h, g);
  }
  if (!first) return;
  QTile mine;
  int my_cost = 0;
  if (tid < h.n_q_tiles) {
    int seg_slot;
    mine = plan_tile(img_s, h, tid, &seg_slot);
    my_cost = mine.n_a + (mine.jb1 - mine.jb0);
    reinterpret_cast<QTile*>(plan + h.off_tiles)[tid] = mine;
    if (seg_slot >= 0) reinterpret_cast<QTile*>(plan + h.off_segwork)[seg_slot] = mine;

    cost_s[tid] = my_cost;
  }
  // the groups of four tiles go to the threads after those of the tiles; if the workgroup is too
  // small for both, the first threads take them as well
  const bool beside = h.n_q_tiles + h.n_quads <= 1024;
  for (int qd = beside ? tid - h.n_q_tiles : tid; qd >= 0 && qd < h.n_quads; qd += 1024) {
    int slot;
    const QTile u = plan_quad(img_s, h, qd, &slot);
    reinterpret_cast<QTile*>(plan + h.off_quadwork)[slot] = u;
  }
  __syncthreads();
  if (tid < h.n_q_tiles) {          // longest first, stable
    int rank = 0;
    for (int x = 0; x < h.n_q_tiles; ++x) {
      const int cx = cost_s[x];
      rank += (cx > my_cost) || (cx == my_cost && x < tid);
    }
    reinterpret_cast<QTile*>(plan + h.off_work)[rank] = mine;
  }
}

// Longest-first order (stable): rank = number of tiles that must run before this one.  One wave
// per tile; its lanes share the comparisons against all other tiles.
__global__ __launch_bounds__(256) void k_plan_sort(int32_t* plan, PlanHeader h) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= h.n_q_tiles) return;                 // whole waves leave together
  const QTile* tiles = reinterpret_cast<const QTile*>(plan + h.off_tiles);
  const QTile mine = tiles[t];
  const int my_cost = mine.n_a + (mine.jb1 - mine.jb0);
  int rank = 0;
  for (int u = lane; u < h.n_q_tiles; u += 64) {
    const int c = tiles[u].n_a + (tiles[u].jb1 - tiles[u].jb0);
    rank += (c > my_cost) || (c == my_cost && u < t);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) rank += __shfl_xor(rank, off);
  if (lane == 0) reinterpret_cast<QTile*>(plan + h.off_work)[rank] = mine;
}

// Dense mask from the stored row descriptors (what the attention kernels consume).
__global__ __launch_bounds__(256) void k_dense_mask(const int32_t* plan, PlanHeader h, uint8_t* mask) {
  const int g = blockIdx.x;      // packed row
  const int b = find_owner(plan + h.off_tok_start, h.batch, g);
  const int base = plan[h.off_tok_start + b];
  const int n = plan[h.off_tok_start + b + 1] - base;
  const int i = g - base;
  const int ae = plan[h.off_aend + g], bs = plan[h.off_bstart + g];
  const int64_t* mask_start = reinterpret_cast<const int64_t*>(plan + h.off_mask_start);
  // rows and columns of the mask follow the caller's row order
  uint8_t* row = mask + mask_start[b] + (caller_row(plan, h, g) - base) * n;
  for (int j = threadIdx.x; j < n; j += blockDim.x)
    row[caller_row(plan, h, base + j) - base] = (j < ae) || (j >= bs && j <= i) ? 1 : 0;
}

hipError_t launch_plan_kernels(int32_t* plan_dev, const PlanHeader& h, const int32_t* host_ints,
                               int n_img, uint8_t* dense_mask, hipStream_t s) {
  hipError_t e;
  const int n1 = h.total_tokens > h.total_segments ? h.total_tokens : h.total_segments;
  if (n_img <= kUploadInts && n1 <= kSmallTokens && h.n_q_tiles <= kSmallTiles) {
    UploadChunk c;
    for (int i = 0; i < n_img; ++i) c.v[i] = host_ints[i];
    for (int i = n_img; i < kUploadInts; ++i) c.v[i] = 0;
    const int token_groups = (n1 + 1023) / 1024;                 // at most three extra workgroups
    k_plan_small<<<dim3(1 + (token_groups < 3 ? token_groups : 3)), dim3(1024), 0, s>>>(plan_dev, h, c, n_img);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  } else {
    e = launch_upload(plan_dev, host_ints, n_img, s);
    if (e != hipSuccess) return e;
    k_plan_tokens<<<dim3((n1 + 255) / 256), dim3(256), 0, s>>>(plan_dev, h);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int nt = (h.n_q_tiles + 255) / 256;
    k_plan_tiles<<<dim3(nt), dim3(256), 0, s>>>(plan_dev, h);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_plan_sort<<<dim3((h.n_q_tiles + 3) / 4), dim3(256), 0, s>>>(plan_dev, h);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (dense_mask) {
    dim3 grid;
    if (!grid_1d(h.total_tokens, 256, &grid)) return hipErrorInvalidConfiguration;
    k_dense_mask<<<grid, dim3(256), 0, s>>>(plan_dev, h, dense_mask);
    e = hipGetLastError();
  }
  return e;
}

// ---------------------------------------------------------------- export
__global__ __launch_bounds__(256) void k_export(const int32_t* plan, PlanHeader h, int32_t* pos,
                                                int32_t* aend, int32_t* bstart, int32_t* judge) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g < h.total_tokens) {
    const int64_t row = caller_row(plan, h, g);
    if (pos) pos[row] = plan[h.off_pos + g];
    if (aend) aend[row] = plan[h.off_aend + g];
    if (bstart) bstart[row] = plan[h.off_bstart + g];
  }
  if (judge && g < h.total_segments) judge[g] = plan[h.off_judge + g];
}

hipError_t launch_plan_export(const int32_t* plan_dev, const PlanHeader& h, int32_t* pos,
                              int32_t* aend, int32_t* bstart, int32_t* judge, hipStream_t s) {
  const int n1 = h.total_tokens > h.total_segments ? h.total_tokens : h.total_segments;
  k_export<<<dim3((n1 + 255) / 256), dim3(256), 0, s>>>(plan_dev, h, pos, aend, bstart, judge);
  return hipGetLastError();
}

// ---------------------------------------------------------------- readout
// One wave per request: lane l takes segments l, l + 64, ..., so the logits of a request arrive
// in one round of loads; the three per-request quantities are then a min, a max and a sum over
// the wave.  A verdict is Correct iff the fp64 margin l_C - l_I is non-negative (ties count as
// Correct) and reaches the threshold.
__global__ __launch_bounds__(256) void k_first_reject(const int32_t* plan, PlanHeader h,
                                                      const float* logits, double thr, int mode,
                                                      int32_t* out) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= h.batch) return;                     // whole waves leave together
  const int s0 = plan[h.off_seg_start + b];
  const int K = plan[h.off_nseg + b];
  const int32_t* bounds = plan + h.off_bounds + s0;
  int first = K, last_ok = -1, bad = 0;
  for (int k = lane; k < K; k += 64) {
    const float2 lg = reinterpret_cast<const float2*>(logits)[s0 + k];
    const double d = (double)lg.x - (double)lg.y;
    const bool ok = (d >= 0.0) && (d >= thr);
    if (ok) last_ok = k;                        // k grows: the last one written is the largest
    else { bad++; first = min(first, k); }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    first = min(first, __shfl_xor(first, off));
    last_ok = max(last_ok, __shfl_xor(last_ok, off));
    bad += __shfl_xor(bad, off);
  }
  if (lane == 0) {
    const int k_star = (mode == 0) ? first - 1 : last_ok;
    int4 o;
    o.x = first;
    o.y = k_star;
    o.z = k_star >= 0 ? bounds[k_star] : 0;
    o.w = bad;
    reinterpret_cast<int4*>(out)[b] = o;
  }
}

hipError_t launch_first_reject(const int32_t* plan_dev, const PlanHeader& h, const float* logits,
                               double thr, int mode, int32_t* out, hipStream_t s) {
  k_first_reject<<<dim3((h.batch + 3) / 4), dim3(256), 0, s>>>(plan_dev, h, logits, thr, mode, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------- decision policy
// One thread per request; every comparison in fp64 on the margin l_C - l_I.
__global__ __launch_bounds__(64) void k_decide(const int32_t* plan, PlanHeader h, const float* logits,
                                               const float* full_logits, pv_policy pol,
                                               int32_t* out) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= h.batch) return;
  const int s0 = plan[h.off_seg_start + b];
  const int K = plan[h.off_nseg + b];
  const int32_t* bounds = plan + h.off_bounds + s0;
  int first = K, bad = 0, trailing = 0, below = 0, argmin = -1;
  double dmin = 0.0;
  for (int k = 0; k < K; ++k) {
    const double d = (double)logits[2 * (s0 + k)] - (double)logits[2 * (s0 + k) + 1];
    const bool ok = (d >= 0.0) && (d >= pol.margin_chunk);
    if (ok) trailing = 0;
    else { bad++; trailing++; if (first == K) first = k; }
    if (d < pol.margin_chunk_relaxed) below++;
    if (argmin < 0 || d < dmin) { argmin = k; dmin = d; }
  }
  const int k_star = first - 1;
  const bool rejects = (K > 0 && (double)bad > pol.rho * (double)K) ||
                       (pol.kappa > 0 && trailing >= pol.kappa);
  const int m = (int)floor(fmax(0.0, (double)k_star + 1.0 - pol.eta));
  const int l_star = m >= 1 ? bounds[m - 1] : 0;
  const int handoff = l_star > 0 ? PV_LABEL_SM_LG : PV_LABEL_LG;
  int label, stage, v_full = -1;
  if (pol.premature) {
    const bool abort = rejects || below >= pol.relaxed_count_min;
    label = abort ? handoff : -1;
    stage = abort ? 1 : 0;
  } else {
    const double df = (double)full_logits[2 * b] - (double)full_logits[2 * b + 1];
    v_full = (df >= 0.0) && (df >= pol.margin_full);
    if (v_full) { label = PV_LABEL_SM; stage = 2; }
    else if (K >= 1 && K <= pol.n_short && df >= pol.margin_short[K - 1]) { label = PV_LABEL_SM; stage = 3; }
    else if (df >= pol.margin_full_relaxed && below == 0) { label = PV_LABEL_SM; stage = 5; }
    else { label = handoff; stage = 6; }
  }
  int32_t* o = out + 12 * b;
  o[0] = label; o[1] = stage; o[2] = l_star; o[3] = k_star; o[4] = first; o[5] = bad;
  o[6] = trailing; o[7] = rejects ? 1 : 0; o[8] = below; o[9] = v_full; o[10] = argmin; o[11] = K;
}

hipError_t launch_decide(const int32_t* plan_dev, const PlanHeader& h, const float* logits,
                         const float* full_logits, const pv_policy& pol, int32_t* out, hipStream_t s) {
  k_decide<<<dim3((h.batch + 63) / 64), dim3(64), 0, s>>>(plan_dev, h, logits, full_logits, pol, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------- judge logits
// One wave per segment: lanes stride over the hidden dimension in 16-byte pieces, two fp32 dot
// products, then a fixed-order butterfly reduction (bit-reproducible).
__global__ __launch_bounds__(256) void k_judge_logits(const int32_t* plan, PlanHeader h,
                                                      const uint16_t* hidden, const uint16_t* w2,
                                                      int hs, float* logits) {
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (seg >= h.total_segments) return;
  const int64_t row = plan[h.off_judge + seg];
  const uint4* hp = reinterpret_cast<const uint4*>(hidden + row * hs);
  const uint4* w0 = reinterpret_cast<const uint4*>(w2);
  const uint4* w1 = reinterpret_cast<const uint4*>(w2 + hs);
  float a0 = 0.0f, a1 = 0.0f;
  for (int c = lane; c < hs / 8; c += 64) {
    const uint4 x = hp[c], u = w0[c], v = w1[c];
    const unsigned xs[4] = {x.x, x.y, x.z, x.w}, us[4] = {u.x, u.y, u.z, u.w}, vs[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xl = __uint_as_float(xs[e] << 16), xh = __uint_as_float(xs[e] & 0xffff0000u);
      a0 = fmaf(xl, __uint_as_float(us[e] << 16), a0);
      a0 = fmaf(xh, __uint_as_float(us[e] & 0xffff0000u), a0);
      a1 = fmaf(xl, __uint_as_float(vs[e] << 16), a1);
      a1 = fmaf(xh, __uint_as_float(vs[e] & 0xffff0000u), a1);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { a0 += __shfl_xor(a0, off); a1 += __shfl_xor(a1, off); }
  if (lane == 0) { logits[2 * seg] = a0; logits[2 * seg + 1] = a1; }
}

hipError_t launch_judge_logits(const int32_t* plan_dev, const PlanHeader& h, const void* hidden,
                               const void* w2, int hidden_size, float* logits, hipStream_t s) {
  if (h.total_segments == 0) return hipSuccess;
  dim3 grid;
  if (!grid_1d(((int64_t)h.total_segments + 3) / 4, 256, &grid)) return hipErrorInvalidConfiguration;
  k_judge_logits<<<grid, dim3(256), 0, s>>>(
      plan_dev, h, (const uint16_t*)hidden, (const uint16_t*)w2, hidden_size, logits);
  return hipGetLastError();
}

}  // namespace pv
