// Internal declarations shared by the library's translation units (not part of the C ABI).
#ifndef PV_INTERNAL_H_
#define PV_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pv.h"

namespace pv {

// Query tokens per work item and keys per tile of the MFMA path.  The plan's tile ranges are
// expressed in these units.
constexpr int kTileM = 32;
constexpr int kTileN = 64;

constexpr int32_t kPlanMagic = 0x50565031;  // "PVP1"

// Header at the start of the plan blob.  All offsets are in int32 units from the blob start, so
// the blob can be copied anywhere.  The header, the per-request arrays and the boundaries are
// computed on the host and uploaded; everything after `off_device_begin` is written by kernels.
struct PlanHeader {
  int32_t magic, batch, total_tokens, total_segments;
  int32_t n_q_tiles, tile_m, tile_n, padded_keys;
  int32_t off_prompt, off_draft, off_nseg, off_seglen;   // [B] each
  int32_t off_tok_start, off_seg_start;                  // [B+1] each
  int32_t off_qtile_start, off_kpad_start;               // [B+1] each
  int32_t off_mask_start;                                // int64 [B+1] (8-byte aligned)
  int32_t off_bounds;                                    // [total_segments]
  int32_t off_short;                                     // [n_short_rows][4]: packed row, first row of its request, a_end, b_start
  int32_t off_device_begin;
  int32_t off_pos, off_aend, off_bstart;                 // [total_tokens] each
  int32_t off_judge;                                     // [total_segments]
  int32_t off_tiles, off_work;                           // [n_q_tiles][8] each
  int32_t total_ints;
  int32_t n_short_rows;
  int32_t layout;                                        // PV_LAYOUT_*
  int32_t off_map;                                       // [total_tokens], interleaved layout only
  int32_t n_seg_tiles;                                   // query tiles with at least one segment row
  int32_t off_segtile_start;                             // [B+1] first such tile of a request, counted over the batch
  int32_t off_segwork;                                   // [n_seg_tiles][8] those tiles, request after request
  int32_t n_quads;                                       // groups of four consecutive query tiles of a request
  int32_t off_quad_start;                                // [B+1] first such group of a request
  int32_t off_quadwork;                                  // [n_quads][8], per request last group first
};
static_assert(sizeof(PlanHeader) == 36 * 4, "PlanHeader must be 36 ints");

// One-dimensional grid of `blocks` workgroups of `threads` threads.  A launch may not span 2^32
// threads or more: a grid that large is reported as an error and never truncated.
inline bool grid_1d(int64_t blocks, int threads, dim3* grid) {
  if (blocks < 1 || blocks * threads > 0xffffffffll) return false;
  *grid = dim3((unsigned)blocks);
  return true;
}

// The kernels work on "virtual" rows in the appended order [prompt | draft | segments] of every
// request.  For the interleaved layout the same tokens sit elsewhere in the caller's tensors; the
// plan then holds, per virtual row, the caller's row.  Everything the plan stores per token (position,
// row descriptor) and the K/V workspaces are indexed by virtual row.
__device__ inline int64_t caller_row(const int32_t* plan, const PlanHeader& h, int64_t g) {
  return h.layout == PV_LAYOUT_INTERLEAVED ? (int64_t)plan[h.off_map + g] : g;
}

// Group sizes 4 and 8 fill the wave slots of a compute unit with one workgroup per (tile, kv head):
// 2 x 4 or 1 x 8 waves, every K/V slot staged once for the whole group.  The other sizes leave
// slots empty (5 waves: one workgroup of 5 in 8 slots; 1 or 2 waves: two workgroups of 1 or 2), so
// the whole pass runs them as workgroups of four query tiles per head instead.  Measured on one
// shape (6 656 tokens, 8 kv heads): faster for G = 1, 2, 3, 5, 6 (1.65x .. 1.06x); with 7 of 8 slots
// used, staging K/V once per group wins again.  The plan lists the groups of four tiles only for
// these sizes (n_quads = 0 otherwise).
inline bool group_uses_query_tiles(int G) { return G != 4 && G < 7; }

// One query tile of the work list (8 ints).
struct QTile {
  int32_t tok_base;    // first packed row of the request
  int32_t t0;          // first local token of the tile
  int32_t rows;        // valid tokens in the tile (1..tile_m)
  int32_t n_full;      // key tiles [0, n_full) are visible to every row: no mask code
  int32_t n_a;         // key tiles [n_full, n_a) need the row predicate
  int32_t jb0, jb1;    // second range of key tiles [jb0, jb1), all with the row predicate
  int32_t kpad_base;   // first padded key row of the request in the rotated-K / V^T workspace
};

struct RopeFreq { double inv_freq[64]; };   // theta^(-2c/D), c < D/2 <= 64

// Workspace of the attention call (byte offsets), derived from pv_sizes.
struct AttnWorkspace {
  int64_t off_cs;      // float2 [total_tokens][D/2] (cos, sin)
  int64_t off_krot;    // bf16 path: [Hkv][padded_keys][D] bf16; fp32 path: [total_tokens][Hkv][D] float
  int64_t off_vt;      // bf16 path: V^T slabs, [Hkv][padded_keys/16][2][D][8] bf16
  int64_t off_part;    // bf16 path, segment-only call: partial results of the key pieces, per
                       // (segment tile, kv head, piece, head of the group): float [32][D] then float2 [32]
  int split;           // pieces per work item of the segment-only call (1: no partial results)
  int64_t total_full;  // bytes the whole-pass call uses (everything before the partial results)
  int64_t total;
};
AttnWorkspace attn_workspace_layout(int64_t total_tokens, int64_t padded_keys, int64_t n_seg_tiles,
                                    int hq, int hkv, int d, int in_dtype);

// --- launchers (each returns the hipError_t of its launches) ---
// Uploads the host image (n_img ints at the start of the plan) and builds the device part.
hipError_t launch_plan_kernels(int32_t* plan_dev, const PlanHeader& h, const int32_t* host_ints,
                               int n_img, uint8_t* dense_mask, hipStream_t s);
hipError_t launch_plan_export(const int32_t* plan_dev, const PlanHeader& h, int32_t* pos,
                              int32_t* aend, int32_t* bstart, int32_t* judge, hipStream_t s);
hipError_t launch_first_reject(const int32_t* plan_dev, const PlanHeader& h, const float* logits,
                               double thr, int mode, int32_t* out, hipStream_t s);
hipError_t launch_decide(const int32_t* plan_dev, const PlanHeader& h, const float* logits,
                         const float* full_logits, const pv_policy& pol, int32_t* out, hipStream_t s);
hipError_t launch_judge_logits(const int32_t* plan_dev, const PlanHeader& h, const void* hidden,
                               const void* w2, int hidden_size, float* logits, hipStream_t s);
hipError_t launch_attn_f32(const int32_t* plan_dev, const PlanHeader& h, const float* q,
                           const float* k, const float* v, float* out, float* lse, int hq,
                           int hkv, int d, float scale, const RopeFreq& freq, bool rope,
                           char* ws, const AttnWorkspace& wl, hipStream_t s);
// The caller's K and V for the preparation: dense tensors, or a pool of pages with a block table.
struct KvArgs {
  const void* k;
  const void* v;
  const int32_t* block_table;   // device, or nullptr for dense tensors
  int page_size;
};
// bf16 path, step 1: rotary table, rotated K and transposed V of the tokens [tok_first, tok_last) into
// the workspace (key_blocks), and the fp32 evaluation of the rows with few keys (q != nullptr).
hipError_t launch_prep_bf16(const int32_t* plan_dev, const PlanHeader& h, const KvArgs& kv, int hkv, int d,
                            const RopeFreq& freq, bool rope, char* ws, const AttnWorkspace& wl,
                            bool key_blocks, int64_t tok_first, int64_t tok_last, const void* q, void* out,
                            float* lse, int hq, float scale, bool out_f32, bool segments_only,
                            hipStream_t s);
// bf16 path, step 2: the main kernel over the prepared keys (whole pass, or segment rows only).
// short_rows_kv != nullptr: the launch also evaluates the rows with few keys (fp32) from these tensors,
// which main_kernel_takes_short_rows says it can; otherwise the preparation launch has done them.
bool main_kernel_takes_short_rows(const PlanHeader& h, int hq, int hkv, bool segments_only);
hipError_t launch_main_bf16(const int32_t* plan_dev, const PlanHeader& h, const void* q, void* out,
                            float* lse, int hq, int hkv, int d, int out_dtype, float scale, bool rope,
                            char* ws, const AttnWorkspace& wl, bool segments_only,
                            const KvArgs* short_rows_kv, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s);

// FP8 K/V path (head_dim 128): preparation, short rows and the main kernel on the FP8 matrix instruction.
hipError_t launch_attn_fp8(const int32_t* plan_dev, const PlanHeader& h, const void* q, const void* k8,
                           const void* v8, const float* k_scale, const float* v_scale, void* out, float* lse,
                           int hq, int hkv, int d, int out_dtype, float scale, const RopeFreq& freq, bool rope,
                           char* ws, const AttnWorkspace& wl, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s);

// Host-side layout of the plan; shared by pv_query_sizes and pv_build_mask.
void plan_layout(int batch, int64_t total_tokens, int64_t total_segments, int64_t n_q_tiles,
                 int64_t padded_keys, int64_t n_short_rows, int layout, int64_t n_seg_tiles,
                 int64_t n_quads, PlanHeader* h);

}  // namespace pv
#endif
