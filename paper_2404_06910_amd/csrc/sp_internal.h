// Internal declarations shared by the translation units of libsp.so (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "sp.h"

namespace sp {

constexpr int kMaxRanges = 1024;   // ancestor key ranges per row group (after merging neighbours); a sanity bound, no array depends on it
constexpr int kPrefillThreads = 256;
constexpr int kMaxDevices = 64;
// per-path accumulator of the saliency launch: fixed-point sum of log-likelihoods, scored rows, flags
struct SalSlot {
  unsigned long long sum;   // two's complement, 2^-36 units
  uint32_t count;
  uint32_t flags;           // 1: a row with lp = -inf, 2: +inf, 4: NaN
};
// per-row result of the saliency row kernel: the log-likelihood in fixed point, or flag bits when it is
// not finite; scored = 0 for rows without a target
struct RowLp {
  long long q;
  uint32_t flags;
  uint32_t scored;
};
constexpr int64_t kSalDefaultRows = int64_t(1) << 16;               // what a new context's workspace is sized for
constexpr int kSalDefaultSlots = 16384;
constexpr int64_t kSalStaticRows = int64_t(1) << 16;                // limits of the no-allocation entry point
constexpr int kSalStaticSlots = 16384;
inline size_t saliency_scratch_bytes(int64_t rows, int32_t slots) {
  return 256 + sizeof(SalSlot) * size_t(slots) + sizeof(RowLp) * size_t(rows);
}
constexpr size_t kSalStaticBytes = 256 + size_t(kSalStaticRows) * sizeof(RowLp) + sizeof(SalSlot) * size_t(kSalStaticSlots);

// A run of segments fused on the query side: child segments that are packed directly behind
// their parent continue the parent's causal sequence (Sec. 3.2: a chain is a classical prompt).
// Rows [tok_start, tok_start+len) see: the ancestor ranges (all keys), then own rows causally.
struct RowGroup {
  int32_t tok_start;
  int32_t len;
  int32_t range_off;   // first ancestor range (root-to-leaf order)
  int32_t n_ranges;
  int32_t anc_keys;    // total keys in the ancestor ranges
  int32_t prompt;
};

struct KeyRange {
  int32_t tok_start;
  int32_t len;
};

struct RangeDesc {
  int32_t beg, end;    // decode ranges [beg, end) of dec_ranges
  int32_t tok_start;   // copy of dec_ranges[beg] (0, 0 when beg == end)
  int32_t len;
};

// One prefill work item: a tile of query rows of one row group, for one group of query heads.
// Self-contained (one 32-byte scalar load), so a workgroup never chases pointers between items.
struct WorkItem {
  int32_t tok_start;   // first packed token of the row group
  int32_t row0;        // first row of the tile inside the group
  int32_t n_rows;      // token rows in the tile (1 .. tile_rows)
  int32_t anc_keys;    // keys in the ancestor ranges
  int32_t range_off;   // first ancestor range
  int32_t n_ranges;
  int32_t head0;       // first query head handled by the workgroup | its KV head << 16
  int32_t r0_start;    // first token of ancestor range 0 (the only one when n_ranges == 1)
};

// Device-side view of a plan (plain pointers, passed by value to kernels).
struct PlanDev {
  const RowGroup *groups;
  const KeyRange *ranges;
  const WorkItem *items;
  const int32_t *wg_begin;       // [n_wg + 1] slice of the (permuted) work list per workgroup slot
  const int32_t *tok_group;      // [n_tokens] row group of each token, -1 = uncovered
  const float *tok_pos;          // [n_tokens] or nullptr
  const float *slopes;           // [n_q_heads] or nullptr
  // decode tables
  const int32_t *path_off;       // [n_prompts+1]
  // first/last+1 decode range and a copy of the first range: one 16-byte read tells a source's
  // ranges when there is only one (the usual case), without a further dependent read
  const RangeDesc *shared_desc;  // [n_prompts] the shared segments of each prompt
  const RangeDesc *path_desc;    // [n_slots] each path slot
  const KeyRange *dec_ranges;
  int32_t n_items;
  int32_t n_wg;
  int32_t n_tokens;
  int32_t n_prompts;
  int32_t n_q_heads, n_kv_heads, head_dim;
};

}  // namespace sp

struct sp_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  std::string err;
  int n_cu = 256;             // compute units of the device (read once)
  // saliency accumulators (zero between launches); a block that became too small is kept until
  // sp_destroy, because a captured graph may still name it
  void *sal = nullptr;        // [launch counter][sal_slots accumulators][sal_rows per-row values]
  int32_t sal_slots = 0;
  int64_t sal_rows = 0;
  std::vector<void *> retired;
  // plan upload: one pinned staging buffer, one event that tells when its last copy has left it,
  // and the device blocks of destroyed plans, kept for the next plan
  void *stage = nullptr;
  size_t stage_bytes = 0;
  hipEvent_t stage_ev = nullptr;
  bool stage_busy = false;
  std::vector<std::pair<void *, size_t>> blob_pool;
  int refs = 1;               // the context itself + every live plan made on it
  bool closed = false;        // sp_destroy was called; the struct lives on until the last plan is gone
};

struct sp_plan {
  sp_ctx *ctx = nullptr;      // nullptr: host-only plan
  int32_t n_prompts = 0, n_segments = 0, n_tokens = 0, n_slots = 0;
  int32_t n_q_heads = 0, n_kv_heads = 0, head_dim = 0;
  sp_dtype dtype = SP_F32;
  int32_t heads_per_wg = 1;   // query heads stacked in one prefill workgroup
  int32_t waves_per_wg = 4;   // waves (32-row blocks) per prefill workgroup
  int32_t tile_rows = 0;      // token rows per prefill tile
  int32_t n_tiles = 0;
  int32_t n_wg = 0;           // persistent prefill workgroups (a multiple of 8)
  int32_t max_ranges = 0;
  int32_t max_dec_ranges = 0; // largest joined-cache range count bound per prompt (shared + per-path max)
  int64_t visible_pairs = 0;
  bool has_pos = false, has_slopes = false;
  // host copies
  std::vector<int32_t> prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path;
  std::vector<sp::RowGroup> groups;
  std::vector<sp::KeyRange> ranges;
  std::vector<sp::WorkItem> items;
  std::vector<int32_t> wg_begin;
  std::vector<int32_t> tok_group;      // token -> row group (host inspection)
  std::vector<int32_t> tok_group_dev;  // the same with tokens of cached segments set to -1
  std::vector<int32_t> path_off, shared_rng_beg, shared_rng_end, path_rng_beg, path_rng_end;
  std::vector<sp::KeyRange> dec_ranges;
  std::vector<int32_t> path_max_ranges;  // per prompt: max ranges of any single path
  std::vector<float> pos, slopes;        // copies of tok_pos / alibi_slopes (empty when not given)
  // device copies (one allocation)
  void *dev_blob = nullptr;
  size_t dev_blob_bytes = 0;  // capacity of the allocation
  sp::PlanDev dev{};
};

namespace sp {

// Kernel launchers (defined next to their kernels).  All return hipError_t from the launch.
struct PrefillArgs {
  const void *Q, *K, *V;
  void *O;
  int64_t q_tok_stride, q_head_stride, kv_tok_stride, kv_head_stride;
  float scale;
};
hipError_t launch_prefill_bf16(const sp_plan *plan, const PrefillArgs &a, hipStream_t s);
hipError_t launch_prefill_f32(const sp_plan *plan, const PrefillArgs &a, hipStream_t s);

hipError_t launch_saliency(const void *logits, sp_dtype dt, int64_t n_rows, int64_t vocab, int64_t row_stride,
                           const int32_t *target, const int32_t *row_path, const float *prior,
                           int32_t n_slots, int mode, void *scratch, int32_t cap_slots, float *score, hipStream_t s);
hipError_t saliency_static_scratch(int device, void **out);

hipError_t launch_topk(const float *score, const int32_t *path_off, int32_t n_prompts, int32_t n_paths_max,
                       int32_t k, int32_t *kept, hipStream_t s);

struct DecodeArgs {
  const int32_t *kept;
  int32_t k;
  const void *Kp, *Vp;
  int64_t kv_tok_stride, kv_head_stride;
  void *Kr, *Vr;
  float *pos_resp;
  int32_t resp_capacity;
  const int32_t *resp_len;
  int32_t resp_len_add;
  const float *new_pos;
  const void *q_new, *k_new, *v_new;
  void *o_out;
  float scale;
};
hipError_t launch_decode(const sp_plan *plan, const DecodeArgs &a, hipStream_t s);

}  // namespace sp
