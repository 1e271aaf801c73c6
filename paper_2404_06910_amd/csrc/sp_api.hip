// Host side of libsp.so: contexts, plan construction (validation, ancestor chains, tile work
// list, decode gather tables), argument checks and kernel dispatch.  No kernels live here.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "sp_internal.h"

namespace {

thread_local std::string g_err;   // failures of calls that have no context

sp_status fail(std::string *dst, sp_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  (dst ? *dst : g_err) = buf;
  return st;
}

std::string *errslot(sp_ctx *ctx) { return ctx ? &ctx->err : nullptr; }

#define SP_HIP(ctx, call)                                                                     \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(errslot(ctx), SP_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));   \
  } while (0)

// ---------------------------------------------------------------------------------------
// Table validation (Sec. 3.2: the prompt DAG; here a forest with one parent per node)
// ---------------------------------------------------------------------------------------
sp_status validate_table(const sp_segtable *t, int32_t n_q_heads, std::string *err) {
  if (!t) return fail(err, SP_ERR_INVALID_ARG, "segment table is NULL");
  if (t->n_prompts <= 0 || t->n_segments <= 0 || t->n_tokens <= 0)
    return fail(err, SP_ERR_INVALID_ARG, "n_prompts, n_segments and n_tokens must be positive");
  if (!t->prompt_seg_off || !t->seg_tok_start || !t->seg_tok_len || !t->seg_parent || !t->seg_path)
    return fail(err, SP_ERR_INVALID_ARG, "segment table has a NULL array");
  if (t->alibi_slopes && !t->tok_pos)
    return fail(err, SP_ERR_INVALID_ARG, "alibi_slopes given without tok_pos");
  const int32_t B = t->n_prompts, S = t->n_segments, T = t->n_tokens;
  if (t->prompt_seg_off[0] != 0 || t->prompt_seg_off[B] != S)
    return fail(err, SP_ERR_BAD_TABLE, "prompt_seg_off must start at 0 and end at n_segments");
  for (int32_t b = 0; b < B; ++b)
    if (t->prompt_seg_off[b + 1] <= t->prompt_seg_off[b])
      return fail(err, SP_ERR_BAD_TABLE, "prompt %d has no segments (prompt_seg_off not increasing)", b);
  std::vector<std::pair<int64_t, int64_t>> spans(S);
  for (int32_t s = 0; s < S; ++s) {
    const int64_t a = t->seg_tok_start[s], n = t->seg_tok_len[s];
    if (n <= 0) return fail(err, SP_ERR_BAD_TABLE, "segment %d has non-positive length", s);
    if (a < 0 || a + n > T) return fail(err, SP_ERR_BAD_TABLE, "segment %d token range out of [0, n_tokens)", s);
    spans[s] = {a, a + n};
  }
  std::sort(spans.begin(), spans.end());
  for (int32_t s = 1; s < S; ++s)
    if (spans[s].first < spans[s - 1].second)
      return fail(err, SP_ERR_BAD_TABLE, "token ranges of two segments overlap near token %lld",
                  (long long)spans[s].first);
  for (int32_t b = 0; b < B; ++b) {
    const int32_t s0 = t->prompt_seg_off[b], s1 = t->prompt_seg_off[b + 1];
    int32_t max_path = -1;
    for (int32_t s = s0; s < s1; ++s) {
      const int32_t p = t->seg_parent[s], path = t->seg_path[s];
      if (p != -1 && (p < s0 || p >= s))
        return fail(err, SP_ERR_BAD_TABLE, "segment %d: parent %d is not an earlier segment of the same prompt", s, p);
      if (path < -1) return fail(err, SP_ERR_BAD_TABLE, "segment %d: path id below -1", s);
      if (p != -1) {
        const int32_t ppath = t->seg_path[p];
        if (path == -1 && ppath != -1)
          return fail(err, SP_ERR_BAD_TABLE, "segment %d is shared but its parent lies on path %d", s, ppath);
        if (path >= 0 && ppath != -1 && ppath != path)
          return fail(err, SP_ERR_BAD_TABLE, "segment %d on path %d has a parent on path %d", s, path, ppath);
      }
      max_path = std::max(max_path, path);
    }
    std::vector<char> used(max_path + 1, 0);
    for (int32_t s = s0; s < s1; ++s)
      if (t->seg_path[s] >= 0) used[t->seg_path[s]] = 1;
    for (int32_t p = 0; p <= max_path; ++p)
      if (!used[p]) return fail(err, SP_ERR_BAD_TABLE, "prompt %d: path ids are not dense (path %d unused)", b, p);
  }
  if (t->tok_pos)
    for (int32_t i = 0; i < T; ++i)
      if (!std::isfinite(t->tok_pos[i])) return fail(err, SP_ERR_BAD_TABLE, "tok_pos[%d] is not finite", i);
  if (t->alibi_slopes)
    for (int32_t h = 0; h < n_q_heads; ++h)
      if (!std::isfinite(t->alibi_slopes[h]) || t->alibi_slopes[h] < 0.f)
        return fail(err, SP_ERR_BAD_TABLE, "alibi_slopes[%d] must be finite and >= 0", h);
  return SP_OK;
}

void push_range(std::vector<sp::KeyRange> &v, size_t first, int32_t start, int32_t len) {
  if (v.size() > first && v.back().tok_start + v.back().len == start)
    v.back().len += len;            // merge neighbours in token space
  else
    v.push_back({start, len});
}

template <class T>
size_t blob_reserve(size_t &off, const std::vector<T> &v) {
  off = (off + 255) & ~size_t(255);
  const size_t at = off;
  off += v.size() * sizeof(T) + 16;
  return at;
}

}  // namespace

// ---------------------------------------------------------------------------------------
// Context
// ---------------------------------------------------------------------------------------
extern "C" const char *sp_version(void) { return "sp-forkjoin 0.1 (gfx950)"; }

extern "C" const char *sp_last_error(const sp_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

static void *alloc_sal(int32_t slots, int64_t rows) {
  void *p = nullptr;
  const size_t bytes = sp::saliency_scratch_bytes(rows, slots);
  if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
  // zero before any stream may use it: the memset runs on the null stream, the kernels on the caller's
  if (hipMemset(p, 0, bytes) != hipSuccess || hipStreamSynchronize(nullptr) != hipSuccess) {
    (void)hipFree(p);
    return nullptr;
  }
  return p;
}

extern "C" sp_status sp_create(sp_ctx **out, int device, void *hip_stream) {
  if (!out) return fail(nullptr, SP_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  int n = 0;
  hipError_t e = hipGetDeviceCount(&n);
  if (e != hipSuccess || n <= 0)
    return fail(nullptr, SP_ERR_HIP, "no usable HIP device (%s)", e == hipSuccess ? "count is 0" : hipGetErrorString(e));
  if (device < 0 || device >= n || device >= sp::kMaxDevices)
    return fail(nullptr, SP_ERR_INVALID_ARG, "device %d out of range [0,%d)", device, std::min(n, sp::kMaxDevices));
  SP_HIP(nullptr, hipSetDevice(device));
  sp_ctx *c = new (std::nothrow) sp_ctx;
  if (!c) return fail(nullptr, SP_ERR_WORKSPACE, "out of host memory");
  c->device = device;
  c->stream = static_cast<hipStream_t>(hip_stream);
  int cu = 0;
  if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cu > 0) c->n_cu = cu;
  // the saliency accumulators are allocated here, so that the hot call allocates nothing in the usual case
  c->sal_slots = sp::kSalDefaultSlots;
  c->sal_rows = sp::kSalDefaultRows;
  c->sal = alloc_sal(c->sal_slots, c->sal_rows);
  if (!c->sal || hipEventCreateWithFlags(&c->stage_ev, hipEventDisableTiming) != hipSuccess) {
    if (c->sal) (void)hipFree(c->sal);
    delete c;
    return fail(nullptr, SP_ERR_WORKSPACE, "could not allocate the context's workspace");
  }
  *out = c;
  return SP_OK;
}

static void ctx_unref(sp_ctx *ctx) {
  if (--ctx->refs == 0) delete ctx;
}

extern "C" void sp_destroy(sp_ctx *ctx) {
  if (!ctx || ctx->closed) return;
  (void)hipSetDevice(ctx->device);
  if (ctx->stage_busy) (void)hipEventSynchronize(ctx->stage_ev);
  if (ctx->sal) (void)hipFree(ctx->sal);
  for (void *p : ctx->retired) (void)hipFree(p);
  for (auto &b : ctx->blob_pool) (void)hipFree(b.first);
  if (ctx->stage) (void)hipHostFree(ctx->stage);
  if (ctx->stage_ev) (void)hipEventDestroy(ctx->stage_ev);
  ctx->sal = nullptr; ctx->stage = nullptr; ctx->stage_ev = nullptr;
  ctx->retired.clear(); ctx->blob_pool.clear();
  ctx->closed = true;
  ctx_unref(ctx);
}

extern "C" sp_status sp_set_stream(sp_ctx *ctx, void *hip_stream) {
  if (!ctx) return fail(nullptr, SP_ERR_INVALID_ARG, "ctx is NULL");
  // plan tables are uploaded on the stream that was current when the plan was made: let the last
  // upload finish before work may be ordered on another stream
  if (ctx->stage_busy && static_cast<hipStream_t>(hip_stream) != ctx->stream) {
    SP_HIP(ctx, hipEventSynchronize(ctx->stage_ev));
    ctx->stage_busy = false;
  }
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  return SP_OK;
}

// Saliency workspace (per-row log-likelihoods, per-slot accumulators).  A block that is too small is
// replaced and kept until sp_destroy (a captured graph may still name it); nothing is ever freed inside a
// hot call, and the usual sizes never allocate: the block made in sp_create covers 65536 rows.
static sp_status ensure_sal(sp_ctx *ctx, int64_t n_rows, int32_t n_slots) {
  if (ctx->sal_slots >= n_slots && ctx->sal_rows >= n_rows) return SP_OK;
  int32_t slots = ctx->sal_slots;
  int64_t rows = ctx->sal_rows;
  while (slots < n_slots) slots *= 2;
  while (rows < n_rows) rows *= 2;
  void *p = alloc_sal(slots, rows);
  if (!p) return fail(&ctx->err, SP_ERR_WORKSPACE, "could not allocate the saliency workspace (%lld rows, %d slots)",
                      (long long)rows, slots);
  ctx->retired.push_back(ctx->sal);
  ctx->sal = p;
  ctx->sal_slots = slots;
  ctx->sal_rows = rows;
  return SP_OK;
}

namespace {

// Hand the items of an ordered work list to n_slots workers (n_slots a multiple of 8; worker s belongs
// to XCD s / (n_slots / 8)).  The list is cut into 8 contiguous, cost-balanced ranges, one per XCD, and
// inside a range the items go, in order, each to the worker with the least work so far (ties: the
// worker that has waited longest) -- the schedule a shared queue would produce, decided here.  At any
// moment an XCD therefore works on a window of consecutive items (the order of the list, chosen in
// build_plan, decides what that window touches in memory).  Costs are small
// positive integers; the least-loaded worker comes out of a bucket queue keyed by load, O(1) per item.
// Output: owner[i] = worker of item i, and begin[s] = first position of worker s's slice in the
// permuted list (items of a worker keep their order).  slow_milli[r]: relative slowness, in thousandths,
// of the workers of dispatch round r (worker index within its XCD / workers per round).
void hand_out(const std::vector<int32_t> &cost, int32_t n_slots, const int32_t *slow_milli, int32_t rounds,
              std::vector<int32_t> &owner, std::vector<int32_t> &begin) {
  // loads are kept in units of 1/16 of a cost unit so that the per-round weights (thousandths) fit
  const size_t n = cost.size();
  const int32_t per_xcd = n_slots / 8, per_round = std::max(1, per_xcd / rounds);
  int64_t total = 0;
  int32_t max_cost = 1;
  for (int32_t c : cost) { total += c; max_cost = std::max(max_cost, c); }
  size_t xcd_begin[9];
  std::fill(xcd_begin, xcd_begin + 9, n);
  xcd_begin[0] = 0;
  {
    int64_t acc = 0;
    int32_t c = 1;
    for (size_t i = 0; i < n && c < 8; ++i) {
      acc += cost[i];
      while (c < 8 && acc * 8 >= total * c) xcd_begin[c++] = i + 1;
    }
  }
  std::vector<int32_t> weight(per_xcd);
  for (int32_t w = 0; w < per_xcd; ++w) weight[w] = (16 * slow_milli[std::min(w / per_round, rounds - 1)] + 500) / 1000;
  const int32_t max_w = *std::max_element(weight.begin(), weight.end());
  owner.resize(n);
  begin.assign(n_slots + 1, 0);
  std::vector<int32_t> next(per_xcd), head, tail;
  for (int32_t x = 0; x < 8; ++x) {
    int64_t range_cost = 0;
    for (size_t i = xcd_begin[x]; i < xcd_begin[x + 1]; ++i) range_cost += cost[i];
    const size_t n_buckets = size_t((range_cost / per_xcd + 2 * int64_t(max_cost) + 2) * max_w);
    head.assign(n_buckets, -1);
    tail.assign(n_buckets, -1);
    for (int32_t w = 0; w < per_xcd; ++w) next[w] = w + 1 < per_xcd ? w + 1 : -1;   // all workers at load 0, in order
    head[0] = 0;
    tail[0] = per_xcd - 1;
    size_t lo = 0;
    for (size_t i = xcd_begin[x]; i < xcd_begin[x + 1]; ++i) {
      while (head[lo] < 0) ++lo;
      const int32_t w = head[lo];
      head[lo] = next[w];
      if (head[lo] < 0) tail[lo] = -1;
      size_t to = lo + size_t(cost[i]) * size_t(weight[w]);
      if (to >= n_buckets) to = n_buckets - 1;       // cannot happen: the least load never exceeds the mean
      next[w] = -1;
      if (tail[to] < 0) head[to] = w; else next[tail[to]] = w;
      tail[to] = w;
      owner[i] = x * per_xcd + w;
      ++begin[owner[i] + 1];
    }
  }
  for (int32_t g = 0; g < n_slots; ++g) begin[g + 1] += begin[g];
}

// Validation, row groups, work list and decode tables of a plan (host only).
sp_status build_plan(sp_ctx *ctx, const sp_segtable *t, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                     sp_dtype dtype, sp_plan *p) {
  std::string *err = errslot(ctx);
  if (n_q_heads <= 0 || n_kv_heads <= 0) return fail(err, SP_ERR_INVALID_ARG, "head counts must be positive");
  if (n_q_heads % n_kv_heads) return fail(err, SP_ERR_UNSUPPORTED, "n_q_heads must be a multiple of n_kv_heads");
  if (n_q_heads > 0xffff) return fail(err, SP_ERR_UNSUPPORTED, "more than 65535 query heads");
  if (head_dim != 64 && head_dim != 128) return fail(err, SP_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(err, SP_ERR_INVALID_ARG, "unknown dtype");
  sp_status st = validate_table(t, n_q_heads, err);
  if (st != SP_OK) return st;

  p->ctx = ctx;
  p->n_prompts = t->n_prompts; p->n_segments = t->n_segments; p->n_tokens = t->n_tokens;
  p->n_q_heads = n_q_heads; p->n_kv_heads = n_kv_heads; p->head_dim = head_dim; p->dtype = dtype;
  const int32_t B = t->n_prompts, S = t->n_segments;
  p->prompt_seg_off.assign(t->prompt_seg_off, t->prompt_seg_off + B + 1);
  p->seg_tok_start.assign(t->seg_tok_start, t->seg_tok_start + S);
  p->seg_tok_len.assign(t->seg_tok_len, t->seg_tok_len + S);
  p->seg_parent.assign(t->seg_parent, t->seg_parent + S);
  p->seg_path.assign(t->seg_path, t->seg_path + S);
  p->has_pos = t->tok_pos != nullptr;
  p->has_slopes = t->alibi_slopes != nullptr;
  if (t->tok_pos) p->pos.assign(t->tok_pos, t->tok_pos + t->n_tokens);
  if (t->alibi_slopes) p->slopes.assign(t->alibi_slopes, t->alibi_slopes + n_q_heads);

  // --- row groups: fuse a child that is packed right behind its parent into the parent's run
  std::vector<int32_t> group_of(S, -1), group_last;
  auto is_cached = [&](int32_t s) { return t->seg_cached && t->seg_cached[s] != 0; };
  // per row group: the row intervals [begin, end) that are computed (rows of cached segments are not)
  std::vector<std::vector<std::pair<int32_t, int32_t>>> live_rows;
  auto add_live = [&](int32_t g, int32_t begin, int32_t end) {
    auto &v = live_rows[g];
    if (!v.empty() && v.back().second == begin) v.back().second = end;
    else v.push_back({begin, end});
  };
  std::vector<int32_t> chain;
  for (int32_t b = 0; b < B; ++b) {
    for (int32_t s = t->prompt_seg_off[b]; s < t->prompt_seg_off[b + 1]; ++s) {
      const int32_t par = t->seg_parent[s];
      if (par >= 0) {
        const int32_t g = group_of[par];
        if (group_last[g] == par && t->seg_tok_start[s] == t->seg_tok_start[par] + t->seg_tok_len[par]) {
          group_of[s] = g;
          if (!is_cached(s)) add_live(g, p->groups[g].len, p->groups[g].len + t->seg_tok_len[s]);
          p->groups[g].len += t->seg_tok_len[s];
          group_last[g] = s;
          continue;
        }
      }
      sp::RowGroup rg{};
      rg.tok_start = t->seg_tok_start[s];
      rg.len = t->seg_tok_len[s];
      rg.prompt = b;
      rg.range_off = static_cast<int32_t>(p->ranges.size());
      chain.clear();
      for (int32_t a = par; a >= 0; a = t->seg_parent[a]) chain.push_back(a);
      int32_t anc = 0;
      for (auto it = chain.rbegin(); it != chain.rend(); ++it) {
        push_range(p->ranges, rg.range_off, t->seg_tok_start[*it], t->seg_tok_len[*it]);
        anc += t->seg_tok_len[*it];
      }
      rg.n_ranges = static_cast<int32_t>(p->ranges.size()) - rg.range_off;
      rg.anc_keys = anc;
      if (rg.n_ranges > sp::kMaxRanges)
        return fail(err, SP_ERR_UNSUPPORTED, "segment %d has %d disjoint ancestor key ranges (limit %d)", s,
                    rg.n_ranges, sp::kMaxRanges);
      p->max_ranges = std::max(p->max_ranges, rg.n_ranges);
      group_of[s] = static_cast<int32_t>(p->groups.size());
      group_last.push_back(s);
      p->groups.push_back(rg);
      live_rows.emplace_back();
      if (!is_cached(s)) add_live(group_of[s], 0, rg.len);
    }
  }
  p->tok_group.assign(t->n_tokens, -1);
  p->visible_pairs = 0;
  for (size_t g = 0; g < p->groups.size(); ++g) {
    const sp::RowGroup &rg = p->groups[g];
    std::fill(p->tok_group.begin() + rg.tok_start, p->tok_group.begin() + rg.tok_start + rg.len,
              static_cast<int32_t>(g));
    for (auto &iv : live_rows[g]) {                       // pairs of the rows that are computed
      const int64_t n = iv.second - iv.first;
      p->visible_pairs += n * rg.anc_keys + (int64_t(iv.second) * (iv.second + 1) - int64_t(iv.first) * (iv.first + 1)) / 2;
    }
  }
  // device copy of the token -> group map: tokens of cached segments produce no rows (fp32 kernel only)
  if (dtype == SP_F32) {
    p->tok_group_dev = p->tok_group;
    for (int32_t s = 0; s < S; ++s)
      if (is_cached(s))
        std::fill(p->tok_group_dev.begin() + t->seg_tok_start[s],
                  p->tok_group_dev.begin() + t->seg_tok_start[s] + t->seg_tok_len[s], -1);
  }

  const int32_t G = n_q_heads / n_kv_heads;
  const int n_cu = ctx ? ctx->n_cu : 256;
  struct Tile { int32_t group, row0, n_rows; };
  std::vector<Tile> tiles;                            // tiles of the current prompt
  // A tile streams every key up to its last row, so the partial tile of an interval goes first, where
  // that stream is shortest, and the full tiles end at the interval's end.
  auto tiles_of_prompt = [&](size_t &g, int32_t b, int32_t tile_rows) {
    tiles.clear();
    for (; g < p->groups.size() && p->groups[g].prompt == b; ++g)
      for (auto &iv : live_rows[g]) {
        const int32_t rem = (iv.second - iv.first) % tile_rows;
        if (rem) tiles.push_back({int32_t(g), iv.first, rem});
        for (int32_t r = iv.first + rem; r < iv.second; r += tile_rows) tiles.push_back({int32_t(g), r, tile_rows});
      }
    p->n_tiles += static_cast<int32_t>(tiles.size());
  };
  auto make_item = [&](const Tile &tl, int32_t head0, int32_t kv_head) {
    const sp::RowGroup &rg = p->groups[tl.group];
    sp::WorkItem w{};
    w.tok_start = rg.tok_start; w.row0 = tl.row0;
    w.n_rows = tl.n_rows;
    w.anc_keys = rg.anc_keys; w.range_off = rg.range_off; w.n_ranges = rg.n_ranges;
    w.head0 = head0 | (kv_head << 16);
    w.r0_start = rg.n_ranges > 0 ? p->ranges[rg.range_off].tok_start : 0;
    return w;
  };
  // --- prefill work list.  Query heads that share a KV head are stacked in one workgroup (4 waves for
  // 4 heads, else 2 waves), each wave owning 32 token rows of one head.
  // Persistent workgroups, 8 waves per compute unit.  The work list (ordered as stated below) is
  // handed out by hand_out() above; cost of an item = LDS stages streamed: one for Q plus the K/V stages,
  // plus the epilogue.  The workgroups that share a compute unit do not run equally fast: the instruction
  // arbiter serves the oldest wave of a SIMD first, so a workgroup dispatched in a later round (slot index
  // / workgroups per round; the dispatcher fills every compute unit once per round) takes 7-15 % longer for
  // the same work (measured from per-workgroup end times, stable from launch to launch).  Its load is
  // weighted accordingly so that all rounds end together.  Items are written straight to their place in
  // the permuted list, so that every workgroup reads one contiguous slice.
  p->heads_per_wg = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  p->waves_per_wg = p->heads_per_wg == 4 ? 4 : 2;
  p->tile_rows = 32 * (p->waves_per_wg / p->heads_per_wg);
  const int32_t n_hg = n_q_heads / p->heads_per_wg;
  {
    std::vector<Tile> all_tiles;
    std::vector<int32_t> prompt_tile_off(B + 1, 0);
    size_t g = 0;
    for (int32_t b = 0; b < B; ++b) {
      tiles_of_prompt(g, b, p->tile_rows);
      all_tiles.insert(all_tiles.end(), tiles.begin(), tiles.end());
      prompt_tile_off[b + 1] = static_cast<int32_t>(all_tiles.size());
    }
    const int32_t stage_keys = 16 * p->waves_per_wg;
    std::vector<int32_t> tile_cost(all_tiles.size());
    for (size_t i = 0; i < all_tiles.size(); ++i) {
      const sp::RowGroup &rg = p->groups[all_tiles[i].group];
      tile_cost[i] = 2 + (rg.anc_keys + all_tiles[i].row0 + all_tiles[i].n_rows + stage_keys - 1) / stage_keys;
    }
    const size_t n_items = all_tiles.size() * size_t(n_hg);
    // Order of the work list: [slice of head groups,] prompt, chunk of head groups, row group, head group of
    // the chunk, tile of the row group.  The tiles of one path come together (a later tile re-reads the K/V
    // rows that the earlier ones fetch), and the same path for the next head follows at once: the K/V (and
    // Q, O) rows of a token lie side by side in memory for all heads, so the workgroups of an XCD, which at
    // any time work on a window of consecutive items, touch a few contiguous regions instead of one head's
    // 256-byte rows strided over a whole prompt (measured against prompt, head group, tile: 7-14 % faster
    // with ungrouped heads, no change with grouped ones).  Every item of the window also streams its
    // ancestors' K/V, which the XCD's L2 (4 MB) has to keep for all heads of the chunk next to the paths' own
    // rows: the chunk is as many head groups as keep that shared part within kSharedKvBudget.  Measured
    // without slices on 32 ungrouped heads of 128 dims behind a 64-token preamble: chunks of 16 heads 167 us
    // and 1.04x the compulsory reads, all 32 heads 172 us and 1.21x, 8 heads 176 us; behind a 576-token
    // chain of kept documents one head at a time reads 0.99x, all heads together 3x at the same speed.
    constexpr int64_t kSharedKvBudget = int64_t(1) << 19;
    // When the head groups divide by the 8 XCDs, the list starts with a loop over 8 slices of them: the
    // cost-balanced cut into one contiguous range per XCD then falls on the slice boundaries, every XCD works
    // through all prompts on its own heads, and the 8 XCDs are at about the same tokens at the same time,
    // which keeps the memory-side accesses together across the whole 8 KB of a token (another 2 % at the
    // same traffic).
    const int32_t n_slice = n_hg % 8 == 0 ? 8 : 1, per_slice = n_hg / n_slice;
    auto for_each_item = [&](auto &&fn) {
      for (int32_t x = 0; x < n_slice; ++x)
      for (int32_t b = 0; b < B; ++b) {
        int32_t anc = 1;
        for (int32_t tl = prompt_tile_off[b]; tl < prompt_tile_off[b + 1]; ++tl)
          anc = std::max(anc, p->groups[all_tiles[tl].group].anc_keys);
        const int64_t per_hg = int64_t(anc) * 2 * head_dim * 2;          // K and V rows of one KV head, bf16
        const int32_t hc = int32_t(std::max<int64_t>(1, std::min<int64_t>(per_slice, kSharedKvBudget / per_hg)));
        for (int32_t h0 = x * per_slice; h0 < (x + 1) * per_slice; h0 += hc)
          for (int32_t a = prompt_tile_off[b], e = a; a < prompt_tile_off[b + 1]; a = e) {
            while (e < prompt_tile_off[b + 1] && all_tiles[e].group == all_tiles[a].group) ++e;
            for (int32_t hg = h0; hg < std::min((x + 1) * per_slice, h0 + hc); ++hg)
              for (int32_t tl = a; tl < e; ++tl) fn(tl, hg);
          }
      }
    };
    std::vector<int32_t> cost(n_items), owner;
    {
      size_t i = 0;
      for_each_item([&](int32_t tl, int32_t) { cost[i++] = tile_cost[tl]; });
    }
    p->n_wg = (((8 / p->waves_per_wg) * n_cu + 7) / 8) * 8;
    const int32_t rounds = 8 / p->waves_per_wg;
    static const int32_t four[4] = {1000, 1085, 1085, 1125}, two[2] = {1000, 1150}, one[1] = {1000};
    hand_out(cost, p->n_wg, rounds == 4 ? four : rounds == 2 ? two : one, rounds, owner, p->wg_begin);
    p->items.resize(n_items);
    std::vector<int32_t> at(p->wg_begin.begin(), p->wg_begin.end() - 1);
    size_t i = 0;
    for_each_item([&](int32_t tl, int32_t hg) {
      p->items[at[owner[i++]]++] = make_item(all_tiles[tl], hg * p->heads_per_wg, hg * p->heads_per_wg / G);
    });
  }

  // --- decode gather tables: shared ranges per prompt, ranges per path slot
  p->path_off.assign(B + 1, 0);
  for (int32_t b = 0; b < B; ++b) {
    int32_t mp = -1;
    for (int32_t s = t->prompt_seg_off[b]; s < t->prompt_seg_off[b + 1]; ++s) mp = std::max(mp, t->seg_path[s]);
    p->path_off[b + 1] = p->path_off[b] + mp + 1;
  }
  p->n_slots = p->path_off[B];
  p->shared_rng_beg.assign(B, 0);
  p->shared_rng_end.assign(B, 0);
  p->path_rng_beg.assign(p->n_slots, 0);
  p->path_rng_end.assign(p->n_slots, 0);
  p->path_max_ranges.assign(B, 0);
  std::vector<std::vector<int32_t>> segs_of_path;
  for (int32_t b = 0; b < B; ++b) {
    const size_t first = p->dec_ranges.size();
    const int32_t np = p->path_off[b + 1] - p->path_off[b];
    segs_of_path.assign(np, {});
    for (int32_t s = t->prompt_seg_off[b]; s < t->prompt_seg_off[b + 1]; ++s) {
      if (t->seg_path[s] < 0) push_range(p->dec_ranges, first, t->seg_tok_start[s], t->seg_tok_len[s]);
      else segs_of_path[t->seg_path[s]].push_back(s);
    }
    p->shared_rng_beg[b] = static_cast<int32_t>(first);
    p->shared_rng_end[b] = static_cast<int32_t>(p->dec_ranges.size());
    for (int32_t q = 0; q < np; ++q) {
      const size_t pf = p->dec_ranges.size();
      for (int32_t s : segs_of_path[q]) push_range(p->dec_ranges, pf, t->seg_tok_start[s], t->seg_tok_len[s]);
      const int32_t slot = p->path_off[b] + q;
      p->path_rng_beg[slot] = static_cast<int32_t>(pf);
      p->path_rng_end[slot] = static_cast<int32_t>(p->dec_ranges.size());
      p->path_max_ranges[b] = std::max(p->path_max_ranges[b], int32_t(p->dec_ranges.size() - pf));
    }
  }
  return SP_OK;
}

// Device copy of a plan's tables: every table is laid out in the context's pinned staging buffer and
// leaves in ONE asynchronous copy on the context's stream, into a device block taken from the blocks
// of destroyed plans when one is large enough (no hipMalloc / hipFree per request).  Work enqueued on
// that stream afterwards finds the tables in place.
sp_status upload_plan(sp_ctx *ctx, sp_plan *p, void *reuse_blob, size_t reuse_bytes) {
  const int32_t B = p->n_prompts;
  auto describe = [&](int32_t beg, int32_t end) {
    sp::RangeDesc d{beg, end, 0, 0};
    if (end > beg) { d.tok_start = p->dec_ranges[beg].tok_start; d.len = p->dec_ranges[beg].len; }
    return d;
  };
  std::vector<sp::RangeDesc> shared_desc(B), path_desc(p->n_slots);
  for (int32_t b = 0; b < B; ++b) shared_desc[b] = describe(p->shared_rng_beg[b], p->shared_rng_end[b]);
  for (int32_t q = 0; q < p->n_slots; ++q) path_desc[q] = describe(p->path_rng_beg[q], p->path_rng_end[q]);
  struct Piece { const void *src; size_t bytes, at; };
  std::vector<Piece> pieces;
  size_t off = 0;
  auto add = [&](const void *src, size_t bytes) {
    off = (off + 255) & ~size_t(255);
    pieces.push_back({src, bytes, off});
    off += bytes + 16;
    return pieces.back().at;
  };
  const size_t o_groups = add(p->groups.data(), p->groups.size() * sizeof(sp::RowGroup)),
               o_ranges = add(p->ranges.data(), p->ranges.size() * sizeof(sp::KeyRange)),
               o_items = add(p->items.data(), p->items.size() * sizeof(sp::WorkItem)),
               o_wgb = add(p->wg_begin.data(), p->wg_begin.size() * 4),
               o_tokg = add(p->tok_group_dev.data(), p->tok_group_dev.size() * 4),
               o_pos = add(p->pos.data(), p->pos.size() * 4), o_slopes = add(p->slopes.data(), p->slopes.size() * 4),
               o_poff = add(p->path_off.data(), p->path_off.size() * 4),
               o_sd = add(shared_desc.data(), shared_desc.size() * sizeof(sp::RangeDesc)),
               o_pd = add(path_desc.data(), path_desc.size() * sizeof(sp::RangeDesc)),
               o_dr = add(p->dec_ranges.data(), p->dec_ranges.size() * sizeof(sp::KeyRange));
  const size_t total = off + 256;
  SP_HIP(ctx, hipSetDevice(ctx->device));
  // device block: the plan's own (an update), else the smallest pooled block that fits, else a new one
  void *blob = nullptr;
  size_t blob_bytes = 0;
  if (reuse_blob && reuse_bytes >= total) {
    blob = reuse_blob; blob_bytes = reuse_bytes;
  } else {
    int best = -1;
    for (size_t i = 0; i < ctx->blob_pool.size(); ++i)
      if (ctx->blob_pool[i].second >= total && (best < 0 || ctx->blob_pool[i].second < ctx->blob_pool[best].second))
        best = int(i);
    if (best >= 0) {
      blob = ctx->blob_pool[best].first; blob_bytes = ctx->blob_pool[best].second;
      ctx->blob_pool.erase(ctx->blob_pool.begin() + best);
    } else {
      blob_bytes = ((total + total / 4) + 65535) & ~size_t(65535);      // headroom: the next table may be larger
      if (hipMalloc(&blob, blob_bytes) != hipSuccess)
        return fail(&ctx->err, SP_ERR_WORKSPACE, "could not allocate %zu bytes for the plan's tables", blob_bytes);
    }
  }
  auto give_back = [&]() { if (blob != reuse_blob) ctx->blob_pool.push_back({blob, blob_bytes}); };
  // staging buffer: wait until the previous upload has left it, grow if needed
  if (ctx->stage_busy) {
    hipError_t e = hipEventSynchronize(ctx->stage_ev);
    if (e != hipSuccess) { give_back(); return fail(&ctx->err, SP_ERR_HIP, "plan upload: %s", hipGetErrorString(e)); }
    ctx->stage_busy = false;
  }
  if (ctx->stage_bytes < total) {
    if (ctx->stage) (void)hipHostFree(ctx->stage);
    ctx->stage = nullptr;
    ctx->stage_bytes = 0;
    const size_t want = std::max(total + total / 4, size_t(1) << 20);
    if (hipHostMalloc(&ctx->stage, want, hipHostMallocDefault) != hipSuccess) {
      give_back();
      return fail(&ctx->err, SP_ERR_WORKSPACE, "could not allocate %zu bytes of pinned staging memory", want);
    }
    ctx->stage_bytes = want;
  }
  char *stg = static_cast<char *>(ctx->stage);
  for (auto &pc : pieces)
    if (pc.bytes) std::memcpy(stg + pc.at, pc.src, pc.bytes);
  hipError_t e = hipMemcpyAsync(blob, stg, total, hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess) e = hipEventRecord(ctx->stage_ev, ctx->stream);
  if (e != hipSuccess) { give_back(); return fail(&ctx->err, SP_ERR_HIP, "plan upload: %s", hipGetErrorString(e)); }
  ctx->stage_busy = true;
  if (p->dev_blob && p->dev_blob != blob) ctx->blob_pool.push_back({p->dev_blob, p->dev_blob_bytes});
  p->dev_blob = blob;
  p->dev_blob_bytes = blob_bytes;
  char *base = static_cast<char *>(blob);
  sp::PlanDev &d = p->dev;
  d = sp::PlanDev{};
  d.groups = reinterpret_cast<const sp::RowGroup *>(base + o_groups);
  d.ranges = reinterpret_cast<const sp::KeyRange *>(base + o_ranges);
  d.items = reinterpret_cast<const sp::WorkItem *>(base + o_items);
  d.wg_begin = reinterpret_cast<const int32_t *>(base + o_wgb);
  d.tok_group = reinterpret_cast<const int32_t *>(base + o_tokg);
  d.tok_pos = p->pos.empty() ? nullptr : reinterpret_cast<const float *>(base + o_pos);
  d.slopes = p->slopes.empty() ? nullptr : reinterpret_cast<const float *>(base + o_slopes);
  d.path_off = reinterpret_cast<const int32_t *>(base + o_poff);
  d.shared_desc = reinterpret_cast<const sp::RangeDesc *>(base + o_sd);
  d.path_desc = reinterpret_cast<const sp::RangeDesc *>(base + o_pd);
  d.dec_ranges = reinterpret_cast<const sp::KeyRange *>(base + o_dr);
  d.n_items = static_cast<int32_t>(p->items.size());
  d.n_wg = p->n_wg;
  d.n_tokens = p->n_tokens;
  d.n_prompts = p->n_prompts;
  d.n_q_heads = p->n_q_heads; d.n_kv_heads = p->n_kv_heads; d.head_dim = p->head_dim;
  return SP_OK;
}

}  // namespace

extern "C" sp_status sp_plan_create(sp_ctx *ctx, const sp_segtable *t, int32_t n_q_heads, int32_t n_kv_heads,
                                    int32_t head_dim, sp_dtype dtype, sp_plan **out) {
  std::string *err = errslot(ctx);
  if (!out) return fail(err, SP_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (ctx && ctx->closed) return fail(nullptr, SP_ERR_INVALID_ARG, "context was destroyed");
  sp_plan *p = new (std::nothrow) sp_plan;
  if (!p) return fail(err, SP_ERR_WORKSPACE, "out of host memory");
  sp_status st = build_plan(ctx, t, n_q_heads, n_kv_heads, head_dim, dtype, p);
  if (st == SP_OK && ctx) st = upload_plan(ctx, p, nullptr, 0);
  if (st != SP_OK) { delete p; return st; }
  if (ctx) ++ctx->refs;
  *out = p;
  return SP_OK;
}

extern "C" sp_status sp_plan_update(sp_plan *plan, const sp_segtable *t) {
  if (!plan) return fail(nullptr, SP_ERR_INVALID_ARG, "plan is NULL");
  sp_ctx *ctx = plan->ctx;
  if (ctx && ctx->closed) return fail(nullptr, SP_ERR_INVALID_ARG, "context was destroyed");
  sp_plan fresh;
  sp_status st = build_plan(ctx, t, plan->n_q_heads, plan->n_kv_heads, plan->head_dim, plan->dtype, &fresh);
  if (st != SP_OK) return st;                         // the plan is unchanged
  if (ctx) {
    // The old tables may still be read by kernels in flight on the stream; the copy that replaces
    // them is ordered behind those kernels on the same stream.
    fresh.dev_blob = plan->dev_blob;
    fresh.dev_blob_bytes = plan->dev_blob_bytes;
    st = upload_plan(ctx, &fresh, plan->dev_blob, plan->dev_blob_bytes);
    if (st != SP_OK) { fresh.dev_blob = nullptr; return st; }
  }
  *plan = std::move(fresh);
  fresh.dev_blob = nullptr;
  return SP_OK;
}

extern "C" void sp_plan_destroy(sp_plan *plan) {
  if (!plan) return;
  sp_ctx *ctx = plan->ctx;
  if (plan->dev_blob) {
    // keep the block for the next plan of this context (work that still reads it is ordered before
    // the next upload on the same stream); a closed context has nothing to keep it in
    if (ctx && !ctx->closed && ctx->blob_pool.size() < 8) ctx->blob_pool.push_back({plan->dev_blob, plan->dev_blob_bytes});
    else (void)hipFree(plan->dev_blob);
  }
  delete plan;
  if (ctx) ctx_unref(ctx);
}

extern "C" sp_status sp_plan_info(const sp_plan *p, int64_t info[8]) {
  if (!p || !info) return fail(nullptr, SP_ERR_INVALID_ARG, "NULL argument");
  info[0] = p->n_prompts; info[1] = p->n_segments; info[2] = p->n_tokens; info[3] = p->n_slots;
  info[4] = int64_t(p->groups.size()); info[5] = p->n_tiles;
  info[6] = int64_t(p->items.size());
  info[7] = p->max_ranges;
  return SP_OK;
}

extern "C" int64_t sp_plan_work_items(const sp_plan *p, int32_t *items_out, int64_t cap_items, int32_t *slot_begin_out,
                                      int64_t cap_slots) {
  if (!p || (cap_items > 0 && !items_out) || (cap_slots > 0 && !slot_begin_out)) return SP_ERR_INVALID_ARG;
  const std::vector<sp::WorkItem> &it = p->items;
  const std::vector<int32_t> &sb = p->wg_begin;
  static_assert(sizeof(sp::WorkItem) == 8 * sizeof(int32_t), "an item is 8 int32");
  const int64_t n = std::min<int64_t>(cap_items, int64_t(it.size()));
  if (n > 0) std::memcpy(items_out, it.data(), size_t(n) * sizeof(sp::WorkItem));
  for (int64_t i = 0; i < cap_slots && i < int64_t(sb.size()); ++i) slot_begin_out[i] = sb[i];
  return int64_t(it.size());
}

extern "C" int64_t sp_plan_key_ranges(const sp_plan *p, int32_t *out, int64_t cap) {
  if (!p || (cap > 0 && !out)) return SP_ERR_INVALID_ARG;
  const int64_t n = std::min<int64_t>(cap, int64_t(p->ranges.size()));
  if (n > 0) std::memcpy(out, p->ranges.data(), size_t(n) * sizeof(sp::KeyRange));
  return int64_t(p->ranges.size());
}

extern "C" int64_t sp_plan_work_slots(const sp_plan *p) {
  if (!p) return SP_ERR_INVALID_ARG;
  return int64_t(p->wg_begin.size()) - 1;
}

extern "C" int64_t sp_plan_visible_pairs(const sp_plan *p) { return p ? p->visible_pairs : SP_ERR_INVALID_ARG; }

extern "C" sp_status sp_plan_path_offsets(const sp_plan *p, int32_t *out) {
  if (!p || !out) return fail(nullptr, SP_ERR_INVALID_ARG, "NULL argument");
  std::copy(p->path_off.begin(), p->path_off.end(), out);
  return SP_OK;
}

extern "C" const int32_t *sp_plan_path_offsets_device(const sp_plan *p) { return p ? p->dev.path_off : nullptr; }

extern "C" int64_t sp_plan_visible_keys(const sp_plan *p, int32_t token, int32_t *out, int64_t cap) {
  if (!p || (cap > 0 && !out)) return SP_ERR_INVALID_ARG;
  if (token < 0 || token >= p->n_tokens) return SP_ERR_INVALID_ARG;
  const int32_t g = p->tok_group[token];
  if (g < 0) return 0;
  const sp::RowGroup &rg = p->groups[g];
  int64_t n = 0;
  auto emit = [&](int32_t tok) { if (n < cap) out[n] = tok; ++n; };
  for (int32_t r = 0; r < rg.n_ranges; ++r) {
    const sp::KeyRange &kr = p->ranges[rg.range_off + r];
    for (int32_t i = 0; i < kr.len; ++i) emit(kr.tok_start + i);
  }
  for (int32_t tok = rg.tok_start; tok <= token; ++tok) emit(tok);
  return n;
}

extern "C" int64_t sp_plan_joined_keys(const sp_plan *p, int32_t prompt, const int32_t *kept, int32_t k,
                                       int32_t *out, int64_t cap) {
  if (!p || (k > 0 && !kept) || (cap > 0 && !out) || k < 0) return SP_ERR_INVALID_ARG;
  if (prompt < 0 || prompt >= p->n_prompts) return SP_ERR_INVALID_ARG;
  int64_t n = 0;
  auto emit_ranges = [&](int32_t a, int32_t b) {
    for (int32_t r = a; r < b; ++r)
      for (int32_t i = 0; i < p->dec_ranges[r].len; ++i) {
        if (n < cap) out[n] = p->dec_ranges[r].tok_start + i;
        ++n;
      }
  };
  emit_ranges(p->shared_rng_beg[prompt], p->shared_rng_end[prompt]);
  const int32_t np = p->path_off[prompt + 1] - p->path_off[prompt];
  for (int32_t j = 0; j < k; ++j) {
    if (kept[j] < 0) continue;
    if (kept[j] >= np) return SP_ERR_BAD_TABLE;
    const int32_t slot = p->path_off[prompt] + kept[j];
    emit_ranges(p->path_rng_beg[slot], p->path_rng_end[slot]);
  }
  return n;
}

// ---------------------------------------------------------------------------------------
// a1 prefill
// ---------------------------------------------------------------------------------------
extern "C" sp_status sp_forkjoin_prefill(sp_ctx *ctx, const sp_plan *plan, const void *Q, const void *K,
                                         const void *V, void *O, int64_t q_tok_stride, int64_t q_head_stride,
                                         int64_t kv_tok_stride, int64_t kv_head_stride, float softmax_scale) {
  if (!ctx) return fail(nullptr, SP_ERR_INVALID_ARG, "ctx is NULL");
  if (!plan || !Q || !K || !V || !O) return fail(&ctx->err, SP_ERR_INVALID_ARG, "NULL argument");
  if (plan->ctx != ctx) return fail(&ctx->err, SP_ERR_INVALID_ARG, "plan was not created on this context");
  if (O == Q || O == K || O == V) return fail(&ctx->err, SP_ERR_INVALID_ARG, "O must not alias an input");
  const int64_t d = plan->head_dim;
  // Q and O are token-major; K and V may be token-major or head-major (a KV cache kept per head)
  if (q_head_stride < d || kv_head_stride < d || q_tok_stride < q_head_stride || q_tok_stride < d || kv_tok_stride < d)
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "strides smaller than head_dim, or Q/O not token-major");
  if (q_tok_stride >= (int64_t(1) << 26) || kv_tok_stride >= (int64_t(1) << 26))
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "token strides must be below 2^26 elements");
  if (kv_head_stride >= (int64_t(1) << 31))
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "K/V head stride must be below 2^31 elements");
  const int64_t align = plan->dtype == SP_BF16 ? 8 : 4;   // 16-byte vector loads
  if (q_tok_stride % align || q_head_stride % align || kv_tok_stride % align || kv_head_stride % align)
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "strides must be multiples of %lld elements", (long long)align);
  if ((reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V) |
       reinterpret_cast<uintptr_t>(O)) & 15)
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "Q, K, V, O must be 16-byte aligned");
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale))
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
  sp::PrefillArgs a{Q, K, V, O, q_tok_stride, q_head_stride, kv_tok_stride, kv_head_stride, softmax_scale};
  SP_HIP(ctx, hipSetDevice(ctx->device));
  hipError_t e = plan->dtype == SP_BF16 ? sp::launch_prefill_bf16(plan, a, ctx->stream)
                                        : sp::launch_prefill_f32(plan, a, ctx->stream);
  if (e != hipSuccess) return fail(&ctx->err, SP_ERR_HIP, "prefill launch: %s", hipGetErrorString(e));
  return SP_OK;
}

// ---------------------------------------------------------------------------------------
// a2 saliency
// ---------------------------------------------------------------------------------------
static sp_status check_saliency_args(sp_ctx *ctx, const void *logits, sp_dtype dtype, int64_t n_rows, int64_t vocab,
                                     int64_t row_stride, const int32_t *target, const int32_t *row_path,
                                     int32_t n_path_slots, sp_saliency_mode mode, const float *score) {
  if (!logits || !target || !row_path || !score) return fail(&ctx->err, SP_ERR_INVALID_ARG, "NULL argument");
  if (n_rows < 0 || vocab <= 0 || n_path_slots <= 0 || row_stride < vocab)
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "bad sizes (n_rows >= 0, vocab > 0, n_path_slots > 0, row_stride >= vocab)");
  if (dtype != SP_F32 && dtype != SP_BF16) return fail(&ctx->err, SP_ERR_INVALID_ARG, "unknown dtype");
  if (mode != SP_SALIENCY_SUM && mode != SP_SALIENCY_MEAN) return fail(&ctx->err, SP_ERR_INVALID_ARG, "unknown mode");
  if (n_rows > (int64_t(1) << 30)) return fail(&ctx->err, SP_ERR_UNSUPPORTED, "n_rows above 2^30");
  const int64_t esz = dtype == SP_BF16 ? 2 : 4;
  if ((reinterpret_cast<uintptr_t>(logits) & 15) || (row_stride * esz) % 16)
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "logits base and row stride must be 16-byte aligned");
  return SP_OK;
}

extern "C" sp_status sp_path_saliency(sp_ctx *ctx, const void *logits, sp_dtype dtype, int64_t n_rows,
                                      int64_t vocab, int64_t row_stride, const int32_t *target,
                                      const int32_t *row_path, const float *prior, int32_t n_path_slots,
                                      sp_saliency_mode mode, float *score) {
  if (!ctx) return fail(nullptr, SP_ERR_INVALID_ARG, "ctx is NULL");
  sp_status st = check_saliency_args(ctx, logits, dtype, n_rows, vocab, row_stride, target, row_path, n_path_slots,
                                     mode, score);
  if (st != SP_OK) return st;
  SP_HIP(ctx, hipSetDevice(ctx->device));
  st = ensure_sal(ctx, n_rows, n_path_slots);
  if (st != SP_OK) return st;
  hipError_t e = sp::launch_saliency(logits, dtype, n_rows, vocab, row_stride, target, row_path, prior,
                                     n_path_slots, int(mode), ctx->sal, ctx->sal_slots, score, ctx->stream);
  if (e != hipSuccess) return fail(&ctx->err, SP_ERR_HIP, "saliency launch: %s", hipGetErrorString(e));
  return SP_OK;
}

// The same computation for callers that cannot allocate: the accumulators are the library's static
// device array (one copy per GPU, shared by every call on that GPU).
extern "C" sp_status sp_path_saliency_static(sp_ctx *ctx, const void *logits, sp_dtype dtype, int64_t n_rows,
                                             int64_t vocab, int64_t row_stride, const int32_t *target,
                                             const int32_t *row_path, const float *prior, int32_t n_path_slots,
                                             sp_saliency_mode mode, float *score) {
  if (!ctx) return fail(nullptr, SP_ERR_INVALID_ARG, "ctx is NULL");
  sp_status st = check_saliency_args(ctx, logits, dtype, n_rows, vocab, row_stride, target, row_path, n_path_slots,
                                     mode, score);
  if (st != SP_OK) return st;
  if (n_path_slots > sp::kSalStaticSlots || n_rows > sp::kSalStaticRows)
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "%lld rows / %d path slots exceed the static scratch (%lld rows, %d slots)",
                (long long)n_rows, n_path_slots, (long long)sp::kSalStaticRows, sp::kSalStaticSlots);
  SP_HIP(ctx, hipSetDevice(ctx->device));
  void *scratch_dev = nullptr;
  hipError_t e = sp::saliency_static_scratch(ctx->device, &scratch_dev);
  if (e != hipSuccess) return fail(&ctx->err, SP_ERR_HIP, "static scratch address: %s", hipGetErrorString(e));
  e = sp::launch_saliency(logits, dtype, n_rows, vocab, row_stride, target, row_path, prior, n_path_slots, int(mode),
                          scratch_dev, sp::kSalStaticSlots, score, ctx->stream);
  if (e != hipSuccess) return fail(&ctx->err, SP_ERR_HIP, "saliency launch: %s", hipGetErrorString(e));
  return SP_OK;
}

// ---------------------------------------------------------------------------------------
// a3 top-k
// ---------------------------------------------------------------------------------------
extern "C" sp_status sp_prune_topk(sp_ctx *ctx, const float *score, const int32_t *path_off, int32_t n_prompts,
                                   int32_t n_paths_max, int32_t k, int32_t *kept) {
  if (!ctx) return fail(nullptr, SP_ERR_INVALID_ARG, "ctx is NULL");
  if (!score || !path_off || !kept) return fail(&ctx->err, SP_ERR_INVALID_ARG, "NULL argument");
  if (n_prompts <= 0 || k <= 0 || n_paths_max <= 0)
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "n_prompts, n_paths_max and k must be positive");
  if (n_paths_max > 4096) return fail(&ctx->err, SP_ERR_UNSUPPORTED, "more than 4096 paths per prompt");
  SP_HIP(ctx, hipSetDevice(ctx->device));
  hipError_t e = sp::launch_topk(score, path_off, n_prompts, n_paths_max, k, kept, ctx->stream);
  if (e != hipSuccess) return fail(&ctx->err, SP_ERR_HIP, "top-k launch: %s", hipGetErrorString(e));
  return SP_OK;
}

// ---------------------------------------------------------------------------------------
// a4 decode
// ---------------------------------------------------------------------------------------
extern "C" sp_status sp_pruned_decode(sp_ctx *ctx, const sp_plan *plan, const int32_t *kept, int32_t k,
                                      const void *K_prefill, const void *V_prefill, int64_t kv_tok_stride,
                                      int64_t kv_head_stride, void *K_resp, void *V_resp, float *pos_resp,
                                      int32_t resp_capacity, const int32_t *resp_len, int32_t resp_len_add,
                                      const float *new_pos, const void *q_new, const void *k_new,
                                      const void *v_new, void *o_out, float softmax_scale) {
  if (!ctx) return fail(nullptr, SP_ERR_INVALID_ARG, "ctx is NULL");
  if (!plan || !K_prefill || !V_prefill || !K_resp || !V_resp || !q_new || !k_new || !v_new || !o_out)
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "NULL argument");
  if (plan->ctx != ctx) return fail(&ctx->err, SP_ERR_INVALID_ARG, "plan was not created on this context");
  if (k < 0 || (k > 0 && !kept)) return fail(&ctx->err, SP_ERR_INVALID_ARG, "k < 0 or kept is NULL");
  if (resp_capacity <= 0 || resp_len_add < 0) return fail(&ctx->err, SP_ERR_INVALID_ARG, "bad response cache sizes");
  if (plan->has_slopes && (!pos_resp || !new_pos))
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "plan has bias slopes: pos_resp and new_pos are required");
  const int64_t d = plan->head_dim;
  const int64_t align = plan->dtype == SP_BF16 ? 8 : 4;
  if (kv_head_stride < d || kv_tok_stride < d || kv_tok_stride % align || kv_head_stride % align)
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "bad kv strides");
  if ((reinterpret_cast<uintptr_t>(K_prefill) | reinterpret_cast<uintptr_t>(V_prefill) |
       reinterpret_cast<uintptr_t>(K_resp) | reinterpret_cast<uintptr_t>(V_resp) | reinterpret_cast<uintptr_t>(q_new) |
       reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new) | reinterpret_cast<uintptr_t>(o_out)) & 15)
    return fail(&ctx->err, SP_ERR_UNSUPPORTED, "tensors must be 16-byte aligned");
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale))
    return fail(&ctx->err, SP_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
  // joined-cache range count bound: shared ranges + k * (largest per-path range count)
  int32_t worst = 0;
  for (int32_t b = 0; b < plan->n_prompts; ++b)
    worst = std::max(worst, plan->shared_rng_end[b] - plan->shared_rng_beg[b] + k * plan->path_max_ranges[b]);
  if (worst > 120) return fail(&ctx->err, SP_ERR_UNSUPPORTED, "joined cache has %d disjoint ranges (limit 120)", worst);
  sp::DecodeArgs a{kept, k, K_prefill, V_prefill, kv_tok_stride, kv_head_stride, K_resp, V_resp, pos_resp,
                   resp_capacity, resp_len, resp_len_add, new_pos, q_new, k_new, v_new, o_out, softmax_scale};
  SP_HIP(ctx, hipSetDevice(ctx->device));
  hipError_t e = sp::launch_decode(plan, a, ctx->stream);
  if (e != hipSuccess) return fail(&ctx->err, SP_ERR_HIP, "decode launch: %s", hipGetErrorString(e));
  return SP_OK;
}

// ---------------------------------------------------------------------------------------
// Equilibrium positions (Sec. 3.2.2 Eq. 1; App. B.2 Eq. 3 and Alg. 1; query rule of Alg. 3)
// ---------------------------------------------------------------------------------------
// Alg. 1 spaces the documents that fork behind the preamble by S/|d_i| (S the harmonic mean of their
// lengths, Eq. 1), so that all of them span [P, P + S).  Alg. 3 writes the query's start as the last
// position of document 1 with no "+ 1" and for document 1 only; it is read here as "one document span
// after the preamble", P + S, shared by all query copies with step 1: the only reading under which
// equal-length documents give exactly the classical positions of [preamble; document; query], which
// Sec. 3.2 requires of the ForkJoin prompt.  The same rule is applied to the children of EVERY node, so
// that iterated superposition (Sec. 4.1.2: forks behind a chain of kept documents) is covered: the
// children of a node start where the node's span ends, advance by S/len with S the harmonic mean of the
// sibling lengths, and an only child therefore continues with step 1.
extern "C" sp_status sp_equilibrium_positions(const sp_segtable *t, float *out) {
  if (!out) return fail(nullptr, SP_ERR_INVALID_ARG, "tok_pos_out is NULL");
  sp_segtable tt;
  if (t) { tt = *t; tt.tok_pos = nullptr; tt.alibi_slopes = nullptr; }
  sp_status st = validate_table(t ? &tt : nullptr, 0, nullptr);
  if (st != SP_OK) return st;
  const int32_t S = t->n_segments;
  // harmonic mean of the lengths of each node's children: S = n / sum(1/len)   (Eq. 1)
  std::vector<double> inv_sum(S, 0.0);
  std::vector<int32_t> n_child(S, 0);
  for (int32_t s = 0; s < S; ++s)
    if (t->seg_parent[s] >= 0) {
      inv_sum[t->seg_parent[s]] += 1.0 / double(t->seg_tok_len[s]);
      n_child[t->seg_parent[s]] += 1;
    }
  std::vector<double> span_end(S, 0.0);   // position right after the segment's span
  std::fill(out, out + t->n_tokens, 0.f);
  for (int32_t s = 0; s < S; ++s) {
    const int32_t par = t->seg_parent[s], len = t->seg_tok_len[s];
    double start = 0.0, step = 1.0, span = double(len);
    if (par >= 0) {
      span = double(n_child[par]) / inv_sum[par];
      step = span / double(len);
      start = span_end[par];
    }
    for (int32_t i = 0; i < len; ++i) {
      const double inc = step * double(i);        // ArangePositions (Eq. 3): start + i * step
      out[t->seg_tok_start[s] + i] = static_cast<float>(start + inc);
    }
    span_end[s] = start + span;
  }
  return SP_OK;
}
