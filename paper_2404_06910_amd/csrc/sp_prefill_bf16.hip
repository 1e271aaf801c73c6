// a1 (bf16 storage): ForkJoin prefill attention on the CDNA4 matrix cores.
//
// What is computed (Sec. 3.2, 3.2.1; App. B.3, the batched model call over per-path caches): every
// token attends to all tokens of its ancestor segments and causally to its own run of segments.
// The paper stresses that this is dense attention over many short sequences, not sparse
// attention over one long one; accordingly a work item is a tile of query rows of one row group,
// and its key list is the *virtual concatenation* [ancestor ranges root-to-leaf ; own run up to
// the tile's last row].  Over that virtual sequence the mask is purely causal with an offset, so
// every 32-key block is either fully visible, on the diagonal (per-element mask) or never
// enumerated at all.  Only the loader knows that the keys come from disjoint token ranges.
//
// Workgroup = 4 waves = 4 blocks of 32 query rows: HPW query heads that share one KV head times
// 4/HPW blocks of 32 tokens; three workgroups per compute unit.  Workgroups are persistent: each
// owns a contiguous slice of the work list and streams one unbroken sequence of 64-row LDS stages
// through a ring of three slots -- per item its Q tile (128 rows = two stages, the second only if
// it has rows), then its K/V tiles of 32 keys (32 K rows + 32 V rows).  Stages are filled by
// LDS-DMA (global_load_lds_dwordx4: global memory straight into LDS, no staging registers) issued
// two stages ahead of the math, also across item boundaries; one barrier per stage.  LDS rows are
// unpadded; 16-byte chunks are XOR-swizzled on the global-address side of the DMA so that both the
// row reads of K (ds_read_b128) and the transpose reads of V (ds_read_b64_tr_b16) are free of bank
// conflicts.
//
// Per wave and 32-key block, with the v_mfma_f32_32x32x16_bf16 tile shape:
//   S^T[key, row]  = K[key, :] . Q[row, :]      A = K fragment (LDS), B = Q fragment (registers)
//   O^T[d, row]   += V^T[d, key] . P^T[key, row] A = V fragment (LDS), B = P in registers
// In the 32x32 accumulator layout lane L holds column (L % 32) -- one query row -- and 16 of the
// 32 keys (rows 8*(i/4) + 4*(L/32) + i%4 for register i).  Hence the softmax statistics of a row
// live in one lane (plus one exchange with lane L^32), the rescale of O^T is a per-lane scalar,
// and the exponentiated scores are already in the B-operand layout of the second product: the
// k-slots of that MFMA are simply bound to the keys this lane holds, and the V fragment is read
// with the same key order.
#include <cstdlib>
#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

constexpr int kItemBatch = 32;     // work items staged in LDS at a time
#ifndef SP_OCC
#define SP_OCC 2
#endif
typedef bf16x4 __attribute__((address_space(3))) lds_bf16x4;
typedef unsigned char __attribute__((address_space(3))) lds_byte;

// max / sum partner exchange between lane L and lane L^32 (v_permlane32_swap)
__device__ __forceinline__ float xhalf_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS-DMA: every lane moves 16 bytes from its global address to LDS byte (lds_base + 16 * lane).
// The compiler does not track these loads; completion is awaited with explicit s_waitcnt vmcnt.
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory", "m0");
}

template <int D, int HPW, bool BIAS>
__global__ __launch_bounds__(256, SP_OCC) void prefill_bf16_kernel(PlanDev pd, const __bf16 *__restrict__ Q,
                                                                  const __bf16 *__restrict__ K,
                                                                  const __bf16 *__restrict__ V,
                                                                  __bf16 *__restrict__ O, uint32_t q_ts,
                                                                  uint32_t q_hs, uint32_t kv_ts, uint32_t kv_hs,
                                                                  float scale, int dbg) {
  constexpr int NW = 4;                    // waves
  constexpr int T = 64 * NW;               // threads
  constexpr int BK = 32;                   // keys per K/V stage; a stage holds 2*BK = 64 rows
  constexpr int ROWB = D * 2;              // bytes per LDS row (unpadded)
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int RPC = 256 / ROWB;          // rows per 256-byte bank cycle (1 or 2)
  constexpr int RG = 64 / CPR;             // rows moved by one wave-wide DMA instruction (4 or 8)
  constexpr int WROWS = 2 * BK / NW;       // stage rows filled by one wave (16)
  constexpr int NDMA = WROWS / RG;         // DMA instructions per wave and stage (4 or 2)
  constexpr int HALFB = BK * ROWB;         // bytes of the K half (= of the V half) of a stage
  constexpr int STAGEB = 2 * HALFB;
  constexpr int NS = 3;                    // ring slots; loads run NS-1 = 2 stages ahead
  constexpr int NJ = D / 16;               // MFMAs along head_dim for S
  constexpr int NC = D / 32;               // 32-wide output blocks of O^T

  // ring[slot]: BK K rows then BK V rows (half a Q tile uses the same 2*BK rows)
  __shared__ __attribute__((aligned(1024))) unsigned char ring[NS * STAGEB];
  __shared__ float Ps[NS][BK];
  __shared__ __attribute__((aligned(16))) WorkItem s_items[kItemBatch];

  // Chunk swizzles (16-byte chunk index XOR f(row)), row = index inside the K half or the V half:
  // K half: 16 consecutive rows reading the same chunk hit 16 different bank groups;
  // V half: the 4 rows x 32 bytes of a transpose read, and its neighbour 16 dims further, are disjoint.
  auto fK = [](int row) { return (row / RPC) % CPR; };
  auto fV = [](int row) { return 4 * ((row / RPC) % (CPR / 4)); };
  // byte offset of chunk ch of stage row r (0 .. 2*BK) inside a slot
  auto row_chunk = [&](int r, int ch) -> int {
    return r < BK ? r * ROWB + ((ch ^ fK(r)) * 16) : HALFB + (r - BK) * ROWB + ((ch ^ fV(r - BK)) * 16);
  };

  // Workgroup ids are dealt round-robin over the 8 XCDs; give every XCD a contiguous run of slices
  // so that workgroups sharing K/V rows (same prompt and KV head) share one L2.
  const int wg = (blockIdx.x % 8) * (pd.n_wg / 8) + blockIdx.x / 8;
  const int slice_begin = pd.wg_begin[wg], slice_end = pd.wg_begin[wg + 1];
  if (slice_begin >= slice_end) return;

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31,
            half = lane >> 5;
  const int G = pd.n_q_heads / pd.n_kv_heads;
  const float scale2 = scale * kLog2e;
  const uint32_t ring_base = (uint32_t)(size_t)(lds_byte *)ring;

  // DMA geometry of this lane: the wave fills stage rows [16*wave, 16*wave + 16), RG rows per
  // instruction; the lane writes slot position (lane % CPR) of row (lane / CPR) of that group and
  // therefore fetches the chunk that the swizzle maps there.
  const int drow = lane / CPR, dslot = lane % CPR;
  const bool dma_is_v = WROWS * wave >= BK;                 // this wave's rows lie in the V half

  // K-fragment read: row l32 (+32*sub), chunks 2j + half  ->  ((2j) ^ (f & ~1)) | ((half ^ f) & 1)
  const int kf_f = fK(l32), kf_lo = (half ^ kf_f) & 1, kf_fh = kf_f & ~1;
  // V transpose read: source lane s of a 16-lane group reads key row s/4, dims 4*(s%4)..+3 of a
  // 16-dim block; lane i receives dim i of the 4 keys.
  const int tr_row = (lane & 15) >> 2;
  const int tr_chlo = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1), tr_sub8 = (lane & 1) * 8;
  const int tr_f = fV(4 * half + tr_row);                  // rows differ from this by multiples of 8

  // stage ids of an item: -2 = Q tile rows 0..63, -1 = Q tile rows 64..127 (skipped when the
  // tile has no such rows), 0 .. n-1 = K/V stages
  auto n_stages = [](const WorkItem &w) { return (w.anc_keys + w.row0 + w.n_rows + BK - 1) / BK; };
  auto has_q1 = [](const WorkItem &w) { return 32 * (2 / HPW) < w.n_rows; };
  auto fetch_item = [&](int local) -> WorkItem {          // local index inside the staged batch
    const int4 a = *reinterpret_cast<const int4 *>(&s_items[local]);
    const int4 b = *(reinterpret_cast<const int4 *>(&s_items[local]) + 1);
    WorkItem w;
    w.tok_start = __builtin_amdgcn_readfirstlane(a.x); w.row0 = __builtin_amdgcn_readfirstlane(a.y);
    w.n_rows = __builtin_amdgcn_readfirstlane(a.z); w.anc_keys = __builtin_amdgcn_readfirstlane(a.w);
    w.range_off = __builtin_amdgcn_readfirstlane(b.x); w.n_ranges = __builtin_amdgcn_readfirstlane(b.y);
    w.head0 = __builtin_amdgcn_readfirstlane(b.z); w.r0_start = __builtin_amdgcn_readfirstlane(b.w);
    return w;
  };
  // virtual key -> packed token for item w
  auto map_tok = [&](const WorkItem &w, int vk) -> int {
    vk = min(vk, w.anc_keys + w.row0 + w.n_rows - 1);           // past the end: re-read the last key (masked)
    if (vk >= w.anc_keys) return w.tok_start + (vk - w.anc_keys);
    if (w.n_ranges == 1) return w.r0_start + vk;
    int tok = 0;
    for (int r = 0; r < w.n_ranges; ++r) {
      const KeyRange kr = pd.ranges[w.range_off + r];
      if (vk >= 0 && vk < kr.len) tok = kr.tok_start + vk;
      vk -= kr.len;
    }
    return tok;
  };
  // issue this wave's NDMA loads of stage st of item w into ring slot `slot`
  auto issue = [&](const WorkItem &w, int st, int slot) {
    const uint32_t lds0 = ring_base + slot * STAGEB + WROWS * wave * ROWB;   // the wave's rows are contiguous
#pragma unroll
    for (int m = 0; m < NDMA; ++m) {
      const int r = WROWS * wave + RG * m + drow;               // stage row filled by this lane
      const int rh = dma_is_v ? r - BK : r;                     // row inside its half
      const int ch = dslot ^ (dma_is_v ? fV(rh) : fK(rh));      // chunk that belongs at this position
      const __bf16 *src;
      if (st < 0) {
        const int tr = 64 * (st + 2) + r;                       // tile row; its 32-row slot = (token block, head)
        const int sl = tr >> 5;
        const int tok = w.tok_start + w.row0 + min(32 * (sl / HPW) + (tr & 31), w.n_rows - 1);
        src = Q + ((uint64_t)(uint32_t)tok * q_ts + (uint32_t)(w.head0 + sl % HPW) * q_hs + ch * 8);
      } else {
        const int tok = map_tok(w, st * BK + rh);
        src = (dma_is_v ? V : K) + ((uint64_t)(uint32_t)tok * kv_ts + (uint32_t)(w.head0 / G) * kv_hs + ch * 8);
      }
      dma16(src, lds0 + m * (RG * ROWB));
    }
  };

  bf16x8 qf[NJ];
  f32x16 o[NC];
  float m_run = kNegBig, l_run = 0.f, slope2 = 0.f, pos_q = 0.f;
  // geometry of the item whose accumulators are live (set at its Q stage)
  int head = 0, r0 = 0, my_limit = 0, wave_last = 0, wave_first_limit = 0;
  bool active = false;

  // normalise and store the live accumulators of item w.  `slot` is a ring slot nobody reads any
  // more and whose rows [16*wave, +16) this wave itself refills next, so they are private to it:
  // O^T (one query row per lane) is transposed through them, 16 rows at a time, so that the global
  // stores are whole 16-byte chunks of contiguous rows.
  auto epilogue = [&](const WorkItem &w, int slot) {
    if (!active) return;
    const float inv = 1.f / xhalf_sum(l_run);
    int zero;                                              // opaque 0: keeps the address arithmetic of the
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));          // epilogue out of the registers of the stream loop
    unsigned char *sl = ring + slot * STAGEB + zero;
    const int rows_here = min(32, w.n_rows - r0);
    __bf16 *ob = O + ((uint64_t)(uint32_t)(w.tok_start + w.row0 + r0) * q_ts + (uint32_t)head * q_hs);
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if ((l32 >> 4) == pass) {
        const int r = WROWS * wave + ((l32 + zero) & 15);
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 w4;
#pragma unroll
            for (int e = 0; e < 4; ++e) w4[e] = static_cast<__bf16>(o[c][4 * q4 + e] * inv);
            *reinterpret_cast<bf16x4 *>(sl + row_chunk(r, 4 * c + q4) + 8 * half) = w4;
          }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int i = 0; i < 16 * CPR / 64; ++i) {
        const int id = lane + zero + 64 * i, row = id / CPR, ch = id % CPR;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(sl + row_chunk(WROWS * wave + row, ch));
        if (16 * pass + row < rows_here && !(dbg & 4))
          st16(ob + ((uint64_t)(uint32_t)(16 * pass + row) * q_ts + ch * 8), v);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // LDS reads done before this wave's DMA refills
  };

  // everything a wave does for stage st of item w, resident in ring slot `slot`
  auto compute = [&](const WorkItem &w, int st, int slot, int it_parity) {
    const unsigned char *sl = ring + slot * STAGEB;
    if (st < 0) {
      // Q stages.  The 32-row block owned by a wave rotates with the item index so that the long
      // (late-row) blocks of the resident workgroups do not pile up on one SIMD.
      const int qs = (wave + it_parity) % NW;               // tile slot (token block, head) of this wave
      if (st == -2) {                                       // new item: geometry and fresh accumulators
        head = w.head0 + qs % HPW;
        r0 = 32 * (qs / HPW);
        active = r0 < w.n_rows;
        const int base = w.anc_keys + w.row0;               // virtual key of tile row 0 = its diagonal
        const int my_row = min(r0 + l32, w.n_rows - 1);     // clamped: padded lanes repeat the last row
        my_limit = base + my_row;
        wave_last = base + min(r0 + 31, w.n_rows - 1);
        wave_first_limit = base + r0;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[c][i] = 0.f;
        m_run = kNegBig;
        l_run = 0.f;
        if (BIAS) {
          slope2 = pd.slopes[head] * kLog2e;
          pos_q = pd.tok_pos[w.tok_start + w.row0 + my_row];
        }
      }
      if ((qs >> 1) == st + 2) {
        // this wave's Q rows are in the stage: B operand of S^T = K Q^T, k-slot block j covers
        // dims [16j + 8*half, +8)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          qf[j] = *reinterpret_cast<const bf16x8 *>(sl + row_chunk(32 * (qs & 1) + l32, 2 * j + half));
      }
      return;
    }
    {
      constexpr int sub = 0;
      const int vk0 = st * BK;
      if (!active || vk0 > wave_last || (dbg & 1)) return;   // block entirely above this wave's diagonal

      f32x16 s;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = 0.f;
      const unsigned char *krow = sl + (32 * sub + l32) * ROWB;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(krow + ((((2 * j) ^ kf_fh) | kf_lo) * 16));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[j], s, 0, 0, 0);
      }

      // scores in log2 units: t = s * scale2 (+ bias); masked entries -> -inf
      if (BIAS) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          s[i] = fmaf(s[i], scale2, slope2 * (Ps[slot][32 * sub + 8 * (i / 4) + 4 * half + (i % 4)] - pos_q));
      }
      if (vk0 + 31 > wave_first_limit) {                   // diagonal block: some rows see only part of it
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (vk0 + 8 * (i / 4) + 4 * half + (i % 4) > my_limit) s[i] = -INFINITY;
      }
      float mx = fmaxf(s[0], s[1]);
#pragma unroll
      for (int i = 2; i < 16; ++i) mx = fmaxf(mx, s[i]);
      if (!BIAS) mx *= scale2;                             // scale2 > 0: max commutes with the scaling
      mx = xhalf_max(mx);
      // The reference maximum is allowed to lag by up to 8 (factor 256 in p), which fp32 sums and
      // bf16 P absorb; the accumulator registers are rescaled only when some row exceeds that.
      if (__any(mx > m_run + 8.f)) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[c][i] *= alpha;
      }
      float ls = 0.f;
      bf16x8 pb[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = BIAS ? fast_exp2(s[i] - m_run) : fast_exp2(fmaf(s[i], scale2, -m_run));
        ls += p;
        pb[i / 8][i % 8] = static_cast<__bf16>(p);
      }
      l_run += ls;
      const unsigned char *vrow = sl + HALFB + (32 * sub + 4 * half + tr_row) * ROWB + tr_sub8;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int choff = (((4 * c) ^ tr_f) + tr_chlo) * 16;
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const unsigned char *vp = vrow + 16 * mm * ROWB + choff;
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * ROWB));
          const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[mm], o[c], 0, 0, 0);
        }
      }
    }
  };

  for (int batch = slice_begin; batch < slice_end; batch += kItemBatch) {
    const int n_local = min(kItemBatch, slice_end - batch);
    __syncthreads();                                     // previous batch fully consumed
    for (int i = tid; i < n_local * 2; i += T)
      reinterpret_cast<int4 *>(s_items)[i] = reinterpret_cast<const int4 *>(pd.items + batch)[i];
    __syncthreads();

    // cursors: c = stage being computed (ring slot c_slot), l = next stage to issue (two ahead)
    int c_it = 0, c_st = -2, l_it = 0, l_st = -2, c_slot = 0, l_slot = 0;
    WorkItem cw = fetch_item(0), lw = cw, pw = cw;         // pw: item whose epilogue is pending
    bool pending = false;
    auto advance = [&](int &it, int &st, WorkItem &w) {
      if (st == -2) st = has_q1(w) ? -1 : 0;
      else if (st + 1 < n_stages(w)) st += 1;
      else {
        it += 1;
        st = -2;
        if (it < n_local) w = fetch_item(it);
      }
    };
    auto issue_next = [&]() {                              // issue the stage at the load cursor, advance it
      if (l_it < n_local) {
        if (!(dbg & 2)) issue(lw, l_st, l_slot);
        if (BIAS && l_st >= 0 && tid < BK) Ps[l_slot][tid] = pd.tok_pos[map_tok(lw, l_st * BK + tid)];
        advance(l_it, l_st, lw);
        l_slot = l_slot + 1 == NS ? 0 : l_slot + 1;
      }
    };
    issue_next();
    issue_next();                                          // every item has at least two stages

    while (true) {
      // Wait for the stage at the compute cursor.  This wave has issued that stage and possibly
      // one younger one: all but the youngest stage's loads must have landed (all of them when
      // nothing younger is in flight); then meet the other waves.
      const int ahead = l_slot - c_slot + (l_slot < c_slot ? NS : 0);   // stages issued, not computed: 1 or 2
      if (ahead == 2) {
        if (NDMA == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");                       // no LDS access may move above the barrier
      if (pending) {                                       // the previous step finished an item
        epilogue(pw, c_slot == 0 ? NS - 1 : c_slot - 1);
        pending = false;
      }
      issue_next();
      compute(cw, c_st, c_slot, c_it + batch);
      if (c_st + 1 >= n_stages(cw)) { pw = cw; pending = true; }
      advance(c_it, c_st, cw);
      c_slot = c_slot + 1 == NS ? 0 : c_slot + 1;
      if (c_it >= n_local) break;
    }
    // drain: the last item's accumulators
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    epilogue(pw, c_slot == 0 ? NS - 1 : c_slot - 1);
  }
}

template <int D, int HPW>
static hipError_t launch_hpw(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  const dim3 grid(unsigned(plan->dev.n_wg));
  const char *e = getenv("SP_DBG");
  const int dbg = e ? atoi(e) : 0;
  const __bf16 *Q = static_cast<const __bf16 *>(a.Q), *K = static_cast<const __bf16 *>(a.K),
               *V = static_cast<const __bf16 *>(a.V);
  __bf16 *O = static_cast<__bf16 *>(a.O);
  const uint32_t qts = uint32_t(a.q_tok_stride), qhs = uint32_t(a.q_head_stride), kts = uint32_t(a.kv_tok_stride),
                 khs = uint32_t(a.kv_head_stride);
  if (plan->has_slopes)
    hipLaunchKernelGGL((prefill_bf16_kernel<D, HPW, true>), grid, dim3(256), 0, s, plan->dev, Q, K, V, O,
                       qts, qhs, kts, khs, a.scale, dbg);
  else
    hipLaunchKernelGGL((prefill_bf16_kernel<D, HPW, false>), grid, dim3(256), 0, s, plan->dev, Q, K, V, O,
                       qts, qhs, kts, khs, a.scale, dbg);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  switch (plan->heads_per_wg) {
    case 4: return launch_hpw<D, 4>(plan, a, s);
    case 2: return launch_hpw<D, 2>(plan, a, s);
    default: return launch_hpw<D, 1>(plan, a, s);
  }
}

hipError_t launch_prefill_bf16(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  return plan->head_dim == 128 ? launch_d<128>(plan, a, s) : launch_d<64>(plan, a, s);
}

}  // namespace sp
