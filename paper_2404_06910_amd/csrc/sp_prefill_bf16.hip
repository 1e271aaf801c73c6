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
// Workgroup = NW waves = NW blocks of 32 query rows: HPW query heads that share one KV head times
// NW/HPW blocks of 32 tokens (4 waves when 4 heads share a KV head; else 2 waves, so that the
// causal imbalance between early and late row blocks stays inside a pair).  Workgroups are
// persistent: each owns a cost-balanced slice of the (permuted) work list, staged in LDS, and
// streams one unbroken sequence of stages through two LDS slots -- for every item first its Q tile
// (32*NW rows = one stage), then its K/V tiles of 16*NW keys.  A stage is moved by LDS-DMA (global
// memory straight into LDS, no staging registers) while the waves work on the other slot, also
// across item boundaries, so no item pays a cold start; one barrier per stage.  O^T tiles leave
// through LDS as whole 16-byte chunks of contiguous rows.
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
#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

constexpr int kItemBatch = 32;     // work items staged in LDS at a time
constexpr int kRangeCache = 8;     // ancestor ranges per item kept in LDS beside them
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

// LDS-DMA: every lane moves 16 bytes from its global address straight into LDS byte
// (lds_base + 16 * lane); no staging registers.  The compiler does not track these loads:
// completion is awaited with an explicit s_waitcnt vmcnt(0) before the stage barrier.
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory", "m0");
}

// The same with the address split into a wave-uniform base (scalar registers) and a 32-bit per-lane
// byte offset: no vector arithmetic per instruction and no 64-bit per-lane pointers to keep alive.
__device__ __forceinline__ void dma16s(const void *sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
               : "memory", "m0");
}

// One dword per lane, 64 consecutive dwords in LDS: the positions of a stage's keys.
__device__ __forceinline__ void dma4(const void *gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_base), "v"(gptr) : "memory", "m0");
}

// A wave-uniform float through the scalar data path (a read; its counter is not the vector one).
__device__ __forceinline__ float sload_f32(const float *p) {
  float v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
  return v;
}

template <int D, int HPW, int NW, bool BIAS>
__global__ __launch_bounds__(64 * NW, 2) void prefill_bf16_kernel(PlanDev pd, const __bf16 *__restrict__ Q,
                                                                  const __bf16 *__restrict__ K,
                                                                  const __bf16 *__restrict__ V,
                                                                  __bf16 *__restrict__ O, uint32_t q_ts,
                                                                  uint32_t q_hs, uint32_t kv_ts, uint32_t kv_hs,
                                                                  float scale) {
  constexpr int T = 64 * NW;               // threads
  constexpr int BK = 16 * NW;              // keys per K/V stage; a stage holds 2*BK = 32*NW rows
  constexpr int ROWB = D * 2;              // bytes per LDS row (unpadded)
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int RPC = 256 / ROWB;          // rows per 256 bytes (1 or 2)
  constexpr int RG = 64 / CPR;             // rows moved by one wave-wide DMA instruction (4 or 8)
  constexpr int NDMA = 32 / RG;            // DMA instructions per wave and stage: a wave fills 32 rows
  constexpr int HALFB = BK * ROWB;         // bytes of the K half (= of the V half) of a stage
  constexpr int STAGEB = 2 * HALFB;
  constexpr int NJ = D / 16;               // MFMAs along head_dim for S
  constexpr int NC = D / 32;               // 32-wide output blocks of O^T
  static_assert(NW % HPW == 0 && NW % 2 == 0, "tile shape");
  static_assert(2 * STAGEB <= 65536, "DMA destinations are kept below 64 KB");

  // Two stage slots.  A slot is 2*BK rows: K rows then V rows (a Q tile uses all 2*BK rows).  Rows
  // are unpadded (the DMA writes 1 KB runs); instead the 16-byte chunks of a row are XOR-swizzled
  // on the global-address side, so that the row reads of K and Q (ds_read_b128, 16 consecutive rows,
  // same chunk) and the transpose reads of V (4 rows x 32 bytes per 16 lanes) spread over the banks.
  __shared__ __attribute__((aligned(1024))) unsigned char ring[2 * STAGEB];
  __shared__ __attribute__((aligned(256))) float Ps[2][BK < 64 ? 64 : BK];   // key positions (bias); one 64-lane DMA each
  __shared__ __attribute__((aligned(256))) float Pq[64];                     // positions of the rows of the Q tile in flight
  __shared__ __attribute__((aligned(16))) WorkItem s_items[kItemBatch];
  __shared__ KeyRange s_ranges[kItemBatch][kRangeCache];       // first ancestor ranges of each staged item
  auto fK = [](int row) { return (row / RPC) % CPR; };
  auto fV = [](int row) { return 4 * ((row / RPC) % (CPR / 4)); };

  // Workgroup ids are dealt round-robin over the 8 XCDs (id % 8).  The host has given every XCD a
  // contiguous range of the work list and handed its items out in order to that XCD's workgroup
  // slots, so the workgroups of an XCD work on a moving window of consecutive items and share
  // their K/V rows through that XCD's L2.  Slot s = xcd * (n_wg / 8) + id / 8 owns items [x0, x1).
  const int wg_slot = (blockIdx.x % 8) * (pd.n_wg / 8) + blockIdx.x / 8;
  const int x0 = pd.wg_begin[wg_slot], x1 = pd.wg_begin[wg_slot + 1];
  const int n_mine = x1 - x0;
  if (n_mine <= 0) return;

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31,
            half = lane >> 5;
  const float scale2 = scale * kLog2e;
  const uint32_t ring_base = (uint32_t)(size_t)(lds_byte *)ring;
  unsigned char *const ringp = ring;

  // ---- DMA geometry.  Wave w fills stage rows [32w, 32w + 32): the K half belongs to the first
  // NW/2 waves, the V half to the others; a Q tile's 32-row slot w is filled by wave w.  One
  // instruction moves RG rows; this lane writes chunk position (lane % CPR) of row (lane / CPR)
  // of the group and therefore fetches the chunk that the swizzle maps there.
  const int drow = lane / CPR, dslot = lane % CPR;
  const bool dma_is_v = wave >= NW / 2;
  const int rbase = 32 * (wave % (NW / 2));                   // first row of this wave inside its half
  uint32_t xkv[NDMA];                                         // swizzled chunk byte offsets per instruction
#pragma unroll
  for (int m = 0; m < NDMA; ++m)
    xkv[m] = (uint32_t)(dslot ^ (dma_is_v ? fV(rbase + RG * m + drow) : fK(rbase + RG * m + drow))) * 16;
  auto xq = [&](int m) { return (uint32_t)(dslot ^ fK(RG * m + drow)) * 16; };   // Q tile: fK on every row
  const uint32_t kv_row_off = (uint32_t)drow * kv_ts * 2, q_row_off = (uint32_t)drow * q_ts * 2;
  const char *Qb = reinterpret_cast<const char *>(Q);
  const char *KVb = reinterpret_cast<const char *>(dma_is_v ? V : K);

  // ---- fragment-read geometry
  // K / Q rows: row l32 (+ multiples of 32), chunk 2j + half  ->  ((2j) ^ (f & ~1)) | ((half ^ f) & 1)
  const int kf_f = fK(l32), kf_lo = (half ^ kf_f) & 1, kf_fh = kf_f & ~1;
  // V transpose read: source lane s of a 16-lane group hands in key row s/4, dims 4*(s%4)..+3 of a
  // 16-dim block, and lane i receives dim i of the 4 keys.
  const int tr_row = (lane & 15) >> 2;
  const int tr_chlo = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1), tr_sub8 = (lane & 1) * 8;
  const int tr_f = fV(4 * half + tr_row);                     // the other rows differ by multiples of 8

  // bias state: slope and position of the wave's query row.  The positions of a stage's keys and of
  // a tile's rows travel by DMA like the rows themselves and the slope through the scalar path, so
  // the stage loop holds no vector load that the compiler tracks: a wait of its own for such a load
  // would also wait for the DMA of the next stage.
  float slope2 = 0.f, pos_q = 0.f;
  static_assert(32 * NW / HPW <= 64, "one DMA instruction carries the positions of a Q tile");
  const uint32_t ps_base = (uint32_t)(size_t)(lds_byte *)&Ps[0][0];
  const uint32_t pq_base = (uint32_t)(size_t)(lds_byte *)&Pq[0];
  constexpr uint32_t kPsSlotB = sizeof(Ps) / 2;

  // a work item as the loop keeps it (all fields wave-uniform)
  struct Item {
    int tok_start, row0, n_rows, anc_keys, range_off, n_ranges, head0, kv_head, r0_start;
  };
  // virtual key -> packed token for item w
  auto map_tok = [&](const Item &w, int local, int vk) -> int {
    vk = min(vk, w.anc_keys + w.row0 + w.n_rows - 1);           // past the end: re-read the last key (masked)
    if (vk >= w.anc_keys) return w.tok_start + (vk - w.anc_keys);
    if (w.n_ranges == 1) return w.r0_start + vk;
    int tok = 0;
    if (w.n_ranges <= kRangeCache) {                            // the LDS copy, else the plan's table
      for (int r = 0; r < w.n_ranges; ++r) {
        const int2 kr = *reinterpret_cast<const int2 *>(&s_ranges[local][r]);
        if (vk >= 0 && vk < kr.y) tok = kr.x + vk;
        vk -= kr.y;
      }
    } else {
      for (int r = 0; r < w.n_ranges; ++r) {
        const KeyRange kr = pd.ranges[w.range_off + r];
        if (vk >= 0 && vk < kr.len) tok = kr.tok_start + vk;
        vk -= kr.len;
      }
    }
    return tok;
  };
  // issue this wave's DMA loads of stage st of item w (st = -1: the Q tile) into slot `slot`
  auto issue = [&](const Item &w, int local, int st, int slot) {
    const uint32_t lds = ring_base + slot * STAGEB + wave * (32 * ROWB);
    if (st < 0) {
      const int tb = 32 * (wave / HPW);                       // first tile row of this wave's Q rows
      const uint64_t hoff = (uint64_t)(uint32_t)(w.head0 + wave % HPW) * q_hs * 2;
      if (BIAS && wave == 0) dma4(pd.tok_pos + (w.tok_start + w.row0 + min(lane, w.n_rows - 1)), pq_base);
      if (w.n_rows == 32 * NW / HPW) {
        // full tile: consecutive tokens, everything but the lane's own offset is wave-uniform
        const uint64_t o0 = (uint64_t)(uint32_t)(w.tok_start + w.row0 + tb) * q_ts * 2 + hoff;
#pragma unroll
        for (int m = 0; m < NDMA; ++m)
          dma16s(Qb + (o0 + (uint64_t)(RG * m) * q_ts * 2), q_row_off + xq(m), lds + m * (RG * ROWB));
      } else {
#pragma unroll
        for (int m = 0; m < NDMA; ++m) {
          const int row = min(tb + RG * m + drow, w.n_rows - 1);   // rows past the tile repeat its last row
          dma16(Qb + ((uint64_t)(uint32_t)(w.tok_start + w.row0 + row) * q_ts * 2 + hoff + xq(m)),
                lds + m * (RG * ROWB));
        }
      }
    } else {
      // A stage whose BK keys are consecutive tokens (inside the own run and not past its end, or
      // inside a single ancestor range) needs no per-lane token lookup.
      const int vk0 = st * BK;
      int tok0 = -1;
      if (vk0 >= w.anc_keys) {
        if (vk0 + BK <= w.anc_keys + w.row0 + w.n_rows) tok0 = w.tok_start + (vk0 - w.anc_keys);
      } else if (vk0 + BK <= w.anc_keys) {
        if (w.n_ranges == 1) {
          tok0 = w.r0_start + vk0;
        } else if (w.n_ranges <= kRangeCache) {
          // several ancestor ranges (cached paths, chains of kept documents): find the one that
          // holds the whole stage, if any, in the LDS copy of the ranges
          int acc = 0;
          for (int r = 0; r < w.n_ranges; ++r) {
            const int2 kr = *reinterpret_cast<const int2 *>(&s_ranges[local][r]);
            const int start = __builtin_amdgcn_readfirstlane(kr.x), len = __builtin_amdgcn_readfirstlane(kr.y);
            if (vk0 >= acc && vk0 + BK <= acc + len) tok0 = start + (vk0 - acc);
            acc += len;
          }
        }
      }
      const uint64_t hoff = (uint64_t)(uint32_t)w.kv_head * kv_hs * 2;
      if (tok0 >= 0) {
        const uint64_t o0 = (uint64_t)(uint32_t)(tok0 + rbase) * kv_ts * 2 + hoff;
#pragma unroll
        for (int m = 0; m < NDMA; ++m)
          dma16s(KVb + (o0 + (uint64_t)(RG * m) * kv_ts * 2), kv_row_off + xkv[m], lds + m * (RG * ROWB));
        if (BIAS && wave == 0) dma4(pd.tok_pos + (tok0 + min(lane, BK - 1)), ps_base + slot * kPsSlotB);
      } else {
#pragma unroll
        for (int m = 0; m < NDMA; ++m) {
          const int tok = map_tok(w, local, vk0 + rbase + RG * m + drow);
          dma16(KVb + ((uint64_t)(uint32_t)tok * kv_ts * 2 + hoff + xkv[m]), lds + m * (RG * ROWB));
        }
        if (BIAS && wave == 0)
          dma4(pd.tok_pos + map_tok(w, local, vk0 + min(lane, BK - 1)), ps_base + slot * kPsSlotB);
      }
    }
  };
  // all loads of this wave have landed; then meet the other waves
  auto land_and_sync = [&](int slot) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  // Work items are read from an LDS copy of the slice (no pointer chasing in the stream loop).
  auto fetch_item = [&](int local) -> Item {              // local index inside the staged batch
    const int4 a = *reinterpret_cast<const int4 *>(&s_items[local]);
    const int4 b = *(reinterpret_cast<const int4 *>(&s_items[local]) + 1);
    Item w;
    w.tok_start = __builtin_amdgcn_readfirstlane(a.x); w.row0 = __builtin_amdgcn_readfirstlane(a.y);
    w.n_rows = __builtin_amdgcn_readfirstlane(a.z); w.anc_keys = __builtin_amdgcn_readfirstlane(a.w);
    w.range_off = __builtin_amdgcn_readfirstlane(b.x); w.n_ranges = __builtin_amdgcn_readfirstlane(b.y);
    const int heads = __builtin_amdgcn_readfirstlane(b.z);    // query head | KV head << 16
    w.head0 = heads & 0xffff; w.kv_head = heads >> 16;
    w.r0_start = __builtin_amdgcn_readfirstlane(b.w);
    return w;
  };
  auto n_stages = [](const Item &w) { return (w.anc_keys + w.row0 + w.n_rows + BK - 1) / BK; };

  bf16x8 qf[NJ];
  f32x16 o[NC];
  float m_run = kNegBig, l_run = 0.f;

  for (int batch = 0; batch < n_mine; batch += kItemBatch) {
    int it = batch;
    const int it_end = min(batch + kItemBatch, n_mine);
    __syncthreads();                                     // previous batch fully consumed
    for (int i = tid; i < (it_end - it) * 2; i += T)
      reinterpret_cast<int4 *>(s_items)[i] =
          reinterpret_cast<const int4 *>(pd.items + (x0 + it + (i >> 1)))[i & 1];
    __syncthreads();
    Item cur = fetch_item(0);
    Item nxt = cur;
    if (it + 1 < it_end) nxt = fetch_item(1);
    int st = -1;                       // current stage of the current item
    int buf = 0;

    issue(cur, 0, -1, 0);
    // the items' ancestor ranges, fetched under the first Q tile (items with one range carry it)
    for (int i = tid; i < (it_end - it) * kRangeCache; i += T) {
      const int li = i / kRangeCache, r = i % kRangeCache;
      const int n_rng = s_items[li].n_ranges;
      if (n_rng > 1 && r < n_rng) s_ranges[li][r] = pd.ranges[s_items[li].range_off + r];
    }
    land_and_sync(0);

    while (true) {
      // which stage follows?  (K/V stage of this item, or the Q tile of the next item)  Its slot
      // was last read before the barrier that ended the previous stage.
      const bool last_stage = st + 1 >= n_stages(cur);
      const bool have_next = !last_stage || it + 1 < it_end;
      if (have_next) {
        __builtin_amdgcn_s_setprio(2);                     // requests leave before another wave's arithmetic
        if (!last_stage) issue(cur, it - batch, st + 1, buf ^ 1);
        else issue(nxt, it + 1 - batch, -1, buf ^ 1);
        __builtin_amdgcn_s_setprio(0);
      }
      const unsigned char *sl = ringp + buf * STAGEB;

      // The 32-row block owned by this wave rotates with the item index so that the long
      // (late-row) blocks of the resident workgroups do not pile up on one SIMD.
      const int slot = (wave + it) % NW;
      const int head = cur.head0 + slot % HPW;
      const int r0 = 32 * (slot / HPW);                     // first tile row of this wave
      const bool active = r0 < cur.n_rows;
      const int base = cur.anc_keys + cur.row0;             // virtual key of tile row 0 = its diagonal
      const int my_row = min(r0 + l32, cur.n_rows - 1);     // clamped: padded lanes repeat the last row
      const int my_limit = base + my_row;                   // last visible virtual key of this lane's row
      const int wave_last = base + min(r0 + 31, cur.n_rows - 1);
      const int wave_first_limit = base + r0;

      if (st < 0) {
        // Q stage: pull this wave's Q fragment (B operand; k-slot block j covers dims [16j + 8*half, +8))
        const unsigned char *qrow = sl + (32 * slot + l32) * ROWB;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          qf[j] = *reinterpret_cast<const bf16x8 *>(qrow + ((((2 * j) ^ kf_fh) | kf_lo) * 16));
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[c][i] = 0.f;
        m_run = kNegBig;
        l_run = 0.f;
        if (BIAS) {
          slope2 = sload_f32(pd.slopes + head) * kLog2e;
          pos_q = Pq[my_row];
        }
      } else {
#pragma unroll
        for (int sub = 0; sub < BK / 32; ++sub) {
          const int vk0 = st * BK + 32 * sub;
          if (!active || vk0 > wave_last) continue;           // block entirely above this wave's diagonal

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
              s[i] = fmaf(s[i], scale2, slope2 * (Ps[buf][32 * sub + 8 * (i / 4) + 4 * half + (i % 4)] - pos_q));
          }
          if (vk0 + 31 > wave_first_limit) {                 // diagonal block: some rows see only part of it
#pragma unroll
            for (int i = 0; i < 16; ++i)
              if (vk0 + 8 * (i / 4) + 4 * half + (i % 4) > my_limit) s[i] = -INFINITY;
          }
          float mx = fmaxf(s[0], s[1]);
#pragma unroll
          for (int i = 2; i < 16; ++i) mx = fmaxf(mx, s[i]);
          if (!BIAS) mx *= scale2;                           // scale2 > 0: max commutes with the scaling
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
          // V^T fragments through the LDS transpose read (4 keys x 16 dims per 16-lane group)
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

        if (last_stage) {
          // Epilogue of the item.  O^T sits in registers one query row per lane; it is transposed
          // through this wave's 32-row slice of the (now dead) K/V stage so that the global stores
          // are whole 16-byte chunks of contiguous rows.
          __syncthreads();                                   // every wave is done reading this stage
          if (active) {
            const float inv = 1.f / xhalf_sum(l_run);
            unsigned char *orow = ringp + buf * STAGEB + (32 * wave + l32) * ROWB + 8 * half;
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 w4;
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = static_cast<__bf16>(o[c][4 * q4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(orow + (((4 * c + q4) ^ kf_f) * 16)) = w4;
              }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int rows_here = min(32, cur.n_rows - r0);
            __bf16 *ob = O + ((uint64_t)(uint32_t)(cur.tok_start + cur.row0 + r0) * q_ts + (uint32_t)head * q_hs);
#pragma unroll
            for (int i = 0; i < 32 * CPR / 64; ++i) {
              const int id = lane + 64 * i, row = id / CPR, ch = id % CPR;
              if (row < rows_here)
                st16(ob + ((uint64_t)(uint32_t)row * q_ts + ch * 8),
                     *reinterpret_cast<const u32x4 *>(ringp + buf * STAGEB + (32 * wave + row) * ROWB +
                                                      ((ch ^ fK(row)) * 16)));
            }
          }
        }
      }

      if (!have_next) break;
      land_and_sync(buf ^ 1);
      buf ^= 1;
      if (!last_stage) {
        ++st;
      } else {
        ++it;
        cur = nxt;
        if (it + 1 < it_end) nxt = fetch_item(it + 1 - batch);
        st = -1;
      }
    }
  }
}

template <int D, int HPW, int NW>
static hipError_t launch_hpw(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  const dim3 grid(unsigned(plan->dev.n_wg));
  const __bf16 *Q = static_cast<const __bf16 *>(a.Q), *K = static_cast<const __bf16 *>(a.K),
               *V = static_cast<const __bf16 *>(a.V);
  __bf16 *O = static_cast<__bf16 *>(a.O);
  const uint32_t qts = uint32_t(a.q_tok_stride), qhs = uint32_t(a.q_head_stride), kts = uint32_t(a.kv_tok_stride),
                 khs = uint32_t(a.kv_head_stride);
  if (plan->has_slopes)
    hipLaunchKernelGGL((prefill_bf16_kernel<D, HPW, NW, true>), grid, dim3(64 * NW), 0, s, plan->dev, Q, K, V, O,
                       qts, qhs, kts, khs, a.scale);
  else
    hipLaunchKernelGGL((prefill_bf16_kernel<D, HPW, NW, false>), grid, dim3(64 * NW), 0, s, plan->dev, Q, K, V, O,
                       qts, qhs, kts, khs, a.scale);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  switch (plan->heads_per_wg) {
    case 4: return launch_hpw<D, 4, 4>(plan, a, s);
    case 2: return launch_hpw<D, 2, 2>(plan, a, s);
    default: return launch_hpw<D, 1, 2>(plan, a, s);
  }
}

hipError_t launch_prefill_bf16(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  return plan->head_dim == 128 ? launch_d<128>(plan, a, s) : launch_d<64>(plan, a, s);
}

}  // namespace sp
