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
// streams one unbroken sequence of LDS stages through a double buffer -- for every item first its
// Q tile (32*NW rows = one stage), then its K/V tiles of 16*NW keys -- so the global loads of the
// next stage (also across item boundaries) are in flight behind the current stage's math and no
// item pays a cold start.  O^T tiles leave through LDS as whole 16-byte chunks of contiguous rows.
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
#ifndef SP_PADK
#define SP_PADK 8
#endif
#ifndef SP_PADV
#define SP_PADV 8
#endif
typedef bf16x4 __attribute__((address_space(3))) lds_bf16x4;

// max / sum partner exchange between lane L and lane L^32 (v_permlane32_swap)
__device__ __forceinline__ float xhalf_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
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
  constexpr int LDK = D + SP_PADK;         // padded LDS rows of the K half (16-byte row reads)
  constexpr int LDV = D + SP_PADV;         // and of the V half (transpose reads of 4 keys x 16 dims)
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int RPP = T / CPR;             // rows covered by one pass of all threads
  constexpr int LOADS = BK / RPP;          // passes per half stage
  constexpr int NJ = D / 16;               // MFMAs along head_dim for S
  constexpr int NC = D / 32;               // 32-wide output blocks of O^T
  static_assert(NW % HPW == 0 && BK % 32 == 0 || BK == 32, "tile shape");

  // A stage is BK K rows + BK V rows; a Q tile (2*BK rows) uses the K half for rows 0..BK and the
  // V half for rows BK..2BK.
  __shared__ __attribute__((aligned(16))) __bf16 stK[2][BK][LDK];
  __shared__ __attribute__((aligned(16))) __bf16 stV[2][BK][LDV];
  // row r of the 2*BK-row view of a stage
  auto srow = [&](int buf, int r) -> __bf16 * { return r < BK ? &stK[buf][r][0] : &stV[buf][r - BK][0]; };
  __shared__ float Ps[2][BK];
  __shared__ __attribute__((aligned(16))) WorkItem s_items[kItemBatch];

  // Workgroup ids are dealt round-robin over the 8 XCDs (id % 8).  The host has given every XCD a
  // contiguous range of the work list and handed its items out in order to that XCD's workgroup
  // slots, so the workgroups of an XCD work on a moving window of consecutive items and share
  // their K/V rows through that XCD's L2.  Slot s = xcd * (n_wg / 8) + id / 8 owns items [x0, x1).
  const int wg_slot = (blockIdx.x % 8) * (pd.n_wg / 8) + blockIdx.x / 8;
  const int x0 = pd.wg_begin[wg_slot], x1 = pd.wg_begin[wg_slot + 1];
  const int n_mine = x1 - x0;
  if (n_mine <= 0) return;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int tr_row = (lane & 15) >> 2;                          // transpose-read source: key row within 4
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);   // and first of 4 dims within 32
  const float scale2 = scale * kLog2e;
  const int lrow = tid / CPR, lcol = (tid % CPR) * 8;           // this thread's row / column in a load pass

  u32x4 areg[LOADS], breg[LOADS];
  float preg = 0.f;

  // a work item as the loop keeps it (all fields wave-uniform)
  struct Item {
    int tok_start, row0, n_rows, anc_keys, range_off, n_ranges, head0, kv_head, r0_start;
  };
  // Byte offsets of this thread inside a load pass; a pass covers RPP consecutive rows, so for runs
  // of consecutive tokens everything else about an address is wave-uniform (scalar base + this).
  const uint32_t kv_lane_off = ((uint32_t)lrow * kv_ts + lcol) * 2;
  const uint32_t q_lane_off = ((uint32_t)lrow * q_ts + lcol) * 2;
  const char *Qb = reinterpret_cast<const char *>(Q), *Kb = reinterpret_cast<const char *>(K),
             *Vb = reinterpret_cast<const char *>(V);

  // virtual key -> packed token for item w
  auto map_tok = [&](const Item &w, int vk) -> int {
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
  // issue the global loads of stage st of item w (st = -1: the Q tile)
  auto gload = [&](const Item &w, int st) {
    if (st < 0) {
      if (w.n_rows == 32 * NW / HPW) {
        // full tile: row r = lrow + m*RPP sits in 32-row slot (m*RPP)/32 at (m*RPP)%32 + lrow
        const uint64_t t0 = (uint32_t)(w.tok_start + w.row0);
#pragma unroll
        for (int m = 0; m < LOADS; ++m) {
          const int ra = m * RPP, rb = BK + m * RPP;              // compile-time row bases of the two halves
          const int sa = ra >> 5, sb = rb >> 5;
          const uint64_t oa = ((t0 + 32 * (sa / HPW) + (ra & 31)) * q_ts + (uint64_t)(uint32_t)(w.head0 + sa % HPW) * q_hs) * 2;
          const uint64_t ob = ((t0 + 32 * (sb / HPW) + (rb & 31)) * q_ts + (uint64_t)(uint32_t)(w.head0 + sb % HPW) * q_hs) * 2;
          areg[m] = ld16(Qb + oa + q_lane_off);
          breg[m] = ld16(Qb + ob + q_lane_off);
        }
        return;
      }
#pragma unroll
      for (int m = 0; m < LOADS; ++m) {
        const int r = lrow + m * RPP;                           // Q-tile rows r and BK + r
        const int s0 = r >> 5, s1 = (BK + r) >> 5;              // their 32-row slots
        const int t0 = w.tok_start + w.row0 + min(32 * (s0 / HPW) + (r & 31), w.n_rows - 1);
        const int t1 = w.tok_start + w.row0 + min(32 * (s1 / HPW) + ((BK + r) & 31), w.n_rows - 1);
        areg[m] = ld16(Q + ((uint64_t)(uint32_t)t0 * q_ts + (uint32_t)(w.head0 + s0 % HPW) * q_hs + lcol));
        breg[m] = ld16(Q + ((uint64_t)(uint32_t)t1 * q_ts + (uint32_t)(w.head0 + s1 % HPW) * q_hs + lcol));
      }
    } else {
      // A stage whose BK keys are consecutive tokens (inside the own run and not past its end, or
      // inside a single ancestor range) needs no per-lane address arithmetic.
      const int vk0 = st * BK;
      int tok0 = -1;
      if (vk0 >= w.anc_keys) {
        if (vk0 + BK <= w.anc_keys + w.row0 + w.n_rows) tok0 = w.tok_start + (vk0 - w.anc_keys);
      } else if (w.n_ranges == 1 && vk0 + BK <= w.anc_keys) {
        tok0 = w.r0_start + vk0;
      }
      if (tok0 >= 0) {
        const uint64_t o0 = ((uint64_t)(uint32_t)tok0 * kv_ts + (uint64_t)(uint32_t)w.kv_head * kv_hs) * 2;
#pragma unroll
        for (int m = 0; m < LOADS; ++m) {
          const uint64_t o = o0 + (uint64_t)(m * RPP) * kv_ts * 2;
          areg[m] = ld16(Kb + o + kv_lane_off);
          breg[m] = ld16(Vb + o + kv_lane_off);
        }
        if (BIAS && tid < BK) preg = pd.tok_pos[tok0 + tid];
        return;
      }
      const uint32_t hoff = (uint32_t)w.kv_head * kv_hs + lcol;
#pragma unroll
      for (int m = 0; m < LOADS; ++m) {
        const uint64_t off = (uint64_t)(uint32_t)map_tok(w, st * BK + lrow + m * RPP) * kv_ts + hoff;
        areg[m] = ld16(K + off);
        breg[m] = ld16(V + off);
      }
      if (BIAS && tid < BK) preg = pd.tok_pos[map_tok(w, st * BK + tid)];
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int m = 0; m < LOADS; ++m) {
      st16(&stK[buf][lrow + m * RPP][lcol], areg[m]);
      st16(&stV[buf][lrow + m * RPP][lcol], breg[m]);
    }
    if (BIAS && tid < BK) Ps[buf][tid] = preg;
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
  float m_run = kNegBig, l_run = 0.f, slope2 = 0.f, pos_q = 0.f;

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

    gload(cur, -1);
    sstore(0);
    __syncthreads();

    while (true) {
      // which stage follows?  (K/V stage of this item, or the Q tile of the next item)
      const bool last_stage = st + 1 >= n_stages(cur);
      const bool have_next = !last_stage || it + 1 < it_end;
      if (have_next) {
        if (!last_stage) gload(cur, st + 1);
        else gload(nxt, -1);
      }

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
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          qf[j] = *reinterpret_cast<const bf16x8 *>(srow(buf, 32 * slot + l32) + 16 * j + 8 * half);
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[c][i] = 0.f;
        m_run = kNegBig;
        l_run = 0.f;
        if (BIAS) {
          slope2 = pd.slopes[head] * kLog2e;
          pos_q = pd.tok_pos[cur.tok_start + cur.row0 + my_row];
        }
      } else {
#pragma unroll
        for (int sub = 0; sub < BK / 32; ++sub) {
          const int vk0 = st * BK + 32 * sub;
          if (!active || vk0 > wave_last) continue;           // block entirely above this wave's diagonal

          f32x16 s;
#pragma unroll
          for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&stK[buf][32 * sub + l32][16 * j + 8 * half]);
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
#pragma unroll
          for (int c = 0; c < NC; ++c) {
#pragma unroll
            for (int mm = 0; mm < 2; ++mm) {
              // V^T fragment through the LDS transpose read: a 16-lane group hands in a 4-key x 16-dim
              // block (lane s: key s/4, dims 4*(s%4)..+3) and lane i receives dim i of the 4 keys.
              const __bf16 *vp = &stV[buf][32 * sub + 16 * mm + 4 * half + tr_row][32 * c + tr_col];
              const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
              const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * LDV));
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
            __bf16 *orow = srow(buf, 32 * wave + l32) + 4 * half;
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 w4;
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = static_cast<__bf16>(o[c][4 * q4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(orow + 32 * c + 8 * q4) = w4;
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
                     *reinterpret_cast<const u32x4 *>(srow(buf, 32 * wave + row) + ch * 8));
            }
          }
        }
      }

      if (!have_next) break;
      sstore(buf ^ 1);
      __syncthreads();
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
