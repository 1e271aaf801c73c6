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
// 4/HPW blocks of 32 tokens.  K/V tiles of 64 keys are staged once per workgroup in LDS (padded
// rows, double buffered) and reused by all four waves.
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

constexpr int kBK = 64;            // keys per LDS stage
typedef bf16x4 __attribute__((address_space(3))) lds_bf16x4;

template <int D, int HPW, bool BIAS>
__global__ __launch_bounds__(256, 2) void prefill_bf16_kernel(PlanDev pd, const __bf16 *__restrict__ Q,
                                                           const __bf16 *__restrict__ K,
                                                           const __bf16 *__restrict__ V, __bf16 *__restrict__ O,
                                                           int64_t q_ts, int64_t q_hs, int64_t kv_ts,
                                                           int64_t kv_hs, float scale, int items_per_xcd) {
  constexpr int LDK = D + 8;               // padded LDS row: consecutive rows shift by 16 bytes
  constexpr int RB = 4 / HPW;              // 32-token blocks per workgroup
  constexpr int CPR = D / 8;               // 16-byte chunks per K/V row
  constexpr int LOADS = kBK * CPR / 256;   // chunks per thread per tile
  constexpr int NJ = D / 16;               // MFMAs along head_dim for S
  constexpr int NC = D / 32;               // 32-wide output blocks of O^T

  __shared__ __attribute__((aligned(16))) __bf16 Ks[2][kBK][LDK];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[2][kBK][LDK];
  __shared__ float Ps[2][kBK];
  __shared__ int32_t rg_start[kMaxRanges], rg_cum[kMaxRanges + 1];

  // Workgroup ids are dealt round-robin over the 8 XCDs; give every XCD a contiguous slice of the
  // work list so that workgroups sharing K/V rows (same prompt and KV head) share one L2.
  const int item = (blockIdx.x % 8) * items_per_xcd + blockIdx.x / 8;
  if (blockIdx.x / 8 >= items_per_xcd || item >= pd.n_items) return;
  const WorkItem it = pd.items[item];
  const RowGroup rg = pd.groups[it.group];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int G = pd.n_q_heads / pd.n_kv_heads;
  const int head = it.head0 + (wave % HPW);
  const int g = it.head0 / G;
  const int r0 = it.row0 + 32 * (wave / HPW);            // first row of this wave inside the group
  const bool active = r0 < rg.len;
  const int A = rg.anc_keys;
  const int tile_end = min(it.row0 + 32 * RB, rg.len);   // rows [row0, tile_end)
  const int n_keys = A + tile_end;                       // virtual keys the workgroup needs
  const int n_kt = (n_keys + kBK - 1) / kBK;
  const int my_row = min(r0 + l32, rg.len - 1);          // clamped: padded lanes repeat the last row
  const int my_limit = A + my_row;                       // last visible virtual key of this lane's row
  const int wave_last = A + min(r0 + 31, rg.len - 1);
  const int wave_first_limit = A + r0;

  if (tid == 0) {
    int cum = 0;
    for (int r = 0; r < rg.n_ranges; ++r) {
      const KeyRange kr = pd.ranges[rg.range_off + r];
      rg_start[r] = kr.tok_start;
      rg_cum[r] = cum;
      cum += kr.len;
    }
    rg_cum[rg.n_ranges] = cum;
  }
  __syncthreads();
  const int nr = rg.n_ranges;
  const int last_vk = A + rg.len - 1;
  auto map_tok = [&](int vk) -> int {
    vk = min(vk, last_vk);                 // rows past the end re-read the last key (masked later)
    if (vk >= A) return rg.tok_start + (vk - A);
    int i = 0;
    while (i + 1 < nr && rg_cum[i + 1] <= vk) ++i;
    return rg_start[i] + (vk - rg_cum[i]);
  };

  // Q fragment of this lane's row: B operand, k-slot block j covers dims [16j + 8*half, +8)
  bf16x8 qf[NJ];
  {
    const __bf16 *qp = Q + (int64_t)(rg.tok_start + my_row) * q_ts + (int64_t)head * q_hs + 8 * half;
#pragma unroll
    for (int j = 0; j < NJ; ++j) qf[j] = *reinterpret_cast<const bf16x8 *>(qp + 16 * j);
  }
  const int tr_row = (lane & 15) >> 2;                     // transpose-read source: key row within 4
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);   // and first of 4 dims within 32
  const float scale2 = scale * kLog2e;
  float slope2 = 0.f, pos_q = 0.f;
  if (BIAS) {
    slope2 = pd.slopes[head] * kLog2e;
    pos_q = pd.tok_pos[rg.tok_start + my_row];
  }

  const __bf16 *Kg = K + (int64_t)g * kv_hs + (tid % CPR) * 8;
  const __bf16 *Vg = V + (int64_t)g * kv_hs + (tid % CPR) * 8;
  u32x4 kreg[LOADS], vreg[LOADS];
  float preg = 0.f;
  auto gload = [&](int kt) {
#pragma unroll
    for (int m = 0; m < LOADS; ++m) {
      const int row = tid / CPR + m * (256 / CPR);
      const int64_t tok = map_tok(kt * kBK + row);
      kreg[m] = ld16(Kg + tok * kv_ts);
      vreg[m] = ld16(Vg + tok * kv_ts);
    }
    if (BIAS && tid < kBK) preg = pd.tok_pos[map_tok(kt * kBK + tid)];
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int m = 0; m < LOADS; ++m) {
      const int row = tid / CPR + m * (256 / CPR);
      st16(&Ks[buf][row][(tid % CPR) * 8], kreg[m]);
      st16(&Vs[buf][row][(tid % CPR) * 8], vreg[m]);
    }
    if (BIAS && tid < kBK) Ps[buf][tid] = preg;
  };

  f32x16 o[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[c][i] = 0.f;
  float m_run = kNegBig, l_run = 0.f;     // running maximum (log2 units) and this half's partial sum

  gload(0);
  sstore(0);
  __syncthreads();

  for (int kt = 0; kt < n_kt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < n_kt) gload(kt + 1);

#pragma unroll
    for (int sub = 0; sub < kBK / 32; ++sub) {
      const int vk0 = kt * kBK + 32 * sub;
      if (!active || vk0 > wave_last) continue;         // block entirely above this wave's diagonal

      f32x16 s;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&Ks[buf][32 * sub + l32][16 * j + 8 * half]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[j], s, 0, 0, 0);
      }

      float t[16];
      const bool diag = vk0 + 31 > wave_first_limit;    // some row of the wave sees only part of the block
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = 8 * (i / 4) + 4 * half + (i % 4);
        float x = s[i] * scale2;
        if (BIAS) x -= slope2 * (pos_q - Ps[buf][32 * sub + key]);
        if (diag && vk0 + key > my_limit) x = -INFINITY;
        t[i] = x;
      }
      float mx = t[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, t[i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      // The reference maximum is allowed to lag by up to 8 (factor 256 in p), which fp32 sums and
      // bf16 P absorb; the 64+ accumulator registers are rescaled only when some row exceeds that.
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
      float p[16];
      float ls = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        p[i] = fast_exp2(t[i] - m_run);
        ls += p[i];
      }
      l_run += ls;
      bf16x8 pb[2];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pb[0][i] = static_cast<__bf16>(p[i]);
        pb[1][i] = static_cast<__bf16>(p[8 + i]);
      }
#pragma unroll
      for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          // V^T fragment through the LDS transpose read: a 16-lane group hands in a 4-key x 16-dim
          // block (lane s: key s/4, dims 4*(s%4)..+3) and lane i receives dim i of the 4 keys.
          const __bf16 *vp = &Vs[buf][32 * sub + 16 * mm + 4 * half + tr_row][32 * c + tr_col];
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * LDK));
          const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[mm], o[c], 0, 0, 0);
        }
      }
    }

    if (kt + 1 < n_kt) sstore(buf ^ 1);
    __syncthreads();
  }

  if (active && r0 + l32 < rg.len) {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.f / l_tot;
    __bf16 *op = O + (int64_t)(rg.tok_start + my_row) * q_ts + (int64_t)head * q_hs;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = static_cast<__bf16>(o[c][4 * q4 + e] * inv);
        *reinterpret_cast<bf16x4 *>(op + 32 * c + 8 * q4 + 4 * half) = w;
      }
  }
}

template <int D, int HPW>
static hipError_t launch_hpw(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  const int n_items = static_cast<int>(plan->items.size());
  const int per_xcd = (n_items + 7) / 8;
  const dim3 grid(unsigned(per_xcd) * 8);
  const __bf16 *Q = static_cast<const __bf16 *>(a.Q), *K = static_cast<const __bf16 *>(a.K),
               *V = static_cast<const __bf16 *>(a.V);
  __bf16 *O = static_cast<__bf16 *>(a.O);
  if (plan->has_slopes)
    hipLaunchKernelGGL((prefill_bf16_kernel<D, HPW, true>), grid, dim3(256), 0, s, plan->dev, Q, K, V, O,
                       a.q_tok_stride, a.q_head_stride, a.kv_tok_stride, a.kv_head_stride, a.scale, per_xcd);
  else
    hipLaunchKernelGGL((prefill_bf16_kernel<D, HPW, false>), grid, dim3(256), 0, s, plan->dev, Q, K, V, O,
                       a.q_tok_stride, a.q_head_stride, a.kv_tok_stride, a.kv_head_stride, a.scale, per_xcd);
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
