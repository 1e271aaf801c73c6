// a4: single-token decode attention over the joined cache (Sec. 3.2.3; Alg. 3 generation loop).
//
// The kept paths' caches are "simply concatenated" in the paper; here nothing is copied: each
// workgroup resolves the concatenation [shared; kept path 0; ...; kept path k-1; response; new]
// through the plan's range tables and the device-resident kept table, and streams K and V rows
// straight from the packed prefill cache.  HBM-bound: every K/V byte is read once per step.
//
// Workgroup = (prompt, KV head, chunk of GC query heads), 256 threads.  A key row of head_dim
// elements is covered by LPK lanes with one 16-byte load each, so 256/LPK keys are in flight
// per load instruction; each such lane group keeps its own online-softmax state and the groups
// are merged through LDS in a fixed order at the end.
#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

constexpr int kDecThreads = 256;
constexpr int kDecMaxRanges = 128;
constexpr int kDecUnroll = 4;

struct DecodeDev {
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

template <typename T, int D, int GC>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(PlanDev pd, DecodeDev a) {
  constexpr int EV = Elem<T>::kVec;       // elements per 16-byte lane load
  constexpr int LPK = D / EV;             // lanes per key row
  constexpr int KPW = kDecThreads / LPK;  // key rows per load instruction of the workgroup
  const int Hq = pd.n_q_heads, Hkv = pd.n_kv_heads, G = Hq / Hkv;
  const int b = blockIdx.x / Hkv, g = blockIdx.x % Hkv;
  const int head0 = g * G + blockIdx.y * GC;
  const int tid = threadIdx.x, kg = tid / LPK, sub = tid % LPK;
  const bool bias = pd.slopes != nullptr;

  __shared__ int32_t r_start[kDecMaxRanges], r_cum[kDecMaxRanges + 1], r_len[kDecMaxRanges];
  __shared__ int32_t s_cnt[kDecMaxRanges], s_keys[kDecMaxRanges];
  __shared__ int32_t s_nr;
  __shared__ float s_m[KPW][GC], s_l[KPW][GC];
  __shared__ float s_acc[KPW][GC][D];

  // query chunk of this lane for each head, pre-scaled so that scores are in log2 units (requested
  // first: these loads run under the table walk below)
  float qf[GC][EV];
  float slope2[GC];
  const float pos_q = (bias && a.new_pos) ? a.new_pos[b] : 0.f;
#pragma unroll
  for (int c = 0; c < GC; ++c) {
    const T *qp = static_cast<const T *>(a.q_new) + ((int64_t)b * Hq + head0 + c) * D + sub * EV;
    Elem<T>::unpack(ld16(qp), qf[c]);
#pragma unroll
    for (int e = 0; e < EV; ++e) qf[c][e] *= a.scale * kLog2e;
    slope2[c] = bias ? pd.slopes[head0 + c] * kLog2e : 0.f;
  }

  // The joined cache [shared ; kept path 0 ; ... ; kept path k-1] as a list of token ranges with
  // running key counts.  Source 0 is the shared part, source j >= 1 the (j-1)-th kept path; one
  // thread per source follows the tables (kept -> path slot descriptor, which carries the first range), so the dependent loads of
  // all sources run side by side; two small prefix sums through LDS put the ranges in order.
  {
    const int n_src = min(a.k + 1, kDecMaxRanges);
    RangeDesc src{0, 0, 0, 0};
    if (tid == 0) {
      src = pd.shared_desc[b];
    } else if (tid < n_src) {
      const int p0 = pd.path_off[b], np = pd.path_off[b + 1] - p0;
      const int kp = a.kept[(int64_t)b * a.k + (tid - 1)];
      if (kp >= 0 && kp < np) src = pd.path_desc[p0 + kp];
    }
    const int beg = src.beg, end = src.end;
    if (tid < n_src) s_cnt[tid] = end - beg;
    __syncthreads();
    int off = 0, keys = 0;
    if (tid < n_src) {
      for (int i = 0; i < tid; ++i) off += s_cnt[i];
      for (int r = beg; r < end; ++r) {
        const int at = off + (r - beg);
        if (at < kDecMaxRanges) {
          const KeyRange kr = r == beg ? KeyRange{src.tok_start, src.len} : pd.dec_ranges[r];
          r_start[at] = kr.tok_start;
          r_len[at] = kr.len;
          keys += kr.len;
        }
      }
      s_keys[tid] = keys;
    }
    __syncthreads();
    if (tid < n_src) {
      int cum = 0;
      for (int i = 0; i < tid; ++i) cum += s_keys[i];
      for (int r = beg; r < end; ++r) {
        const int at = off + (r - beg);
        if (at < kDecMaxRanges) {
          r_cum[at] = cum;
          cum += r_len[at];
        }
      }
      if (tid == n_src - 1) {
        const int n = min(off + (end - beg), kDecMaxRanges);
        r_cum[n] = cum;
        s_nr = n;
      }
    }
  }
  __syncthreads();
  const int nr = s_nr;
  const int n_pref = r_cum[nr];
  const int len_b = (a.resp_len ? a.resp_len[b] : 0) + a.resp_len_add;
  const int len_r = len_b < a.resp_capacity ? (len_b < 0 ? 0 : len_b) : a.resp_capacity;
  const int n_total = n_pref + len_r + 1;

  const T *Kp = static_cast<const T *>(a.Kp) + (int64_t)g * a.kv_head_stride + sub * EV;
  const T *Vp = static_cast<const T *>(a.Vp) + (int64_t)g * a.kv_head_stride + sub * EV;
  const int64_t resp_row = (int64_t)Hkv * D;
  const T *Kr = static_cast<const T *>(a.Kr) + ((int64_t)b * a.resp_capacity * Hkv + g) * D + sub * EV;
  const T *Vr = static_cast<const T *>(a.Vr) + ((int64_t)b * a.resp_capacity * Hkv + g) * D + sub * EV;
  const T *kn = static_cast<const T *>(a.k_new) + ((int64_t)b * Hkv + g) * D + sub * EV;
  const T *vn = static_cast<const T *>(a.v_new) + ((int64_t)b * Hkv + g) * D + sub * EV;

  // append the new token's K/V (and position) to the response cache: one workgroup per (b, g)
  if (blockIdx.y == 0 && len_b >= 0 && len_b < a.resp_capacity) {
    T *dk = static_cast<T *>(a.Kr) + (((int64_t)b * a.resp_capacity + len_b) * Hkv + g) * D;
    T *dv = static_cast<T *>(a.Vr) + (((int64_t)b * a.resp_capacity + len_b) * Hkv + g) * D;
    if (tid < LPK) st16(dk + sub * EV, ld16(kn));
    else if (tid < 2 * LPK) st16(dv + sub * EV, ld16(vn));
    if (g == 0 && tid == 0 && a.pos_resp && a.new_pos) a.pos_resp[(int64_t)b * a.resp_capacity + len_b] = a.new_pos[b];
  }

  float m[GC], l[GC], acc[GC][EV];
#pragma unroll
  for (int c = 0; c < GC; ++c) {
    m[c] = kNegBig; l[c] = 0.f;
#pragma unroll
    for (int e = 0; e < EV; ++e) acc[c][e] = 0.f;
  }

  // One batch = kDecUnroll keys per lane group.  Batches are software-pipelined: the loads of the
  // next batch are issued before the arithmetic of the current one (two register sets).
  struct Batch {
    u32x4 kraw[kDecUnroll], vraw[kDecUnroll];
    float pk[kDecUnroll];
    bool ok[kDecUnroll];
  };
  auto load_batch = [&](int vk0, Batch &bt) {
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      const int vk = vk0 + u * KPW;
      bt.ok[u] = vk < n_total;
      const T *kptr = kn, *vptr = vn;        // also the in-bounds stand-in for lanes past the end
      bt.pk[u] = pos_q;
      if (vk < n_pref) {
        int i = 0;
        while (i + 1 < nr && r_cum[i + 1] <= vk) ++i;
        const int64_t tok = r_start[i] + (vk - r_cum[i]);
        kptr = Kp + tok * a.kv_tok_stride;
        vptr = Vp + tok * a.kv_tok_stride;
        if (bias) bt.pk[u] = pd.tok_pos[tok];
      } else if (vk < n_pref + len_r) {
        const int64_t row = vk - n_pref;
        kptr = Kr + row * resp_row;
        vptr = Vr + row * resp_row;
        if (bias) bt.pk[u] = a.pos_resp[(int64_t)b * a.resp_capacity + row];
      }
      bt.kraw[u] = ld16(kptr);
      bt.vraw[u] = ld16(vptr);
    }
  };
  auto compute_batch = [&](const Batch &bt) {
    float t[kDecUnroll][GC];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      float kf[EV];
      Elem<T>::unpack(bt.kraw[u], kf);
#pragma unroll
      for (int c = 0; c < GC; ++c) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EV; ++e) d = fmaf(qf[c][e], kf[e], d);
#pragma unroll
        for (int off = LPK / 2; off >= 1; off >>= 1) d += __shfl_xor(d, off);
        // distance penalty -slope * (pos_q - pos_k), in log2 units
        t[u][c] = bt.ok[u] ? d - slope2[c] * (pos_q - bt.pk[u]) : -INFINITY;
      }
    }
#pragma unroll
    for (int c = 0; c < GC; ++c) {
      float mx = t[0][c];
#pragma unroll
      for (int u = 1; u < kDecUnroll; ++u) mx = fmaxf(mx, t[u][c]);
      const float m_new = fmaxf(m[c], mx);
      const float alpha = fast_exp2(m[c] - m_new);
      m[c] = m_new;
      l[c] *= alpha;
#pragma unroll
      for (int e = 0; e < EV; ++e) acc[c][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      float vf[EV];
      Elem<T>::unpack(bt.vraw[u], vf);
#pragma unroll
      for (int c = 0; c < GC; ++c) {
        const float p = fast_exp2(t[u][c] - m[c]);
        l[c] += p;
#pragma unroll
        for (int e = 0; e < EV; ++e) acc[c][e] = fmaf(p, vf[e], acc[c][e]);
      }
    }
  };
  {
    constexpr int STEP = KPW * kDecUnroll;
    Batch b0, b1;
    int vk0 = kg;
    if (vk0 < n_total) load_batch(vk0, b0);
    while (vk0 < n_total) {
      if (vk0 + STEP < n_total) load_batch(vk0 + STEP, b1);
      compute_batch(b0);
      vk0 += STEP;
      if (vk0 >= n_total) break;
      if (vk0 + STEP < n_total) load_batch(vk0 + STEP, b0);
      compute_batch(b1);
      vk0 += STEP;
    }
  }

  // merge the KPW lane groups in a fixed order
#pragma unroll
  for (int c = 0; c < GC; ++c) {
    if (sub == 0) { s_m[kg][c] = m[c]; s_l[kg][c] = l[c]; }
#pragma unroll
    for (int e = 0; e < EV; ++e) s_acc[kg][c][sub * EV + e] = acc[c][e];
  }
  __syncthreads();
  for (int idx = tid; idx < GC * D; idx += kDecThreads) {
    const int c = idx / D, e = idx % D;
    float M = s_m[0][c];
    for (int j = 1; j < KPW; ++j) M = fmaxf(M, s_m[j][c]);
    float num = 0.f, den = 0.f;
    for (int j = 0; j < KPW; ++j) {
      const float w = fast_exp2(s_m[j][c] - M);
      num = fmaf(w, s_acc[j][c][e], num);
      den = fmaf(w, s_l[j][c], den);
    }
    T *o = static_cast<T *>(a.o_out) + ((int64_t)b * Hq + head0 + c) * D + e;
    Elem<T>::store1(o, num / den);
  }
}

template <typename T, int D>
static hipError_t launch_decode_t(const sp_plan *plan, const DecodeDev &d, hipStream_t s) {
  const int G = plan->n_q_heads / plan->n_kv_heads;
  const int gc = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  const dim3 grid(unsigned(plan->n_prompts) * plan->n_kv_heads, unsigned(G / gc));
  if (gc == 4) hipLaunchKernelGGL((decode_kernel<T, D, 4>), grid, dim3(kDecThreads), 0, s, plan->dev, d);
  else if (gc == 2) hipLaunchKernelGGL((decode_kernel<T, D, 2>), grid, dim3(kDecThreads), 0, s, plan->dev, d);
  else hipLaunchKernelGGL((decode_kernel<T, D, 1>), grid, dim3(kDecThreads), 0, s, plan->dev, d);
  return hipGetLastError();
}

hipError_t launch_decode(const sp_plan *plan, const DecodeArgs &a, hipStream_t s) {
  DecodeDev d{a.kept, a.k, a.Kp, a.Vp, a.kv_tok_stride, a.kv_head_stride, a.Kr, a.Vr, a.pos_resp, a.resp_capacity,
              a.resp_len, a.resp_len_add, a.new_pos, a.q_new, a.k_new, a.v_new, a.o_out, a.scale};
  if (plan->dtype == SP_BF16)
    return plan->head_dim == 128 ? launch_decode_t<__bf16, 128>(plan, d, s) : launch_decode_t<__bf16, 64>(plan, d, s);
  return plan->head_dim == 128 ? launch_decode_t<float, 128>(plan, d, s) : launch_decode_t<float, 64>(plan, d, s);
}

}  // namespace sp
