// a1 (fp32 storage): ForkJoin prefill attention over the prompt DAG (Sec. 3.2, 3.2.1; App. B.3)
// in plain fp32 vector arithmetic.  This is the precision path (tolerance 1e-4); the bf16 path
// uses the matrix cores.  One wave handles one (token, query head) row: the lanes split the head
// dimension, the row's visible keys (ancestor ranges root-to-leaf, then its own run causally)
// are visited in order with an online softmax, four keys per step.
#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

template <int D>
__global__ __launch_bounds__(256) void prefill_f32_kernel(PlanDev pd, const float *__restrict__ Q,
                                                          const float *__restrict__ K,
                                                          const float *__restrict__ V, float *__restrict__ O,
                                                          int64_t q_ts, int64_t q_hs, int64_t kv_ts, int64_t kv_hs,
                                                          float scale) {
  // 16 lanes cover one key row with 16-byte loads (D = 64: 4 floats per lane; D = 128: 2 loads)
  constexpr int EPL = D / 16;            // elements per lane
  const int Hq = pd.n_q_heads, G = Hq / pd.n_kv_heads;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t row_id = (int64_t)blockIdx.x * 4 + wave;
  if (row_id >= (int64_t)pd.n_tokens * Hq) return;
  const int tok = int(row_id / Hq), h = int(row_id % Hq), g = h / G;
  const int grp = pd.tok_group[tok];
  if (grp < 0) return;
  const RowGroup rg = pd.groups[grp];
  const int n_vis = rg.anc_keys + (tok - rg.tok_start) + 1;
  const int quad = lane >> 4, sub = lane & 15;       // 4 keys in flight per wave
  const bool bias = pd.slopes != nullptr;
  const float slope2 = bias ? pd.slopes[h] * kLog2e : 0.f;
  const float pos_q = bias ? pd.tok_pos[tok] : 0.f;

  float qf[EPL];
  {
    const float *qp = Q + (int64_t)tok * q_ts + (int64_t)h * q_hs + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] = qp[e] * (scale * kLog2e);
  }
  float m = kNegBig, l = 0.f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  for (int vk0 = 0; vk0 < n_vis; vk0 += 4) {
    const int vk = vk0 + quad;
    const bool ok = vk < n_vis;
    // virtual key index -> packed token: walk the ancestor ranges, else own run
    int ktok = rg.tok_start + (vk - rg.anc_keys);
    if (!ok) ktok = tok;
    else if (vk < rg.anc_keys) {
      int rem = vk;
      for (int r = 0; r < rg.n_ranges; ++r) {
        const KeyRange kr = pd.ranges[rg.range_off + r];
        if (rem < kr.len) { ktok = kr.tok_start + rem; break; }
        rem -= kr.len;
      }
    }
    const float *kp = K + (int64_t)ktok * kv_ts + (int64_t)g * kv_hs + sub * EPL;
    const float *vp = V + (int64_t)ktok * kv_ts + (int64_t)g * kv_hs + sub * EPL;
    float d = 0.f, vf[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) { d = fmaf(qf[e], kp[e], d); vf[e] = vp[e]; }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) d += __shfl_xor(d, off);
    float t = -INFINITY;
    if (ok) t = bias ? d - slope2 * (pos_q - pd.tok_pos[ktok]) : d;
    // maximum over the 4 keys of this step (lanes 16 and 32 apart)
    float mx = fmaxf(t, __shfl_xor(t, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float alpha = fast_exp2(m - m_new);
    const float p = fast_exp2(t - m_new);
    m = m_new;
    l = l * alpha + p;                 // per-quad partial sums, combined at the end
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e] * alpha);
  }
  // combine the four quads (all share the same running maximum m)
  l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
#pragma unroll
  for (int e = 0; e < EPL; ++e) { acc[e] += __shfl_xor(acc[e], 16); acc[e] += __shfl_xor(acc[e], 32); }
  if (quad == 0) {
    float *op = O + (int64_t)tok * q_ts + (int64_t)h * q_hs + sub * EPL;
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < EPL; ++e) op[e] = acc[e] * inv;
  }
}

hipError_t launch_prefill_f32(const sp_plan *plan, const PrefillArgs &a, hipStream_t s) {
  const int64_t rows = (int64_t)plan->n_tokens * plan->n_q_heads;
  const dim3 grid(unsigned((rows + 3) / 4));
  if (plan->head_dim == 128)
    hipLaunchKernelGGL(prefill_f32_kernel<128>, grid, dim3(256), 0, s, plan->dev, static_cast<const float *>(a.Q),
                       static_cast<const float *>(a.K), static_cast<const float *>(a.V), static_cast<float *>(a.O),
                       a.q_tok_stride, a.q_head_stride, a.kv_tok_stride, a.kv_head_stride, a.scale);
  else
    hipLaunchKernelGGL(prefill_f32_kernel<64>, grid, dim3(256), 0, s, plan->dev, static_cast<const float *>(a.Q),
                       static_cast<const float *>(a.K), static_cast<const float *>(a.V), static_cast<float *>(a.O),
                       a.q_tok_stride, a.q_head_stride, a.kv_tok_stride, a.kv_head_stride, a.scale);
  return hipGetLastError();
}

}  // namespace sp
