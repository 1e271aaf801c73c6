// a2: Bayesian path saliency (Sec. 3.2.3; App. B.1 Eq. 2).
//
// Kernel 1 streams every scored logit row once (HBM-bound): per row the log-likelihood of the
// target token, lp = x[target] - logsumexp(x).  Kernel 2 reduces lp over the rows of each path
// slot in a fixed order (no float atomics), applies SUM or MEAN and adds the prior.
#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

constexpr int kSalThreads = 256;
constexpr int kSalUnroll = 4;      // 16-byte vectors in flight per thread and step

template <typename T>
__global__ __launch_bounds__(kSalThreads) void row_loglik_kernel(const T *__restrict__ logits, int64_t vocab,
                                                               int64_t row_stride,
                                                               const int32_t *__restrict__ target,
                                                               float *__restrict__ lp_out) {
  constexpr int EV = Elem<T>::kVec;
  const int64_t r = blockIdx.x;
  const int32_t tgt = target[r];
  if (tgt < 0) {                                 // row not scored: do not touch its logits
    if (threadIdx.x == 0) lp_out[r] = 0.f;
    return;
  }
  const T *row = logits + r * row_stride;
  const int64_t n_vec = vocab / EV;
  const u32x4 *vrow = reinterpret_cast<const u32x4 *>(row);

  // running maximum m (natural units) and s = sum exp(x - m), per thread
  float m = kNegBig, s = 0.f;
  int64_t i = threadIdx.x;
  for (; i + int64_t(kSalUnroll - 1) * kSalThreads < n_vec; i += int64_t(kSalUnroll) * kSalThreads) {
    u32x4 raw[kSalUnroll];
#pragma unroll
    for (int u = 0; u < kSalUnroll; ++u) raw[u] = ld16_stream(vrow + i + int64_t(u) * kSalThreads);
    float x[kSalUnroll * EV];
#pragma unroll
    for (int u = 0; u < kSalUnroll; ++u) Elem<T>::unpack(raw[u], x + u * EV);
    float mx = x[0];
#pragma unroll
    for (int j = 1; j < kSalUnroll * EV; ++j) mx = fmaxf(mx, x[j]);
    const float m_new = fmaxf(m, mx);
    const float mb = m_new * kLog2e;
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < kSalUnroll * EV; ++j) acc += fast_exp2(fmaf(x[j], kLog2e, -mb));
    s = fmaf(s, fast_exp2((m - m_new) * kLog2e), acc);
    m = m_new;
  }
  for (; i < n_vec; i += kSalThreads) {          // remaining whole vectors
    const u32x4 raw = vrow[i];
    float x[EV];
    Elem<T>::unpack(raw, x);
    float mx = x[0];
#pragma unroll
    for (int j = 1; j < EV; ++j) mx = fmaxf(mx, x[j]);
    const float m_new = fmaxf(m, mx);
    const float mb = m_new * kLog2e;
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < EV; ++j) acc += fast_exp2(fmaf(x[j], kLog2e, -mb));
    s = fmaf(s, fast_exp2((m - m_new) * kLog2e), acc);
    m = m_new;
  }
  {                                              // scalar tail (vocab not a multiple of the vector)
    const int64_t j = n_vec * EV + threadIdx.x;
    if (j < vocab) {
      const float x = Elem<T>::load1(row + j);
      const float m_new = fmaxf(m, x);
      s = fmaf(s, fast_exp2((m - m_new) * kLog2e), fast_exp2((x - m_new) * kLog2e));
      m = m_new;
    }
  }
  // combine (m, s) over the workgroup: fixed butterfly inside a wave, then across the 4 waves
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float m_o = __shfl_xor(m, off), s_o = __shfl_xor(s, off);
    const float m_new = fmaxf(m, m_o);
    s = s * fast_exp2((m - m_new) * kLog2e) + s_o * fast_exp2((m_o - m_new) * kLog2e);
    m = m_new;
  }
  __shared__ float sm[kSalThreads / 64], ss[kSalThreads / 64];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sm[wave] = m; ss[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sm[0];
#pragma unroll
    for (int w = 1; w < kSalThreads / 64; ++w) M = fmaxf(M, sm[w]);
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < kSalThreads / 64; ++w) S += ss[w] * fast_exp2((sm[w] - M) * kLog2e);
    const int64_t t = tgt < vocab ? tgt : vocab - 1;
    const float xt = Elem<T>::load1(row + t);
    lp_out[r] = xt - (M + __logf(S));
  }
}

// Rows that are not scored carry lp = 0, so the SUM needs only row_path and lp; the MEAN also
// counts the scored rows.  All loads of a thread are independent (issued together), partial sums
// are combined in a fixed tree order.
constexpr int kRedThreads = 1024;
__global__ __launch_bounds__(kRedThreads) void path_reduce_kernel(const float *__restrict__ lp,
                                                                  const int32_t *__restrict__ target,
                                                                  const int32_t *__restrict__ row_path,
                                                                  int64_t n_rows, const float *__restrict__ prior,
                                                                  int mode, float *__restrict__ score) {
  const int slot = blockIdx.x;
  float acc = 0.f;
  int cnt = 0;
  for (int64_t r0 = 0; r0 < n_rows; r0 += 4 * kRedThreads) {
    int32_t rp[4];
    float v[4];
    int32_t tg[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t r = r0 + threadIdx.x + u * kRedThreads;
      const bool in = r < n_rows;
      rp[u] = in ? row_path[r] : -1;
      v[u] = in ? lp[r] : 0.f;
      tg[u] = (in && mode == 1) ? target[r] : 0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (rp[u] == slot) { acc += v[u]; cnt += tg[u] >= 0 ? 1 : 0; }
  }
  __shared__ float sa[kRedThreads];
  __shared__ int sc[kRedThreads];
  sa[threadIdx.x] = acc; sc[threadIdx.x] = cnt;
  __syncthreads();
  for (int off = kRedThreads / 2; off >= 1; off >>= 1) {
    if (threadIdx.x < off) { sa[threadIdx.x] += sa[threadIdx.x + off]; sc[threadIdx.x] += sc[threadIdx.x + off]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    float v = sa[0];
    if (mode == 1) v = sc[0] > 0 ? v / float(sc[0]) : 0.f;
    if (prior) v += prior[slot];
    score[slot] = v;
  }
}

hipError_t launch_saliency(const void *logits, sp_dtype dt, int64_t n_rows, int64_t vocab, int64_t row_stride,
                           const int32_t *target, const int32_t *row_path, const float *prior, int32_t n_slots,
                           int mode, float *lp_ws, float *score, hipStream_t s) {
  if (n_rows > 0) {
    if (dt == SP_BF16)
      hipLaunchKernelGGL(row_loglik_kernel<__bf16>, dim3(unsigned(n_rows)), dim3(kSalThreads), 0, s,
                         static_cast<const __bf16 *>(logits), vocab, row_stride, target, lp_ws);
    else
      hipLaunchKernelGGL(row_loglik_kernel<float>, dim3(unsigned(n_rows)), dim3(kSalThreads), 0, s,
                         static_cast<const float *>(logits), vocab, row_stride, target, lp_ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(path_reduce_kernel, dim3(n_slots), dim3(kRedThreads), 0, s, lp_ws, target, row_path, n_rows, prior,
                     mode, score);
  return hipGetLastError();
}

}  // namespace sp
