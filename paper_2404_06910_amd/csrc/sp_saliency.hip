// a2: Bayesian path saliency (Sec. 3.2.3; App. B.1 Eq. 2), one launch.
//
// One workgroup streams one scored logit row once (HBM-bound): the log-likelihood of the row's target
// token, lp = x[target] - logsumexp(x).  The per-path reduction is fused into the same launch without
// floating-point atomics: every row adds its lp, converted to 64-bit fixed point (2^-36 units), to its
// path slot with an INTEGER atomic -- integer addition is associative, so the sum does not depend on the
// order in which the rows arrive and equal inputs give bit-identical scores.  Rows whose lp is not finite
// set a flag bit of the slot instead.  A launch-wide counter finds the workgroup that finishes last; it
// turns the sums into scores (SUM or MEAN, plus the prior) and puts every accumulator it used back to
// zero, which is the state the next launch expects.
#include <mutex>

#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

constexpr int kSalThreads = 256;
constexpr int kSalUnroll = 4;      // 16-byte vectors in flight per thread and step
constexpr double kFixOne = 68719476736.0;        // 2^36
constexpr float kFixLimit = 6.0e7f;              // |lp| above this (about 2^26) is treated as infinite

// Scratch of the entry point that allocates nothing: the launch counter plus one SalSlot per path slot,
// kSalStaticBytes on every GPU the library runs on, zero at load and left at zero by every launch.
static __device__ __align__(256) unsigned char scratch[kSalStaticBytes];

template <typename T>
__global__ __launch_bounds__(kSalThreads) void saliency_kernel(const T *__restrict__ logits, int64_t vocab,
                                                             int64_t row_stride,
                                                             const int32_t *__restrict__ target,
                                                             const int32_t *__restrict__ row_path,
                                                             const float *__restrict__ prior, int32_t n_slots,
                                                             int mode, SalSlot *__restrict__ acc,
                                                             uint32_t *__restrict__ done,
                                                             float *__restrict__ score) {
  constexpr int EV = Elem<T>::kVec;
  const int64_t r = blockIdx.x;
  const int32_t tgt = target[r];
  __shared__ float sm[kSalThreads / 64], ss[kSalThreads / 64];
  __shared__ int s_last;
  float m = kNegBig, s = 0.f;
  const T *row = logits + r * row_stride;
  if (tgt >= 0) {                                // a row that is not scored does not touch its logits
    const int64_t n_vec = vocab / EV;
    const u32x4 *vrow = reinterpret_cast<const u32x4 *>(row);
    // running maximum m (natural units) and s = sum exp(x - m), per thread
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
      float a = 0.f;
#pragma unroll
      for (int j = 0; j < kSalUnroll * EV; ++j) a += fast_exp2(fmaf(x[j], kLog2e, -mb));
      s = fmaf(s, fast_exp2((m - m_new) * kLog2e), a);
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
      float a = 0.f;
#pragma unroll
      for (int j = 0; j < EV; ++j) a += fast_exp2(fmaf(x[j], kLog2e, -mb));
      s = fmaf(s, fast_exp2((m - m_new) * kLog2e), a);
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
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sm[wave] = m; ss[wave] = s; }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (tgt >= 0) {
      float M = sm[0];
#pragma unroll
      for (int w = 1; w < kSalThreads / 64; ++w) M = fmaxf(M, sm[w]);
      float S = 0.f;
#pragma unroll
      for (int w = 0; w < kSalThreads / 64; ++w) S += ss[w] * fast_exp2((sm[w] - M) * kLog2e);
      const int64_t t = tgt < vocab ? tgt : vocab - 1;
      const float lp = Elem<T>::load1(row + t) - (M + __logf(S));
      int32_t slot = row_path[r];
      slot = slot < 0 ? 0 : (slot >= n_slots ? n_slots - 1 : slot);
      SalSlot *a = acc + slot;
      // every update is an atomic that returns; the counter below is touched only after they have
      // been performed, so the workgroup that reads the last count sees every sum complete
      unsigned long long r0 = 0;
      unsigned r1 = 0;
      if (lp != lp || fabsf(lp) > kFixLimit) {
        const unsigned bit = lp != lp ? 4u : (lp < 0.f ? 1u : 2u);
        r1 = __hip_atomic_fetch_or(&a->flags, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        const long long q = __double2ll_rn(double(lp) * kFixOne);
        r0 = __hip_atomic_fetch_add(&a->sum, (unsigned long long)q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      const unsigned r2 = __hip_atomic_fetch_add(&a->count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("" ::"v"(r0), "v"(r1), "v"(r2) : "memory");
    }
    const unsigned before = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = before == gridDim.x - 1 ? 1 : 0;
  }
  __syncthreads();
  if (!s_last) return;
  // the last workgroup: sums -> scores, accumulators back to zero
  for (int i = threadIdx.x; i < n_slots; i += kSalThreads) {
    SalSlot *a = acc + i;
    const unsigned long long sum = __hip_atomic_load(&a->sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned cnt = __hip_atomic_load(&a->count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned fl = __hip_atomic_load(&a->flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float v = float(double((long long)sum) * (1.0 / kFixOne));
    if (fl) v = ((fl & 4u) || (fl & 3u) == 3u) ? __builtin_nanf("") : ((fl & 1u) ? -INFINITY : INFINITY);
    if (mode == 1) v = cnt > 0 ? v / float(cnt) : 0.f;
    if (prior) v += prior[i];
    score[i] = v;
    __hip_atomic_store(&a->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a->count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a->flags, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (threadIdx.x == 0) __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// n_rows == 0: no row arrives, so the scores are written directly
__global__ void saliency_empty_kernel(const float *__restrict__ prior, int32_t n_slots, float *__restrict__ score) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_slots) score[i] = prior ? prior[i] : 0.f;
}

hipError_t launch_saliency(const void *logits, sp_dtype dt, int64_t n_rows, int64_t vocab, int64_t row_stride,
                           const int32_t *target, const int32_t *row_path, const float *prior, int32_t n_slots,
                           int mode, void *scratch_dev, float *score, hipStream_t s) {
  if (n_rows <= 0) {
    hipLaunchKernelGGL(saliency_empty_kernel, dim3((n_slots + 255) / 256), dim3(256), 0, s, prior, n_slots, score);
    return hipGetLastError();
  }
  // layout of the scratch block: the launch counter in the first 256 bytes, then one SalSlot per path slot
  uint32_t *done = static_cast<uint32_t *>(scratch_dev);
  SalSlot *acc = reinterpret_cast<SalSlot *>(static_cast<unsigned char *>(scratch_dev) + 256);
  if (dt == SP_BF16)
    hipLaunchKernelGGL(saliency_kernel<__bf16>, dim3(unsigned(n_rows)), dim3(kSalThreads), 0, s,
                       static_cast<const __bf16 *>(logits), vocab, row_stride, target, row_path, prior, n_slots, mode,
                       acc, done, score);
  else
    hipLaunchKernelGGL(saliency_kernel<float>, dim3(unsigned(n_rows)), dim3(kSalThreads), 0, s,
                       static_cast<const float *>(logits), vocab, row_stride, target, row_path, prior, n_slots, mode,
                       acc, done, score);
  return hipGetLastError();
}

// Address of this device's copy of the static scratch array.  In host code the array's name is only a
// stand-in, not a device address: the address comes from the runtime, once per device, with that device
// current (the caller has made it current), and is kept per device.
hipError_t saliency_static_scratch(int device, void **out) {
  static std::mutex mu;
  static void *ptrs[kMaxDevices] = {};
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[device]) {
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    ptrs[device] = p;
  }
  *out = ptrs[device];
  return hipSuccess;
}

}  // namespace sp
