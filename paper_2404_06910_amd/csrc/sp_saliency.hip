// a2: Bayesian path saliency (Sec. 3.2.3; App. B.1 Eq. 2).
//
// Kernel 1 (HBM-bound, one workgroup per scored logit row) streams the row once and stores the
// log-likelihood of its target token, lp = x[target] - logsumexp(x), as 64-bit fixed point (2^-36 units),
// with one plain store.  It touches no atomic: a workgroup is not retired before its memory operations are
// acknowledged, and a device-scope atomic takes microseconds to come back while HBM is saturated (measured:
// 16 to 42 us per launch, whether the kernel waits for its atomics or not).
// Kernel 2 (one thread per row, a few dozen workgroups) reduces per path slot without floating-point
// atomics and without rescanning the rows per slot: every row adds its value to its slot with an INTEGER
// atomic -- integer addition is associative, so the sum does not depend on the order of arrival and equal
// inputs give bit-identical scores; rows whose lp is not finite set a flag bit instead.  A counter finds
// the workgroup that finishes last; it turns the sums into scores (SUM or MEAN, plus the prior) and puts
// every accumulator back to zero, the state the next launch expects.
#include <mutex>

#include "sp_device.h"
#include "sp_internal.h"

namespace sp {

constexpr int kSalThreads = 256;
constexpr int kSalUnroll = 4;      // 16-byte vectors in flight per thread and step
constexpr double kFixOne = 68719476736.0;        // 2^36
constexpr float kFixLimit = 6.0e7f;              // |lp| above this (about 2^26) is treated as infinite

// Scratch of the entry point that allocates nothing: the launch counter, the per-slot accumulators and
// the per-row log-likelihoods of the largest problem it accepts (kSalStaticRows rows, kSalStaticSlots path slots), on every
// GPU the library runs on; zero at load, and the accumulators are left at zero by every launch.
static __device__ __align__(256) unsigned char scratch[kSalStaticBytes];

template <typename T>
__global__ __launch_bounds__(kSalThreads) void saliency_kernel(const T *__restrict__ logits, int64_t vocab,
                                                             int64_t row_stride,
                                                             const int32_t *__restrict__ target,
                                                             RowLp *__restrict__ lp_out) {
  constexpr int EV = Elem<T>::kVec;
  const int64_t r = blockIdx.x;
  const int32_t tgt = target[r];
  __shared__ float sm[kSalThreads / 64], ss[kSalThreads / 64];
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
    // combine (m, s) over the workgroup: fixed butterfly inside a wave, then across the waves
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
  if (threadIdx.x != 0) return;
  if (tgt < 0) { lp_out[r] = RowLp{0ll, 0u, 0u}; return; }
  float M = sm[0];
#pragma unroll
  for (int w = 1; w < kSalThreads / 64; ++w) M = fmaxf(M, sm[w]);
  float S = 0.f;
#pragma unroll
  for (int w = 0; w < kSalThreads / 64; ++w) S += ss[w] * fast_exp2((sm[w] - M) * kLog2e);
  const int64_t t = tgt < vocab ? tgt : vocab - 1;
  const float lp = Elem<T>::load1(row + t) - (M + __logf(S));
  // fixed point here, where every row has a thread of its own; a value that is not finite becomes a flag
  RowLp o{0ll, 0u, 1u};
  if (lp != lp || fabsf(lp) > kFixLimit) o.flags = lp != lp ? 4u : (lp < 0.f ? 1u : 2u);
  else o.q = __double2ll_rn(double(lp) * kFixOne);
  lp_out[r] = o;
}

constexpr int kRedThreads = 256;
__global__ __launch_bounds__(kRedThreads) void saliency_reduce_kernel(const RowLp *__restrict__ lp,
                                                                      const int32_t *__restrict__ row_path,
                                                                      int64_t n_rows, const float *__restrict__ prior,
                                                                      int32_t n_slots, int mode, SalSlot *__restrict__ acc,
                                                                      uint32_t *__restrict__ done,
                                                                      float *__restrict__ score) {
  const int64_t r = (int64_t)blockIdx.x * kRedThreads + threadIdx.x;
  __shared__ int s_last;
  RowLp v{0ll, 0u, 0u};
  int32_t slot = 0;
  if (r < n_rows) {
    v = lp[r];
    slot = row_path[r];
    slot = slot < 0 ? 0 : (slot >= n_slots ? n_slots - 1 : slot);
  }
  // Rows of one path usually sit next to each other, and atomics on one address are performed one after
  // the other: a wave first adds up, per slot, what its own lanes hold (up to kWaveSlots different slots),
  // and one lane sends the total.  Lanes left over send their own value.  The atomics return a value that
  // is kept alive: the barrier below is passed only after they have been performed, so the workgroup that
  // reads the last count sees every sum complete.
  constexpr int kWaveSlots = 4;
  const int lane = threadIdx.x & 63;
  unsigned long long pending = __ballot(v.scored != 0u);
  for (int it = 0; it < kWaveSlots && pending; ++it) {
    const int lead = __ffsll((long long)pending) - 1;
    const int32_t s0 = __shfl(slot, lead);
    const bool mine = ((pending >> lane) & 1ull) && slot == s0;
    long long q = mine && !v.flags ? v.q : 0ll;
    unsigned cnt = mine ? 1u : 0u, fl = mine ? v.flags : 0u;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      q += __shfl_xor(q, off);
      cnt += __shfl_xor(cnt, off);
      fl |= __shfl_xor(fl, off);
    }
    if (lane == lead) {
      SalSlot *a = acc + s0;
      unsigned long long r0 = 0;
      unsigned r1 = 0;
      if (q) r0 = __hip_atomic_fetch_add(&a->sum, (unsigned long long)q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (fl) r1 = __hip_atomic_fetch_or(&a->flags, fl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned r2 = __hip_atomic_fetch_add(&a->count, cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("" ::"v"(r0), "v"(r1), "v"(r2) : "memory");
    }
    pending &= ~__ballot(mine);
  }
  if ((pending >> lane) & 1ull) {
    SalSlot *a = acc + slot;
    unsigned long long r0 = 0;
    unsigned r1 = 0;
    if (v.flags) r1 = __hip_atomic_fetch_or(&a->flags, v.flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else r0 = __hip_atomic_fetch_add(&a->sum, (unsigned long long)v.q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned r2 = __hip_atomic_fetch_add(&a->count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(r0), "v"(r1), "v"(r2) : "memory");
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned before = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = before == gridDim.x - 1 ? 1 : 0;
  }
  __syncthreads();
  if (!s_last) return;
  // the last workgroup: sums -> scores, accumulators back to zero
  for (int i = threadIdx.x; i < n_slots; i += kRedThreads) {
    SalSlot *a = acc + i;
    SalSlot v;
    v.sum = __hip_atomic_load(&a->sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.count = __hip_atomic_load(&a->count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.flags = __hip_atomic_load(&a->flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float x = float(double((long long)v.sum) * (1.0 / kFixOne));
    if (v.flags) x = ((v.flags & 4u) || (v.flags & 3u) == 3u) ? __builtin_nanf("") : ((v.flags & 1u) ? -INFINITY : INFINITY);
    if (mode == 1) x = v.count > 0 ? x / float(v.count) : 0.f;
    if (prior) x += prior[i];
    score[i] = x;
    __hip_atomic_store(&a->sum, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a->count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&a->flags, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (threadIdx.x == 0) __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// scratch: the launch counter (256 bytes), one SalSlot per path slot of the capacity, then one RowLp per
// row; the counter and the accumulators are zero before the launch and left at zero.
hipError_t launch_saliency(const void *logits, sp_dtype dt, int64_t n_rows, int64_t vocab, int64_t row_stride,
                           const int32_t *target, const int32_t *row_path, const float *prior, int32_t n_slots,
                           int mode, void *scratch, int32_t cap_slots, float *score, hipStream_t s) {
  uint32_t *done = static_cast<uint32_t *>(scratch);
  SalSlot *acc = reinterpret_cast<SalSlot *>(static_cast<unsigned char *>(scratch) + 256);
  RowLp *lp = reinterpret_cast<RowLp *>(acc + cap_slots);
  if (n_rows > 0) {
    if (dt == SP_BF16)
      hipLaunchKernelGGL(saliency_kernel<__bf16>, dim3(unsigned(n_rows)), dim3(kSalThreads), 0, s,
                         static_cast<const __bf16 *>(logits), vocab, row_stride, target, lp);
    else
      hipLaunchKernelGGL(saliency_kernel<float>, dim3(unsigned(n_rows)), dim3(kSalThreads), 0, s,
                         static_cast<const float *>(logits), vocab, row_stride, target, lp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const unsigned grid = n_rows > 0 ? unsigned((n_rows + kRedThreads - 1) / kRedThreads) : 1u;
  hipLaunchKernelGGL(saliency_reduce_kernel, dim3(grid), dim3(kRedThreads), 0, s, lp, row_path, n_rows, prior, n_slots,
                     mode, acc, done, score);
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
