// Token-level distillation loss (Eq. 1, Sec. 3.2) against a teacher stored as its top-k logits
// per token (App. A): forward (per-token KL, student log-sum-exp, mean) and the gradient with
// respect to the student's logits.  Both are one streaming pass over the [T, V] logits: one
// workgroup per token, 16-byte loads, a running (max, sum) per thread that is rescaled once per
// batch of loads, and a workgroup reduction at the end.  HBM-bound by construction.
#include "bc_common.h"

namespace bc {
namespace {

constexpr int kDistillThreads = 256;
constexpr int kDistillWaves = kDistillThreads / 64;
constexpr int kDistillBatch = 8;       // 16-byte loads in flight per thread
constexpr float kLn2 = 0.6931471805599453f;

struct DistillParams {
  const void* z;            // [T, V] student logits
  const float* tl;          // [T, k] teacher top-k logits
  const int32_t* tidx;      // [T, k] their token ids
  float* loss;              // [T]
  float* lse;               // [T]   (forward: nullable output; backward: input)
  void* dz;                 // [T, V] backward output, dtype of z
  int64_t T;
  int32_t V, k;
  float grad_scale;
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
// every thread gets the result; red: kDistillWaves floats of LDS, reusable after the call
__device__ __forceinline__ float block_max(float x, float* red) {
  x = wave_max(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < kDistillWaves; ++i) r = fmaxf(r, red[i]);
  return r;
}
__device__ __forceinline__ float block_sum(float x, float* red) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < kDistillWaves; ++i) r += red[i];   // fixed order: reproducible
  return r;
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
// 16 bytes read once: no reuse, so keep them out of the way of the caches
__device__ __forceinline__ uint4 load16_stream(const uint4* p) {
  const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(r.x, r.y, r.z, r.w);
}

template <typename T> __device__ __forceinline__ float load_elem(const void* p, int64_t i);
template <> __device__ __forceinline__ float load_elem<float>(const void* p, int64_t i) {
  return static_cast<const float*>(p)[i];
}
template <> __device__ __forceinline__ float load_elem<bf16_t>(const void* p, int64_t i) {
  return __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16);
}
__device__ __forceinline__ uint32_t bf16_rne(float f) {   // finite or inf/nan preserved
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
typedef __attribute__((ext_vector_type(2))) float ds_f32x2_t;
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {   // RNE, a in the low half
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(ds_f32x2_t{a, b}, bf16x2_t));
}
__device__ __forceinline__ void store16_stream(uint4* p, const uint4& w) {
  __builtin_nontemporal_store(u32x4_t{w.x, w.y, w.z, w.w}, reinterpret_cast<u32x4_t*>(p));
}
template <typename T> __device__ __forceinline__ void store_elem(void* p, int64_t i, float x);
template <> __device__ __forceinline__ void store_elem<float>(void* p, int64_t i, float x) {
  static_cast<float*>(p)[i] = x;
}
template <> __device__ __forceinline__ void store_elem<bf16_t>(void* p, int64_t i, float x) {
  static_cast<uint16_t*>(p)[i] = static_cast<uint16_t>(bf16_rne(x));
}

// Running log-sum-exp of one row in the base-2 domain: returns (max, sum of 2^(x*log2e - max))
// reduced over the workgroup.  VEC: rows are 16-byte aligned and V is a whole number of units.
template <typename T, bool VEC>
__device__ __forceinline__ void row_lse(const void* zrow, int32_t V, float* red, float& m_out,
                                        float& s_out) {
  constexpr int EPU = Elem<T>::per16;
  float m = kNegBig, s = 0.f;
  if (VEC) {
    const uint4* row = static_cast<const uint4*>(zrow);
    const int units = V / EPU;
    for (int u0 = threadIdx.x; u0 < units; u0 += kDistillThreads * kDistillBatch) {
      uint4 r[kDistillBatch] = {};
#pragma unroll
      for (int b = 0; b < kDistillBatch; ++b) {
        const int u = u0 + b * kDistillThreads;
        if (u < units) r[b] = load16_stream(row + u);
      }
      float x[kDistillBatch][EPU];
      float bm = kNegBig;
#pragma unroll
      for (int b = 0; b < kDistillBatch; ++b) {
        const int u = u0 + b * kDistillThreads;
        unpack16(r[b], x[b], T{});
#pragma unroll
        for (int e = 0; e < EPU; ++e) {
          x[b][e] = (u < units) ? x[b][e] * kLog2e : kNegBig;
          bm = fmaxf(bm, x[b][e]);
        }
      }
      const float mn = fmaxf(m, bm);
      s *= fast_exp2(m - mn);
      m = mn;
      float acc = 0.f;
#pragma unroll
      for (int b = 0; b < kDistillBatch; ++b)
#pragma unroll
        for (int e = 0; e < EPU; ++e) acc += fast_exp2(x[b][e] - m);
      s += acc;
    }
  } else {
    for (int v = threadIdx.x; v < V; v += kDistillThreads) {
      const float x = load_elem<T>(zrow, v) * kLog2e;
      const float mn = fmaxf(m, x);
      s = s * fast_exp2(m - mn) + fast_exp2(x - mn);
      m = mn;
    }
  }
  const float M = block_max(m, red);
  s_out = block_sum(s * fast_exp2(m - M), red);
  m_out = M;
}

// Teacher side of one token: softmax over its k stored logits.  Each thread keeps the entries
// i = tid, tid + 256, ... (at most kMaxPerThread of them).
constexpr int kMaxPerThread = 4;   // k <= 1024

template <typename T, bool VEC>
__global__ void __launch_bounds__(kDistillThreads)
topk_kl_fwd_kernel(DistillParams p) {
  __shared__ float red[kDistillWaves];
  const int64_t t = blockIdx.x;
  const void* zrow = static_cast<const char*>(p.z) + t * p.V * Elem<T>::size;
  // the k gathered student logits and the teacher row first: their latency hides behind the stream
  float zs[kMaxPerThread], tl[kMaxPerThread];
  bool bad = false;
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) {
    const int i = threadIdx.x + j * kDistillThreads;
    zs[j] = 0.f; tl[j] = kNegBig;
    if (i < p.k) {
      int32_t id = p.tidx[t * p.k + i];
      if (id < 0 || id >= p.V) { bad = true; id = 0; }
      zs[j] = load_elem<T>(zrow, id);
      tl[j] = p.tl[t * p.k + i];
    }
  }
  float m2, s2;
  row_lse<T, VEC>(zrow, p.V, red, m2, s2);
  const float lse_s = (m2 + __log2f(s2)) * kLn2;
  float tm = kNegBig;
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) tm = fmaxf(tm, tl[j]);
  tm = block_max(tm, red);
  float ts = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) ts += fast_exp2((tl[j] - tm) * kLog2e);
  ts = block_sum(ts, red);
  const float lse_t = tm + __log2f(ts) * kLn2;
  float kl = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) {
    const int i = threadIdx.x + j * kDistillThreads;
    if (i < p.k) {
      const float lpt = tl[j] - lse_t;
      kl += fast_exp2(lpt * kLog2e) * (lpt - (zs[j] - lse_s));
    }
  }
  if (bad) kl = __builtin_nanf("");
  kl = block_sum(kl, red);
  if (threadIdx.x == 0) {
    p.loss[t] = kl;
    if (p.lse) p.lse[t] = lse_s;
  }
}

// mean of T floats in double, one workgroup, fixed order
__global__ void __launch_bounds__(1024) mean_kernel(const float* x, int64_t T, float* out) {
  __shared__ double part[1024];
  double a = 0.0;
  for (int64_t i = threadIdx.x; i < T; i += 1024) a += static_cast<double>(x[i]);
  part[threadIdx.x] = a;
  __syncthreads();
  for (int s = 512; s >= 1; s >>= 1) {
    if (static_cast<int>(threadIdx.x) < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = static_cast<float>(part[0] / static_cast<double>(T));
}

template <typename T, bool VEC>
__global__ void __launch_bounds__(kDistillThreads)
topk_kl_bwd_kernel(DistillParams p) {
  __shared__ float red[kDistillWaves];
  constexpr int EPU = Elem<T>::per16;
  const int64_t t = blockIdx.x;
  const void* zrow = static_cast<const char*>(p.z) + t * p.V * Elem<T>::size;
  void* drow = static_cast<char*>(p.dz) + t * p.V * Elem<T>::size;
  const float nl = -p.lse[t] * kLog2e;
  const float gs = p.grad_scale;
  // teacher probabilities of this token
  float tl[kMaxPerThread];
  int32_t id[kMaxPerThread];
  float tm = kNegBig;
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) {
    const int i = threadIdx.x + j * kDistillThreads;
    tl[j] = kNegBig; id[j] = -1;
    if (i < p.k) {
      tl[j] = p.tl[t * p.k + i];
      const int32_t x = p.tidx[t * p.k + i];
      id[j] = (x >= 0 && x < p.V) ? x : -1;
    }
    tm = fmaxf(tm, tl[j]);
  }
  tm = block_max(tm, red);
  float ts = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) ts += fast_exp2((tl[j] - tm) * kLog2e);
  ts = block_sum(ts, red);
  const float inv_ts = 1.f / ts;

  if (VEC) {
    const uint4* row = static_cast<const uint4*>(zrow);
    uint4* out = static_cast<uint4*>(drow);
    const int units = p.V / EPU;
    for (int u0 = threadIdx.x; u0 < units; u0 += kDistillThreads * kDistillBatch) {
      uint4 r[kDistillBatch] = {};
#pragma unroll
      for (int b = 0; b < kDistillBatch; ++b) {
        const int u = u0 + b * kDistillThreads;
        if (u < units) r[b] = load16_stream(row + u);
      }
#pragma unroll
      for (int b = 0; b < kDistillBatch; ++b) {
        const int u = u0 + b * kDistillThreads;
        if (u >= units) continue;
        float x[EPU];
        unpack16(r[b], x, T{});
#pragma unroll
        for (int e = 0; e < EPU; ++e) x[e] = gs * fast_exp2(fmaf(x[e], kLog2e, nl));
        uint4 w;
        if constexpr (EPU == 4) {
          w = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]),
                         __float_as_uint(x[3]));
        } else {
          w = make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]),
                         pack_bf16(x[6], x[7]));
        }
        store16_stream(out + u, w);
      }
    }
  } else {
    for (int v = threadIdx.x; v < p.V; v += kDistillThreads)
      store_elem<T>(drow, v, gs * fast_exp2(fmaf(load_elem<T>(zrow, v), kLog2e, nl)));
  }
  // the k teacher ids: overwrite with softmax minus the teacher probability, computed afresh from
  // the logit (one rounding).  The barrier orders these stores after the streaming stores of the
  // same workgroup.
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) {
    if (id[j] >= 0) {
      const float ps = fast_exp2(fmaf(load_elem<T>(zrow, id[j]), kLog2e, nl));
      const float pt = fast_exp2((tl[j] - tm) * kLog2e) * inv_ts;
      store_elem<T>(drow, id[j], gs * (ps - pt));
    }
  }
}

int32_t check_distill(int64_t T, int32_t V, int32_t k, const void* z, int32_t dtype,
                      const float* tl, const int32_t* tidx) {
  if (!z || !tl || !tidx) return BC_ERR_ARG;
  if (dtype != BC_F32 && dtype != BC_BF16) return BC_ERR_SHAPE;
  if (T < 0 || T > 0x7fffffffLL || V < 1 || k < 1 || k > V ||
      k > kMaxPerThread * kDistillThreads)
    return BC_ERR_SHAPE;
  return BC_OK;
}

bool rows_vectorisable(const void* a, const void* b, int32_t V, int32_t dtype) {
  return aligned16(a) && (!b || aligned16(b)) &&
         (static_cast<int64_t>(V) * elem_size(dtype)) % 16 == 0;
}

}  // namespace
}  // namespace bc

extern "C" int32_t bc_topk_kl_loss(int64_t T, int32_t V, int32_t k, const void* student_logits,
                                   int32_t logits_dtype, const float* teacher_logits,
                                   const int32_t* teacher_idx, float* loss_per_token,
                                   float* lse, float* loss_mean, void* stream) {
  using namespace bc;
  int32_t st = check_distill(T, V, k, student_logits, logits_dtype, teacher_logits, teacher_idx);
  if (st != BC_OK) return st;
  if (!loss_per_token) return BC_ERR_ARG;
  if (T == 0) return BC_OK;
  DistillParams p{};
  p.z = student_logits; p.tl = teacher_logits; p.tidx = teacher_idx;
  p.loss = loss_per_token; p.lse = lse; p.T = T; p.V = V; p.k = k;
  const bool vec = rows_vectorisable(student_logits, nullptr, V, logits_dtype);
  const dim3 grid(static_cast<unsigned>(T)), block(kDistillThreads);
  hipStream_t s = as_stream(stream);
  if (logits_dtype == BC_BF16) {
    if (vec) hipLaunchKernelGGL((topk_kl_fwd_kernel<bf16_t, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((topk_kl_fwd_kernel<bf16_t, false>), grid, block, 0, s, p);
  } else {
    if (vec) hipLaunchKernelGGL((topk_kl_fwd_kernel<float, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((topk_kl_fwd_kernel<float, false>), grid, block, 0, s, p);
  }
  if (loss_mean) hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(1024), 0, s, loss_per_token, T, loss_mean);
  return launch_status();
}

extern "C" int32_t bc_topk_kl_loss_bwd(int64_t T, int32_t V, int32_t k,
                                       const void* student_logits, int32_t logits_dtype,
                                       const float* teacher_logits, const int32_t* teacher_idx,
                                       const float* lse, float grad_scale, void* dlogits,
                                       void* stream) {
  using namespace bc;
  int32_t st = check_distill(T, V, k, student_logits, logits_dtype, teacher_logits, teacher_idx);
  if (st != BC_OK) return st;
  if (!lse || !dlogits || dlogits == student_logits) return BC_ERR_ARG;
  if (T == 0) return BC_OK;
  DistillParams p{};
  p.z = student_logits; p.tl = teacher_logits; p.tidx = teacher_idx;
  p.lse = const_cast<float*>(lse); p.dz = dlogits; p.T = T; p.V = V; p.k = k;
  p.grad_scale = grad_scale;
  const bool vec = rows_vectorisable(student_logits, dlogits, V, logits_dtype);
  const dim3 grid(static_cast<unsigned>(T)), block(kDistillThreads);
  hipStream_t s = as_stream(stream);
  if (logits_dtype == BC_BF16) {
    if (vec) hipLaunchKernelGGL((topk_kl_bwd_kernel<bf16_t, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((topk_kl_bwd_kernel<bf16_t, false>), grid, block, 0, s, p);
  } else {
    if (vec) hipLaunchKernelGGL((topk_kl_bwd_kernel<float, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((topk_kl_bwd_kernel<float, false>), grid, block, 0, s, p);
  }
  return launch_status();
}
