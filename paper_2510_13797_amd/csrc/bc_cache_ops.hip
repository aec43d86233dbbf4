// Cache maintenance kernels: prompt fill, row append, beacon append + eviction
// (Alg. 1 and Sec. 3.1 of the paper).  Pure data movement plus integer tables; all copies
// move 16-byte units so a row write is one coalesced burst per KV head.
#include "bc_common.h"

namespace bc {

struct CacheView {
  char* k_slab;
  char* v_slab;
  const int64_t* base;
  const int32_t* cap;
  const int32_t* P;
  int32_t* c;
  int32_t* nb;
  int32_t* w;
  int32_t* err;
  int32_t Hkv;
  int32_t row_bytes;   // d * element size
};

static CacheView make_view(const bc_shape* sh, const bc_cache* c) {
  CacheView v;
  v.k_slab = static_cast<char*>(c->k_slab);
  v.v_slab = static_cast<char*>(c->v_slab);
  v.base = c->base; v.cap = c->cap; v.P = c->P; v.c = c->c;
  v.nb = c->nb; v.w = c->w; v.err = c->err;
  v.Hkv = sh->Hkv;
  v.row_bytes = sh->d * elem_size(sh->kv_dtype);
  return v;
}

// byte offset of row j of (sequence s, KV head kvh)
__device__ __forceinline__ int64_t row_offset(const CacheView& cv, int s, int kvh, int cap, int j) {
  return ((cv.base[s] * cv.Hkv + (int64_t)kvh * cap + j) * (int64_t)cv.row_bytes);
}

// ---------------------------------------------------------------------------
// Prompt fill: one 16-byte unit per thread; sequence found by binary search.
// ---------------------------------------------------------------------------
// admit == NULL: fill every sequence whose span equals P[s]; otherwise fill the slots selected by
// admit[] (their P[s] is being rewritten by the table kernel of the same call).
__global__ void cache_init_kernel(CacheView cv, const char* __restrict__ kp,
                                  const char* __restrict__ vp,
                                  const int64_t* __restrict__ off, int B, int64_t total_rows,
                                  const uint8_t* __restrict__ admit) {
  const int units_per_row = cv.row_bytes >> 4;
  const int64_t units_per_tok = (int64_t)units_per_row * cv.Hkv;
  const int64_t n = total_rows * units_per_tok;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t tok = i / units_per_tok;
    const int rem = (int)(i - tok * units_per_tok);
    const int kvh = rem / units_per_row, u = rem - kvh * units_per_row;
    int lo = 0, hi = B;                       // largest s with off[s] <= tok
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (off[mid] <= tok) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int j = (int)(tok - off[s]);
    const int cap = cv.cap[s];
    const int64_t span = off[s + 1] - off[s];
    if (span > cap) continue;                          // flagged by the table kernel
    if (admit ? !admit[s] : span != cv.P[s]) continue;
    const int64_t dst = row_offset(cv, s, kvh, cap, j) + ((int64_t)u << 4);
    *reinterpret_cast<uint4*>(cv.k_slab + dst) = reinterpret_cast<const uint4*>(kp)[i];
    *reinterpret_cast<uint4*>(cv.v_slab + dst) = reinterpret_cast<const uint4*>(vp)[i];
  }
}

__global__ void cache_init_tables_kernel(CacheView cv, const int64_t* __restrict__ off, int B) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= B) return;
  const int64_t span = off[s + 1] - off[s];
  if (span != cv.P[s]) atomicOr(cv.err, BC_ERRBIT_STATE);
  else if (span > cv.cap[s]) atomicOr(cv.err, BC_ERRBIT_CAPACITY);
  cv.nb[s] = 0;
  cv.w[s] = 0;
}

// Slots taken over by new sequences: prompt length, ratio, counters, live flag.
__global__ void admit_tables_kernel(CacheView cv, int32_t* P, const int64_t* __restrict__ off,
                                    const int32_t* __restrict__ new_c,
                                    const uint8_t* __restrict__ admit, uint8_t* live, int B) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= B || !admit[s]) return;
  const int64_t span = off[s + 1] - off[s];
  if (span < 0 || span > cv.cap[s]) { atomicOr(cv.err, BC_ERRBIT_CAPACITY); return; }
  P[s] = (int32_t)span;
  if (new_c) cv.c[s] = new_c[s];
  cv.nb[s] = 0;
  cv.w[s] = 0;
  if (live) live[s] = 1;
}

// ---------------------------------------------------------------------------
// Row append: one workgroup per sequence.
// ---------------------------------------------------------------------------
__global__ void append_kernel(CacheView cv, const char* __restrict__ k, const char* __restrict__ v,
                              const uint8_t* __restrict__ active, int kind) {
  const int s = blockIdx.x;
  if (active && !active[s]) return;
  const int c = cv.c[s], wv = cv.w[s], nbv = cv.nb[s], cap = cv.cap[s];
  const int L = cv.P[s] + nbv + wv;
  if (kind == BC_ROW_TOKEN) {
    if (c > 0 && wv >= c) {
      if (threadIdx.x == 0) atomicOr(cv.err, BC_ERRBIT_STATE);
      return;
    }
  } else if (c <= 0 || wv != c) {
    return;
  }
  if (L >= cap) {
    if (threadIdx.x == 0) atomicOr(cv.err, BC_ERRBIT_CAPACITY);
    return;
  }
  const int upr = cv.row_bytes >> 4;
  const int n = upr * cv.Hkv;
  const uint4* ks = reinterpret_cast<const uint4*>(k) + (int64_t)s * n;
  const uint4* vs = reinterpret_cast<const uint4*>(v) + (int64_t)s * n;
  for (int i = threadIdx.x; i < 2 * n; i += blockDim.x) {
    const int which = i >= n, r = which ? i - n : i;
    const int kvh = r / upr, u = r - kvh * upr;
    const int64_t dst = row_offset(cv, s, kvh, cap, L) + ((int64_t)u << 4);
    if (which) *reinterpret_cast<uint4*>(cv.v_slab + dst) = vs[r];
    else       *reinterpret_cast<uint4*>(cv.k_slab + dst) = ks[r];
  }
  __syncthreads();                       // every thread has read w before it changes
  if (threadIdx.x == 0) cv.w[s] = (kind == BC_ROW_TOKEN) ? wv + 1 : c + 1;
}

// ---------------------------------------------------------------------------
// Beacon append + eviction + compaction: one workgroup per sequence.  With the
// [prompt | beacons | window] order the compaction is a single row write per KV head:
// the beacon lands on the first window slot and the window length drops to zero.
// ---------------------------------------------------------------------------
__global__ void compress_evict_kernel(CacheView cv, const char* __restrict__ bk,
                                      const char* __restrict__ bv,
                                      const uint8_t* __restrict__ active, int require_full) {
  const int s = blockIdx.x;
  if (active && !active[s]) return;
  const int c = cv.c[s];
  if (c <= 0) return;
  const int wv = cv.w[s], nbv = cv.nb[s], cap = cv.cap[s];
  const int dst_row = cv.P[s] + nbv;
  const int upr = cv.row_bytes >> 4;
  const int n = upr * cv.Hkv;
  if (bk) {
    if (wv == c + 1) {
      if (threadIdx.x == 0) atomicOr(cv.err, BC_ERRBIT_STATE);
      return;
    }
    if (!(wv == c || (!require_full && wv >= 1 && wv <= c))) return;
    const uint4* ks = reinterpret_cast<const uint4*>(bk) + (int64_t)s * n;
    const uint4* vs = reinterpret_cast<const uint4*>(bv) + (int64_t)s * n;
    for (int i = threadIdx.x; i < 2 * n; i += blockDim.x) {
      const int which = i >= n, r = which ? i - n : i;
      const int kvh = r / upr, u = r - kvh * upr;
      const int64_t dst = row_offset(cv, s, kvh, cap, dst_row) + ((int64_t)u << 4);
      if (which) *reinterpret_cast<uint4*>(cv.v_slab + dst) = vs[r];
      else       *reinterpret_cast<uint4*>(cv.k_slab + dst) = ks[r];
    }
  } else {
    if (wv != c + 1) return;
    const int src_row = dst_row + c;     // the beacon at the tail; c >= 1 so src != dst
    for (int i = threadIdx.x; i < 2 * n; i += blockDim.x) {
      const int which = i >= n, r = which ? i - n : i;
      const int kvh = r / upr, u = r - kvh * upr;
      char* slab = which ? cv.v_slab : cv.k_slab;
      const int64_t src = row_offset(cv, s, kvh, cap, src_row) + ((int64_t)u << 4);
      const int64_t dst = row_offset(cv, s, kvh, cap, dst_row) + ((int64_t)u << 4);
      *reinterpret_cast<uint4*>(slab + dst) = *reinterpret_cast<const uint4*>(slab + src);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    cv.nb[s] = nbv + 1;
    cv.w[s] = 0;
  }
}

__global__ void set_ratio_kernel(CacheView cv, const int32_t* __restrict__ new_c,
                                 const uint8_t* __restrict__ active, int B) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= B || (active && !active[s])) return;
  const int nc = new_c[s], wv = cv.w[s];
  if (nc > 0 && wv >= nc && wv != 0) { atomicOr(cv.err, BC_ERRBIT_STATE); return; }
  cv.c[s] = nc;
}

}  // namespace bc

using namespace bc;

extern "C" int32_t bc_set_ratio(const bc_shape* shape, const bc_cache* cache, const int32_t* new_c,
                                const uint8_t* active, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!new_c) return BC_ERR_ARG;
  CacheView cv = make_view(shape, cache);
  set_ratio_kernel<<<(shape->B + 255) / 256, 256, 0, as_stream(stream)>>>(cv, new_c, active, shape->B);
  return launch_status();
}

extern "C" int32_t bc_cache_init(const bc_shape* shape, const bc_cache* cache, const void* k_prompt,
                                 const void* v_prompt, const int64_t* prompt_offsets,
                                 int64_t total_rows, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!prompt_offsets || total_rows < 0) return BC_ERR_ARG;
  if (total_rows > 0 && (!k_prompt || !v_prompt || !aligned16(k_prompt) || !aligned16(v_prompt)))
    return BC_ERR_ARG;
  CacheView cv = make_view(shape, cache);
  hipStream_t s = as_stream(stream);
  cache_init_tables_kernel<<<(shape->B + 255) / 256, 256, 0, s>>>(cv, prompt_offsets, shape->B);
  if (total_rows > 0) {
    const int64_t units = total_rows * shape->Hkv * (cv.row_bytes >> 4);
    const int64_t blocks = (units + 255) / 256;
    const int grid = (int)(blocks < 65536 ? blocks : 65536);
    cache_init_kernel<<<grid, 256, 0, s>>>(cv, static_cast<const char*>(k_prompt),
                                           static_cast<const char*>(v_prompt), prompt_offsets,
                                           shape->B, total_rows, nullptr);
  }
  return launch_status();
}

extern "C" int32_t bc_cache_admit(const bc_shape* shape, const bc_cache* cache, const void* k_prompt,
                                  const void* v_prompt, const int64_t* prompt_offsets,
                                  int64_t total_rows, const int32_t* new_c, const uint8_t* admit,
                                  uint8_t* live, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!prompt_offsets || !admit || total_rows < 0) return BC_ERR_ARG;
  if (total_rows > 0 && (!k_prompt || !v_prompt || !aligned16(k_prompt) || !aligned16(v_prompt)))
    return BC_ERR_ARG;
  CacheView cv = make_view(shape, cache);
  hipStream_t s = as_stream(stream);
  // the fill does not read the tables the other kernel writes, so their order is free
  if (total_rows > 0) {
    const int64_t units = total_rows * shape->Hkv * (cv.row_bytes >> 4);
    const int64_t blocks = (units + 255) / 256;
    const int grid = (int)(blocks < 65536 ? blocks : 65536);
    cache_init_kernel<<<grid, 256, 0, s>>>(cv, static_cast<const char*>(k_prompt),
                                           static_cast<const char*>(v_prompt), prompt_offsets,
                                           shape->B, total_rows, admit);
  }
  admit_tables_kernel<<<(shape->B + 255) / 256, 256, 0, s>>>(cv, cache->P, prompt_offsets, new_c,
                                                             admit, live, shape->B);
  return launch_status();
}

extern "C" int32_t bc_append_kv(const bc_shape* shape, const bc_cache* cache, const void* k,
                                const void* v, const uint8_t* active, int32_t kind, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!k || !v || !aligned16(k) || !aligned16(v)) return BC_ERR_ARG;
  if (kind != BC_ROW_TOKEN && kind != BC_ROW_BEACON) return BC_ERR_ARG;
  CacheView cv = make_view(shape, cache);
  append_kernel<<<shape->B, 64, 0, as_stream(stream)>>>(cv, static_cast<const char*>(k),
                                                        static_cast<const char*>(v), active, kind);
  return launch_status();
}

extern "C" int32_t bc_compress_evict(const bc_shape* shape, const bc_cache* cache,
                                     const void* beacon_k, const void* beacon_v,
                                     const uint8_t* active, int32_t require_full_window,
                                     void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if ((beacon_k == nullptr) != (beacon_v == nullptr)) return BC_ERR_ARG;
  if (beacon_k && (!aligned16(beacon_k) || !aligned16(beacon_v))) return BC_ERR_ARG;
  if (!beacon_k && !require_full_window) return BC_ERR_ARG;
  CacheView cv = make_view(shape, cache);
  compress_evict_kernel<<<shape->B, 64, 0, as_stream(stream)>>>(
      cv, static_cast<const char*>(beacon_k), static_cast<const char*>(beacon_v), active,
      require_full_window ? 1 : 0);
  return launch_status();
}

extern "C" int32_t bc_tables_to_host(const bc_shape* shape, const bc_cache* cache, int32_t* nb_host,
                                     int32_t* w_host, int32_t* err_host, void* stream) {
  if (!shape || !cache || shape->B < 1) return BC_ERR_ARG;
  hipStream_t s = as_stream(stream);
  const size_t n = sizeof(int32_t) * (size_t)shape->B;
  if (nb_host && hipMemcpyAsync(nb_host, cache->nb, n, hipMemcpyDeviceToHost, s) != hipSuccess)
    return BC_ERR_HIP;
  if (w_host && hipMemcpyAsync(w_host, cache->w, n, hipMemcpyDeviceToHost, s) != hipSuccess)
    return BC_ERR_HIP;
  if (err_host &&
      hipMemcpyAsync(err_host, cache->err, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess)
    return BC_ERR_HIP;
  return hipStreamSynchronize(s) == hipSuccess ? BC_OK : BC_ERR_HIP;
}

extern "C" const char* bc_status_str(int32_t status) {
  switch (status) {
    case BC_OK: return "ok";
    case BC_ERR_ARG: return "bad argument (null or misaligned pointer, bad flag)";
    case BC_ERR_SHAPE: return "unsupported shape or dtype";
    case BC_ERR_CAPACITY: return "sequence slab is full";
    case BC_ERR_STATE: return "operation not allowed in this cache state";
    case BC_ERR_WORKSPACE: return "workspace missing or too small";
    case BC_ERR_HIP: return "HIP call or kernel launch failed";
    default: return "unknown status";
  }
}

extern "C" int32_t bc_version(void) { return 100; }
