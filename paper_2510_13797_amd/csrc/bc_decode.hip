// bc_decode_attn: single-token grouped-query attention over the ragged compressed cache
// (Sec. 2 and Sec. 3.1 of the paper: standard attention over whatever is resident).
//
// Split-K flash decoding.  Work item = (sequence, KV head) pair x chunk of R rows; grid =
// (max chunks, pairs), workgroups whose chunk lies beyond L exit at once.  Inside a
// workgroup of 4 waves every global load instruction of a wave reads 1 KB of consecutive
// bytes (RPI whole rows); the LPR lanes that share a row each hold 16 bytes of it, so a
// lane owns EPL head-dim elements of q, K, V and of the accumulator for all G query
// heads of the group.  Scores are completed by a DPP all-reduce over the LPR lanes; the
// softmax is kept online per lane group with one rescale per U rows.  Lane groups,
// waves and finally chunks are merged in a fixed order (the last chunk to finish, found
// by a ticket counter, merges the chunk partials), so results are bit-reproducible.
#include "bc_common.h"

namespace bc {

struct DecodeParams {
  const char* k_slab;
  const char* v_slab;
  const int64_t* base;
  const int32_t* cap;
  const int32_t* P;
  const int32_t* nb;
  const int32_t* w;
  int32_t* err;
  const char* q;
  float* out;
  const uint8_t* active;
  int32_t* counters;   // [pairs] tickets, zero between launches
  float* part_o;       // [pairs][max_chunks][G][D]
  float* part_ml;      // [pairs][max_chunks][2][G]
  int32_t Hq, Hkv, g;  // g = real group size (<= G)
  int32_t rows_per_wg; // R, multiple of the rows one pass covers
  int32_t max_chunks;
  float qscale;        // softmax scale * log2(e)
};

constexpr int kWaves = 4;

template <typename T, int D, int G, int U>
__global__ __launch_bounds__(256) void decode_kernel(DecodeParams p) {
  constexpr int ES = Elem<T>::size;
  constexpr int EPL = Elem<T>::per16;   // elements per lane per row
  constexpr int LPR = D / EPL;          // lanes per row
  constexpr int RPI = 64 / LPR;         // rows per wave load instruction
  constexpr int RB = D * ES;            // row bytes
  constexpr int ROWS_PER_PASS = kWaves * RPI * U;

  const int pair = blockIdx.y;
  const int s = pair / p.Hkv, kvh = pair - s * p.Hkv;
  if (p.active && !p.active[s]) return;
  const int L = p.P[s] + p.nb[s] + p.w[s];
  if (L <= 0) {
    if (blockIdx.x == 0 && kvh == 0 && threadIdx.x == 0) atomicOr(p.err, BC_ERRBIT_STATE);
    return;
  }
  const int R = p.rows_per_wg;
  const int nchunks = (L + R - 1) / R;
  const int chunk = blockIdx.x;
  if (chunk >= nchunks) return;
  const int row0 = chunk * R;
  const int row_end = min(L, row0 + R);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane / LPR, ls = lane - lr * LPR;
  const int cap = p.cap[s];
  const int64_t stream_off = (p.base[s] * p.Hkv + (int64_t)kvh * cap) * RB + ls * 16;
  const char* kbase = p.k_slab + stream_off;
  const char* vbase = p.v_slab + stream_off;

  // q slice of every head of the group, pre-scaled so that exp() becomes exp2()
  float qf[G][EPL];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    if (h < p.g) {
      const uint4 r = *reinterpret_cast<const uint4*>(
          p.q + ((int64_t)(s * p.Hq + kvh * p.g + h) * D) * ES + ls * 16);
      unpack16(r, qf[h], T{});
#pragma unroll
      for (int e = 0; e < EPL; ++e) qf[h][e] *= p.qscale;
    } else {
#pragma unroll
      for (int e = 0; e < EPL; ++e) qf[h][e] = 0.f;
    }
  }

  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = kNegBig; l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
  }

  for (int pr = row0 + wave * (RPI * U); pr < row_end; pr += ROWS_PER_PASS) {
    uint4 kk[U], vv[U];
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = pr + u * RPI + lr;
      valid[u] = r < row_end;
      const int rc = valid[u] ? r : (L - 1);         // stay inside the resident rows
      kk[u] = *reinterpret_cast<const uint4*>(kbase + (int64_t)rc * RB);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = pr + u * RPI + lr;
      const int rc = valid[u] ? r : (L - 1);
      vv[u] = *reinterpret_cast<const uint4*>(vbase + (int64_t)rc * RB);
    }
    float sc[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      unpack16(kk[u], kf, T{});
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float a = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) a = fmaf(qf[h][e], kf[e], a);
        a = group_allreduce_sum<LPR>(a);
        sc[u][h] = valid[u] ? a : kNegBig;
      }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mn = m[h];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, sc[u][h]);
      const float alpha = exp2f(m[h] - mn);
      m[h] = mn;
      l[h] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[h][e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float pw = valid[u] ? exp2f(sc[u][h] - mn) : 0.f;
        sc[u][h] = pw;
        l[h] += pw;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPL];
      unpack16(vv[u], vf, T{});
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(sc[u][h], vf[e], acc[h][e]);
    }
  }

  // merge the RPI lane groups of a wave (fixed butterfly order)
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float mo = __shfl_xor(m[h], off, 64);
      const float lo = __shfl_xor(l[h], off, 64);
      const float mn = fmaxf(m[h], mo);
      const float a = exp2f(m[h] - mn), b = exp2f(mo - mn);
      m[h] = mn;
      l[h] = l[h] * a + lo * b;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float ao = __shfl_xor(acc[h][e], off, 64);
        acc[h][e] = acc[h][e] * a + ao * b;
      }
    }
  }

  __shared__ float s_acc[kWaves][G][D];
  __shared__ float s_m[kWaves][G], s_l[kWaves][G];
  __shared__ int s_ticket;
  if (lr == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_acc[wave][h][ls * EPL + e] = acc[h][e];
      if (ls == 0) { s_m[wave][h] = m[h]; s_l[wave][h] = l[h]; }
    }
  }
  __syncthreads();

  // merge the waves: one output element (head, x) per thread per iteration
  const int nout = p.g * D;
  float* po = p.part_o + ((int64_t)pair * p.max_chunks + chunk) * (G * D);
  float* pml = p.part_ml + ((int64_t)pair * p.max_chunks + chunk) * (2 * G);
  float* outp = p.out + (int64_t)(s * p.Hq + kvh * p.g) * D;
  for (int i = tid; i < nout; i += 256) {
    const int h = i / D, x = i - h * D;
    float mx = s_m[0][h];
#pragma unroll
    for (int wv = 1; wv < kWaves; ++wv) mx = fmaxf(mx, s_m[wv][h]);
    float lsum = 0.f, o = 0.f;
#pragma unroll
    for (int wv = 0; wv < kWaves; ++wv) {
      const float a = exp2f(s_m[wv][h] - mx);
      lsum += s_l[wv][h] * a;
      o += s_acc[wv][h][x] * a;
    }
    if (nchunks == 1) {
      outp[i] = o / lsum;
    } else {
      po[i] = o;
      if (x == 0) { pml[h] = mx; pml[G + h] = lsum; }
    }
  }
  if (nchunks == 1) return;

  // publish the partial, take a ticket; the last chunk of the pair merges all of them
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    s_ticket = atomicAdd(p.counters + pair, 1);
  }
  __syncthreads();
  if (s_ticket != nchunks - 1) return;
  if (tid == 0) p.counters[pair] = 0;       // ready for the next launch
  __threadfence();
  const float* ao = p.part_o + (int64_t)pair * p.max_chunks * (G * D);
  const float* aml = p.part_ml + (int64_t)pair * p.max_chunks * (2 * G);
  for (int i = tid; i < nout; i += 256) {
    const int h = i / D;
    float mx = kNegBig;
    for (int ch = 0; ch < nchunks; ++ch) mx = fmaxf(mx, aml[ch * 2 * G + h]);
    float lsum = 0.f, o = 0.f;
    for (int ch = 0; ch < nchunks; ++ch) {
      const float a = exp2f(aml[ch * 2 * G + h] - mx);
      lsum += aml[ch * 2 * G + G + h] * a;
      o += ao[(int64_t)ch * (G * D) + i] * a;
    }
    outp[i] = o / lsum;
  }
}

static int g_rows_per_wg = 0;
static int g_variant = 0;

struct DecodePlan {
  int G;              // padded group size of the instantiated kernel
  int rows_per_pass;  // rows one pass of a workgroup covers
  int R;              // rows per workgroup
  int max_chunks;
  size_t counters_bytes, part_o_bytes, part_ml_bytes;
};

static int padded_group(int g) { return g <= 1 ? 1 : g <= 2 ? 2 : g <= 4 ? 4 : g <= 6 ? 6 : 8; }

static DecodePlan make_plan(const bc_shape* sh, int max_cap) {
  DecodePlan pl;
  pl.G = padded_group(sh->Hq / sh->Hkv);
  const int epl = 16 / elem_size(sh->kv_dtype);
  const int lpr = sh->d / epl, rpi = 64 / lpr;
  const int U = 8;
  pl.rows_per_pass = kWaves * rpi * U;
  int R = g_rows_per_wg > 0 ? g_rows_per_wg : pl.rows_per_pass;
  R = ((R + pl.rows_per_pass - 1) / pl.rows_per_pass) * pl.rows_per_pass;
  // keep the number of chunk partials per pair bounded for long uncompressed caches
  while ((max_cap + R - 1) / R > 64) R += pl.rows_per_pass;
  pl.R = R;
  pl.max_chunks = (max_cap + R - 1) / R;
  const size_t pairs = (size_t)sh->B * sh->Hkv;
  pl.counters_bytes = ((pairs * 4 + 255) / 256) * 256;
  pl.part_o_bytes = pairs * pl.max_chunks * pl.G * sh->d * 4;
  pl.part_ml_bytes = pairs * pl.max_chunks * 2 * pl.G * 4;
  return pl;
}

template <typename T, int D>
static void launch_decode(const DecodeParams& p, int G, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: decode_kernel<T, D, 1, 8><<<grid, 256, 0, st>>>(p); break;
    case 2: decode_kernel<T, D, 2, 8><<<grid, 256, 0, st>>>(p); break;
    case 4: decode_kernel<T, D, 4, 8><<<grid, 256, 0, st>>>(p); break;
    case 6: decode_kernel<T, D, 6, 8><<<grid, 256, 0, st>>>(p); break;
    default: decode_kernel<T, D, 8, 8><<<grid, 256, 0, st>>>(p); break;
  }
}

}  // namespace bc

using namespace bc;

extern "C" void bc_set_decode_tuning(int32_t rows_per_workgroup, int32_t variant) {
  g_rows_per_wg = rows_per_workgroup > 0 ? rows_per_workgroup : 0;
  g_variant = variant;
}

extern "C" size_t bc_decode_workspace_bytes(const bc_shape* shape, int32_t max_cap) {
  if (check_shape(shape) != BC_OK || max_cap < 1) return 0;
  // sized for the smallest chunk any tuning can select, so a tuning change never outgrows it
  const int saved = g_rows_per_wg;
  g_rows_per_wg = 0;
  const DecodePlan pl = make_plan(shape, max_cap);
  g_rows_per_wg = saved;
  return pl.counters_bytes + pl.part_o_bytes + pl.part_ml_bytes;
}

extern "C" int32_t bc_decode_attn(const bc_shape* shape, const bc_cache* cache, const void* q,
                                  float* out, const uint8_t* active, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return BC_ERR_ARG;
  const DecodePlan pl = make_plan(shape, cache->max_cap);
  if (!workspace || !aligned16(workspace) ||
      workspace_bytes < pl.counters_bytes + pl.part_o_bytes + pl.part_ml_bytes)
    return BC_ERR_WORKSPACE;

  DecodeParams p;
  p.k_slab = static_cast<const char*>(cache->k_slab);
  p.v_slab = static_cast<const char*>(cache->v_slab);
  p.base = cache->base; p.cap = cache->cap; p.P = cache->P; p.nb = cache->nb; p.w = cache->w;
  p.err = cache->err;
  p.q = static_cast<const char*>(q);
  p.out = out;
  p.active = active;
  char* ws = static_cast<char*>(workspace);
  p.counters = reinterpret_cast<int32_t*>(ws);
  p.part_o = reinterpret_cast<float*>(ws + pl.counters_bytes);
  p.part_ml = reinterpret_cast<float*>(ws + pl.counters_bytes + pl.part_o_bytes);
  p.Hq = shape->Hq; p.Hkv = shape->Hkv; p.g = shape->Hq / shape->Hkv;
  p.rows_per_wg = pl.R;
  p.max_chunks = pl.max_chunks;
  p.qscale = shape->scale * kLog2e;

  const dim3 grid(pl.max_chunks, shape->B * shape->Hkv);
  hipStream_t hs = as_stream(stream);
  if (shape->kv_dtype == BC_BF16) {
    if (shape->d == 128) launch_decode<bf16_t, 128>(p, pl.G, grid, hs);
    else launch_decode<bf16_t, 64>(p, pl.G, grid, hs);
  } else {
    if (shape->d == 128) launch_decode<float, 128>(p, pl.G, grid, hs);
    else launch_decode<float, 64>(p, pl.G, grid, hs);
  }
  return launch_status();
}

extern "C" int32_t bc_decode_step(const bc_shape* shape, const bc_cache* cache, const void* k,
                                  const void* v, const void* q, float* out, const void* beacon_k,
                                  const void* beacon_v, const uint8_t* active, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  int32_t st = bc_append_kv(shape, cache, k, v, active, BC_ROW_TOKEN, stream);
  if (st != BC_OK) return st;
  st = bc_decode_attn(shape, cache, q, out, active, workspace, workspace_bytes, stream);
  if (st != BC_OK) return st;
  if (beacon_k || beacon_v)
    st = bc_compress_evict(shape, cache, beacon_k, beacon_v, active, 1, stream);
  return st;
}
