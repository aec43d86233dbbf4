// bc_prefill_attn_bwd: gradients of the beacon-masked prefill attention (Fig. 2, Sec. 3.2 of the
// paper: training runs the masked forward in parallel and differentiates through it).
//
// With S = scale*Q.K^T on the visible pairs, A = softmax(S), O = A.V and upstream dO:
//   Delta_r = sum_x dO[r,x]*O[r,x]        dV = A^T.dO        dA = dO.V^T
//   dS = A*(dA - Delta)                   dQ = scale*dS.K    dK = scale*dS^T.Q
// A is recomputed from the saved log-sum-exp.  Two kernels, both on the compacted structure of
// the mask, no atomics (results are reproducible), plus a small fixed-order reduction:
//
//  dq kernel   one workgroup = 64 query rows x 2 query heads, walking the same key list as the
//              forward kernel (prompt run, gathered beacon run, masked band).  Also writes
//              (lse*log2e, Delta) per row, head-major, for the second kernel.
//  dkv kernel  one workgroup = 64 keys of one KV head; three kinds of key block:
//                prompt keys      -> stream every later row of every head of the group (dense)
//                gathered beacons -> the same, from the first beacon's row on (dense)
//                response tokens  -> only the rows up to the end of their window (masked band)
//              so the dense part of the work is spent on the ~P + S/(c+1) keys every row sees.
//              A dense block is long (every later row x every head); it is cut in two by query
//              heads, the halves write partial dK/dV to the workspace and a third kernel adds
//              them in a fixed order.  Response blocks store their result directly.
//
// All contractions are 16x16x32 bf16 MFMA; A and dS are split into two bf16 parts before they
// enter a product (their rounding would otherwise dominate the error); tiles of 32 rows are
// gathered into LDS by 16-byte LDS-DMA loads (3-stage ring, one barrier per tile).
#include "bc_common.h"

namespace bc {

constexpr int kBwWaves = 4;
constexpr int kBwBM = 64;                 // rows (dq kernel) or keys (dkv kernel) per workgroup
constexpr int kBwBN = 32;                 // streamed entries per tile
constexpr int kBwStages = 3;
constexpr int kBwStatLds = kBwStages * 256;          // per-row statistics of the staged tiles (dkv kernel)
// What follows from the head dimension D (128 or 64): rows of 256 or 128 bytes.
template <int D> struct BwDims {
  static constexpr int ROWB = D * 2;                 // bytes of a row of one head
  static constexpr int UPR = ROWB / 16;              // 16-byte units per row
  static constexpr int KS = D / 32;                  // k-steps of a product over the head dimension
  static constexpr int NJ = D / 16;                  // 16-column blocks of a gradient tile
  static constexpr int TILE = kBwBN * ROWB;          // bytes of one staged tile
  static constexpr int RPI = 1024 / ROWB;            // rows per LDS-DMA instruction
  static constexpr int NLD = kBwBN / (RPI * kBwWaves);   // instructions per wave, tile and tensor
  static constexpr int LDS = kBwStages * 2 * TILE;   // 48 or 24 KB; the epilogues need 4 x 16 x D floats
  static_assert(LDS >= kBwWaves * 16 * D * 4, "the gradient tiles fit the ring's LDS");
};

typedef __attribute__((address_space(3))) void bw_lds_void_t;
typedef __attribute__((address_space(1))) const void bw_global_void_t;
typedef __attribute__((ext_vector_type(4))) short bw_s16x4_t;
typedef __attribute__((ext_vector_type(8))) short bw_s16x8_t;
typedef __attribute__((address_space(3))) bw_s16x4_t bw_lds_s16x4_t;
typedef __attribute__((ext_vector_type(2))) float bw_f32x2_t;

struct BwdParams {
  const char* q;
  const char* k;
  const char* v;
  const float* out;
  const float* lse;
  const char* dout;
  const int64_t* row_off;
  const int32_t* P;
  const int32_t* c;
  float* dq;
  float* dk;
  float* dv;
  float* stat;          // [Hq][total_rows][2]: lse*log2(e), Delta
  float* part;          // [hsplit][2][total_rows][Hkv][D]: dk, dv partials of the dense key blocks
  int32_t D;            // head dimension (the reduction kernel reads it; the others are templates)
  int32_t hsplit;       // head splits of a dense key block (1: none), heads per split = ceil(g / hsplit)
  int64_t total_rows;
  int32_t Hq, Hkv, g;
  int32_t npairs;       // (trajectory, KV head) pairs
  int32_t pstride;      // npairs rounded up to a multiple of 8
  float scale;
  float qscale;         // scale * log2(e)
};

__device__ __forceinline__ uint32_t bw_pack(float a, float b) {       // two floats -> bf16x2, RNE
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(bw_f32x2_t{a, b}, bf16x2_t));
}

// 8 floats (consecutive k indices) -> hi and lo bf16x8 operands with hi + lo ~ x to 16 bits
__device__ __forceinline__ void bw_split(const float (&x)[8], bf16x8_t& hi, bf16x8_t& lo,
                                         const HalfSelectors& sel) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const uint32_t hp = bw_pack(x[e], x[e + 1]);
    h[e >> 1] = hp;
    l[e >> 1] = bw_pack(minus_half(x[e], hp, sel.low), minus_half(x[e + 1], hp, sel.high));
  }
  hi = __builtin_bit_cast(bf16x8_t, make_uint4(h[0], h[1], h[2], h[3]));
  lo = __builtin_bit_cast(bf16x8_t, make_uint4(l[0], l[1], l[2], l[3]));
}

// A operand "rows of the tile": lane (m = lane&15, kb = lane>>4) of sub-tile t reads tile entry
// 8*(m/4) + 4*t + m%4, head-dim bytes 64*i + 16*kb (tile is row-major, 16-byte units swizzled)
template <int D>
__device__ __forceinline__ bf16x8_t bw_rows_operand(const char* tile, int t, int i, int n, int kb) {
  const int row = ((n >> 2) << 3) + 4 * t + (n & 3);
  return *reinterpret_cast<const bf16x8_t*>(tile + row * (2 * D) + (((4 * i + kb) ^ tile_swz<D>(row)) << 4));
}

// A operand "tile transposed": M = 16 head-dim columns 16*j .., K = the 32 tile entries
template <int D>
__device__ __forceinline__ bf16x8_t bw_cols_operand(const char* tile, int j, int lane) {
  const int rl = lane & 15, kb = lane >> 4;
  const int rowa = 8 * kb + (rl >> 2), rowb = rowa + 4;
  const int sub = (rl & 1) << 3;
  const int u = 2 * j + ((rl & 3) >> 1);
  const bw_s16x4_t a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (bw_lds_s16x4_t*)(tile + rowa * (2 * D) + ((u ^ tile_swz<D>(rowa)) << 4) + sub));
  const bw_s16x4_t a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (bw_lds_s16x4_t*)(tile + rowb * (2 * D) + ((u ^ tile_swz<D>(rowb)) << 4) + sub));
  return __builtin_bit_cast(bf16x8_t, (bw_s16x8_t)__builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7));
}

// [16 entries][D] fp32 accumulators of one wave (accumulator layout: lane (n, kb) holds
// columns 16*j + 4*kb .. +3 of entry n) -> LDS -> one burst of D floats per entry.
// dst_row(t) returns the destination pointer of entry t or nullptr.
template <int D, typename F>
__device__ __forceinline__ void bw_store_tile(float* my, const f32x4_t (&acc)[D / 16], float mul, int lane,
                                              F dst_row) {
  constexpr int OLPR = D / 4;                 // lanes that cover one row, 16 bytes each
  constexpr int ORPP = 64 / OLPR;             // rows per pass
  const int n = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int j = 0; j < D / 16; ++j)
    *reinterpret_cast<f32x4_t*>(my + n * D + (((4 * j + kb) ^ n) << 2)) = acc[j] * mul;
#pragma unroll
  for (int pass = 0; pass < 16 / ORPP; ++pass) {
    const int t = ORPP * pass + lane / OLPR, unit = lane & (OLPR - 1);
    const f32x4_t val = *reinterpret_cast<const f32x4_t*>(my + t * D + ((unit ^ t) << 2));
    float* dst = dst_row(t);
    if (dst) __builtin_nontemporal_store(val, reinterpret_cast<f32x4_t*>(dst + unit * 4));   // written once
  }
}

// ---------------------------------------------------------------------------
// dq kernel
// ---------------------------------------------------------------------------
constexpr int kDqHeads = 2;      // query heads per workgroup

template <int D>
__global__ __launch_bounds__(kBwWaves * 64, 2) void prefill_bwd_dq_kernel(BwdParams p) {
  using Dm = BwDims<D>;
  constexpr int ROWB = Dm::ROWB, UPR = Dm::UPR, KS = Dm::KS, NJ = Dm::NJ, kBwTile = Dm::TILE, RPI = Dm::RPI,
                NLD = Dm::NLD;
  __shared__ __attribute__((aligned(1024))) char lds[Dm::LDS];
  // grid: x = (head pair, trajectory, KV head), y = query tile, longest tiles of every
  // trajectory first (workgroups are dispatched x-fastest)
  // (the head pairs of one (trajectory, KV head) are `pstride` workgroups apart, a multiple of 8:
  // workgroups go to the XCDs in turn, so the workgroups that read the same K/V tiles share an L2)
  const int hh = blockIdx.x / p.pstride, pair = blockIdx.x - hh * p.pstride;
  if (pair >= p.npairs) return;
  const int kvh = pair % p.Hkv, b = pair / p.Hkv;
  const int64_t off0 = p.row_off[b];
  const int S = (int)(p.row_off[b + 1] - off0);
  const int qt = gridDim.y - 1 - blockIdx.y;
  const int r0 = qt * kBwBM;
  if (r0 >= S) return;
  const int r1 = min(r0 + kBwBM - 1, S - 1);
  const int P = p.P[b];
  const WindowStride ws = window_stride(p.c[b], S);
  const int c = ws.c, cp1 = ws.stride;

  int nA = 0, nB = 0, band_start = 0;
  if (c > 0 && r0 >= P) {
    const int m0 = (int)window_of(ws, (uint32_t)(r0 - P));
    nA = P; nB = m0; band_start = P + m0 * cp1;
  }
  const int nC = r1 - band_start + 1;
  const int TA = (nA + kBwBN - 1) / kBwBN, TB = (nB + kBwBN - 1) / kBwBN;
  const int NT = TA + TB + (nC + kBwBN - 1) / kBwBN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const HalfSelectors sel = half_selectors();
  const int n = lane & 15, kb = lane >> 4;
  const int64_t kv_row_bytes = (int64_t)p.Hkv * ROWB;
  const char* kbase = p.k + (off0 * p.Hkv + kvh) * ROWB;
  const char* vbase = p.v + (off0 * p.Hkv + kvh) * ROWB;

  struct TileDesc { int j0, step, nvalid; bool predicate; };
  auto tile_desc = [&](int kt) -> TileDesc {
    TileDesc t;
    if (kt < TA) { t.j0 = kt * kBwBN; t.step = 1; t.nvalid = nA - kt * kBwBN; t.predicate = false; }
    else if (kt < TA + TB) {
      const int m = (kt - TA) * kBwBN;
      t.j0 = P + m * cp1 + c; t.step = cp1; t.nvalid = nB - m; t.predicate = false;
    } else {
      const int x = (kt - TA - TB) * kBwBN;
      t.j0 = band_start + x; t.step = 1; t.nvalid = nC - x; t.predicate = true;
    }
    t.nvalid = min(t.nvalid, kBwBN);
    return t;
  };
  const int ld_rr = RPI * wave + lane / UPR;
  auto issue_tile = [&](int kt, int stage) {
    const TileDesc t = tile_desc(kt);
#pragma unroll
    for (int half = 0; half < NLD; ++half) {
      const int rr = ld_rr + RPI * kBwWaves * half;
      const int j = rr < t.nvalid ? t.j0 + rr * t.step : r1;
      const int64_t goff = (int64_t)j * kv_row_bytes + (((lane & (UPR - 1)) ^ tile_swz<D>(rr)) << 4);
      char* dst = lds + stage * (2 * kBwTile) + (wave + kBwWaves * half) * 1024;
      __builtin_amdgcn_global_load_lds((bw_global_void_t*)(kbase + goff), (bw_lds_void_t*)dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((bw_global_void_t*)(vbase + goff),
                                       (bw_lds_void_t*)(dst + kBwTile), 16, 0, 0);
    }
  };
  issue_tile(0, 0);
  if (NT > 1) issue_tile(1, 1);

  // this lane's query row; Q^T and dO^T as B operands; log-sum-exp and Delta of the row
  const int r = r0 + 16 * wave + n;
  const bool row_ok = r <= r1;
  const bool full_rows = r0 + kBwBM - 1 <= r1;
  const int rq = row_ok ? r : r1;
  bf16x8_t qb[kDqHeads][KS], dob[kDqHeads][KS];
  float lse2[kDqHeads], delta[kDqHeads];
#pragma unroll
  for (int h = 0; h < kDqHeads; ++h) {
    const int head = hh * kDqHeads + h;
    const bool head_ok = head < p.g;
    const int64_t rh = (off0 + rq) * p.Hq + kvh * p.g + (head_ok ? head : 0);
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      uint4 x = make_uint4(0u, 0u, 0u, 0u), y = make_uint4(0u, 0u, 0u, 0u);
      if (head_ok) {
        x = *reinterpret_cast<const uint4*>(p.q + (rh * D + 32 * i + 8 * kb) * 2);
        y = *reinterpret_cast<const uint4*>(p.dout + (rh * D + 32 * i + 8 * kb) * 2);
        const float4 o0 = *reinterpret_cast<const float4*>(p.out + rh * D + 32 * i + 8 * kb);
        const float4 o1 = *reinterpret_cast<const float4*>(p.out + rh * D + 32 * i + 8 * kb + 4);
        float dy[8];
        unpack16(y, dy, bf16_t{});
        part += dy[0] * o0.x + dy[1] * o0.y + dy[2] * o0.z + dy[3] * o0.w +
                dy[4] * o1.x + dy[5] * o1.y + dy[6] * o1.z + dy[7] * o1.w;
      }
      qb[h][i] = __builtin_bit_cast(bf16x8_t, x);
      dob[h][i] = __builtin_bit_cast(bf16x8_t, y);
    }
    part = rows_allreduce_sum(part);
    delta[h] = part;
    lse2[h] = head_ok ? p.lse[rh] * kLog2e : 0.f;
    if (head_ok && row_ok && kb == 0) {
      float* st = p.stat + ((int64_t)(kvh * p.g + head) * p.total_rows + off0 + r) * 2;
      st[0] = lse2[h];
      st[1] = delta[h];
    }
  }
  const int win_r = (c > 0 && r >= P) ? (int)window_of(ws, (uint32_t)(r - P)) : -1;

  f32x4_t dQ[kDqHeads][NJ];
#pragma unroll
  for (int h = 0; h < kDqHeads; ++h)
#pragma unroll
    for (int j = 0; j < NJ; ++j) dQ[h][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  int stage = 0;
  for (int kt = 0; kt < NT; ++kt) {
    if (kt + 1 < NT) wait_vmcnt<2 * NLD>();
    else wait_vmcnt<0>();
    __syncthreads();
    if (kt + 2 < NT) issue_tile(kt + 2, stage >= 1 ? stage - 1 : kBwStages - 1);
    const char* tk = lds + stage * (2 * kBwTile);
    const char* tv = tk + kBwTile;
    stage = stage + 1 == kBwStages ? 0 : stage + 1;
    const TileDesc td = tile_desc(kt);
    // a band tile that starts behind the last of this wave's 16 rows holds nothing they may see
    if (td.predicate && td.j0 > r0 + 16 * wave + 15) continue;

    // a full tile of the prompt or beacon run under a full query tile needs no per-key tests
    // (uniform over the workgroup: skipped by a scalar branch)
    const bool MASKED = td.predicate || td.nvalid < kBwBN || !full_rows;
    bool vis[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vis[e] = true;
    if (MASKED) {
      const int lim = row_ok ? td.nvalid - 8 * kb : 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) vis[e] = e < lim;
      if (td.predicate) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int j = td.j0 + 8 * kb + e;
          bool see = j < P || c <= 0;
          if (!see) {
            const uint32_t u = (uint32_t)(j - P);
            const uint32_t qd = window_of(ws, u);
            see = (int)(u - qd * (uint32_t)cp1) == c || (int)qd == win_r;
          }
          vis[e] = vis[e] && j <= r && see;
        }
      }
    }

    bf16x8_t dshi[kDqHeads], dslo[kDqHeads];
    // scores and dA of both heads first: the K and V operands are read once, and the eight
    // accumulation chains are independent
    f32x4_t Sx[kDqHeads][2], dPx[kDqHeads][2];
#pragma unroll
    for (int h = 0; h < kDqHeads; ++h)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        Sx[h][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        dPx[h][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        const bf16x8_t ka = bw_rows_operand<D>(tk, t, i, n, kb), va = bw_rows_operand<D>(tv, t, i, n, kb);
#pragma unroll
        for (int h = 0; h < kDqHeads; ++h) {
          Sx[h][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qb[h][i], Sx[h][t], 0, 0, 0);
          dPx[h][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, dob[h][i], dPx[h][t], 0, 0, 0);
        }
      }
#pragma unroll
    for (int h = 0; h < kDqHeads; ++h) {
      float ds[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float a = fast_exp2(fmaf(Sx[h][e >> 2][e & 3], p.qscale, -lse2[h]));
        ds[e] = a * (dPx[h][e >> 2][e & 3] - delta[h]);
      }
      if (MASKED) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ds[e] = vis[e] ? ds[e] : 0.f;
      }
      bw_split(ds, dshi[h], dslo[h], sel);
    }
    // dQ^T += K^T . dS^T
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const bf16x8_t kt_op = bw_cols_operand<D>(tk, j, lane);
#pragma unroll
      for (int h = 0; h < kDqHeads; ++h) {
        dQ[h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kt_op, dshi[h], dQ[h][j], 0, 0, 0);
        dQ[h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kt_op, dslo[h], dQ[h][j], 0, 0, 0);
      }
    }
  }
  __syncthreads();

  float* my = reinterpret_cast<float*>(lds + wave * (16 * D * 4));
#pragma unroll
  for (int h = 0; h < kDqHeads; ++h) {
    const int head = hh * kDqHeads + h;
    if (head >= p.g) continue;
    bw_store_tile<D>(my, dQ[h], p.scale, lane, [&](int t) -> float* {
      const int rr = r0 + 16 * wave + t;
      return rr <= r1 ? p.dq + ((off0 + rr) * p.Hq + kvh * p.g + head) * D : nullptr;
    });
  }
}

// ---------------------------------------------------------------------------
// dkv kernel
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBwWaves * 64, 2) void prefill_bwd_dkv_kernel(BwdParams p) {
  using Dm = BwDims<D>;
  constexpr int ROWB = Dm::ROWB, UPR = Dm::UPR, KS = Dm::KS, NJ = Dm::NJ, kBwTile = Dm::TILE, RPI = Dm::RPI,
                NLD = Dm::NLD, kBwLds = Dm::LDS;
  __shared__ __attribute__((aligned(1024))) char lds[kBwLds + kBwStatLds];
  // grid: x = (trajectory, KV head), y = key block; the long dense blocks of every trajectory
  // are dispatched before any short one
  if ((int)blockIdx.x >= p.npairs) return;      // the grid's x extent is padded to a multiple of 8 (XCD count)
  const int kvh = blockIdx.x % p.Hkv, b = blockIdx.x / p.Hkv;
  const int64_t off0 = p.row_off[b];
  const int S = (int)(p.row_off[b + 1] - off0);
  const int P0 = p.P[b];
  const WindowStride ws = window_stride(p.c[b], S);
  const int c = ws.c, cp1 = ws.stride;
  // key blocks of this (trajectory, KV head): prompt keys | gathered beacons | response rows.
  // Without compression every row behaves like a prompt row (plain causal).
  const int Pk = c > 0 ? min(P0, S) : S;                        // keys treated as dense-causal
  const int nresp = S - Pk;                                     // response rows (tokens and beacons)
  const int nbeac = c > 0 ? (int)window_of(ws, (uint32_t)nresp) : 0;   // complete windows
  const int NPB = (Pk + kBwBM - 1) / kBwBM, NBB = (nbeac + kBwBM - 1) / kBwBM;
  const int NLB = (nresp + kBwBM - 1) / kBwBM;
  // The dense blocks (prompt keys, beacons) stream every later row of every head; each is cut
  // into `hsplit` workgroups by query heads, whose partial sums a second kernel adds in a fixed
  // order.  The short response blocks take all heads and store their result directly.
  const int nd = NPB + NBB;
  int blk, h_begin = 0, h_end = p.g, split = -1;
  if ((int)blockIdx.y < nd * p.hsplit) {
    blk = blockIdx.y / p.hsplit;
    if (p.hsplit > 1) {
      split = blockIdx.y - blk * p.hsplit;
      const int hps = (p.g + p.hsplit - 1) / p.hsplit;
      h_begin = split * hps; h_end = min(p.g, h_begin + hps);
    }
  } else {
    blk = nd + ((int)blockIdx.y - nd * p.hsplit);
  }
  if (blk >= nd + NLB) return;
  const int kind = blk < NPB ? 0 : blk < NPB + NBB ? 1 : 2;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const HalfSelectors sel = half_selectors();
  const int n = lane & 15, kb = lane >> 4;

  // this lane's key (column n of the wave's 16 keys) and the row range the block streams
  int jkey;            // row of the key
  bool key_ok;
  int rs, re;          // first and last streamed row
  if (kind == 0) {
    const int j0 = blk * kBwBM;
    jkey = j0 + 16 * wave + n; key_ok = jkey < Pk;
    rs = j0; re = S - 1;
  } else if (kind == 1) {
    const int m0 = (blk - NPB) * kBwBM;
    const int m = m0 + 16 * wave + n;
    key_ok = m < nbeac; jkey = Pk + m * cp1 + c;
    rs = Pk + m0 * cp1 + c; re = S - 1;
  } else {
    const int j0 = Pk + (blk - NPB - NBB) * kBwBM;
    jkey = j0 + 16 * wave + n; key_ok = jkey < S;
    if (key_ok) {                              // beacon rows belong to the beacon blocks
      const uint32_t u = (uint32_t)(jkey - Pk);
      const uint32_t qd = window_of(ws, u);
      if ((int)(u - qd * (uint32_t)cp1) == c) key_ok = false;
    }
    const int jl = min(j0 + kBwBM - 1, S - 1);
    const int wl = (int)window_of(ws, (uint32_t)(jl - Pk));
    rs = j0; re = min(S - 1, Pk + (wl + 1) * cp1 - 1);      // through the closing beacon
  }
  // first row tile of a dense block from which every streamed row sees every key of the block
  // (never, for a block with missing keys or of response tokens)
  int dense_from_rt = 0x7fffffff;
  if (kind == 0 && blk * kBwBM + kBwBM <= Pk) dense_from_rt = kBwBM / kBwBN;
  if (kind == 1 && (blk - NPB) * kBwBM + kBwBM <= nbeac)
    dense_from_rt = ((kBwBM - 1) * cp1 + kBwBN) / kBwBN;
  if (!key_ok) jkey = rs;                      // loads stay in range; contributions are masked
  const int win_j = (c > 0 && jkey >= Pk) ? (int)window_of(ws, (uint32_t)(jkey - Pk)) : -1;
  // the rows this wave's 16 keys can be seen from: [first key, last row of the last key's reach]
  int wave_first_key = __builtin_amdgcn_readfirstlane(jkey);      // (lane 0 holds the smallest key)
  int wave_last_row = !key_ok ? -1 : kind == 2 ? min(re, Pk + (win_j + 1) * cp1 - 1) : re;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) wave_last_row = max(wave_last_row, __shfl_xor(wave_last_row, off, 64));
  wave_last_row = __builtin_amdgcn_readfirstlane(wave_last_row);
  if (wave_last_row < 0) { wave_first_key = rs; wave_last_row = re; }     // no valid key: nothing is skipped (all masked)

  // K^T and V^T of the wave's keys as B operands (column n = key, k = head-dim index)
  bf16x8_t kop[KS], vop[KS];
#pragma unroll
  for (int i = 0; i < KS; ++i) {
    const int64_t e = ((off0 + jkey) * p.Hkv + kvh) * D + 32 * i + 8 * kb;
    kop[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(p.k + e * 2));
    vop[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(p.v + e * 2));
  }

  const int ntile = (re - rs) / kBwBN + 1;     // row tiles per head
  const int NT = ntile * (h_end - h_begin);     // streamed tiles: head-major
  const int ld_rr = RPI * wave + lane / UPR;
  // tiles are issued in order, so the (head, row tile) pair of the next tile to issue is kept
  // in two counters instead of being recovered by a division
  // Row tiles are streamed from the last row of the range backwards: all dense key blocks of a
  // (trajectory, KV head) pair need the rows from the end of the trajectory back to their own
  // keys, start together (they are neighbours in dispatch order, on the same XCD) and so walk the
  // same tiles at the same time - the later readers of a tile find it in the L2.
  int issue_h = h_begin, issue_rt = ntile - 1;
  auto issue_tile = [&](int stage) {
    const int h = issue_h, rt = issue_rt;
    if (--issue_rt < 0) { issue_rt = ntile - 1; ++issue_h; }
#pragma unroll
    for (int half = 0; half < NLD; ++half) {
      const int tr = ld_rr + RPI * kBwWaves * half;           // entry of the tile
      const int rr = min(rs + rt * kBwBN + tr, S - 1);
      const int64_t goff = ((off0 + rr) * p.Hq + kvh * p.g + h) * ROWB + (((lane & (UPR - 1)) ^ tile_swz<D>(tr)) << 4);
      char* dst = lds + stage * (2 * kBwTile) + (wave + kBwWaves * half) * 1024;
      __builtin_amdgcn_global_load_lds((bw_global_void_t*)(p.q + goff), (bw_lds_void_t*)dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((bw_global_void_t*)(p.dout + goff),
                                       (bw_lds_void_t*)(dst + kBwTile), 16, 0, 0);
    }
    if (wave == 0) {
      // (lse*log2e, Delta) of the tile's 32 rows: 64 floats, one 4-byte LDS-DMA load per lane
      const int rr = min(rs + rt * kBwBN + (lane >> 1), S - 1);
      const float* sp = p.stat + ((int64_t)(kvh * p.g + h) * p.total_rows + off0 + rr) * 2 + (lane & 1);
      __builtin_amdgcn_global_load_lds((bw_global_void_t*)sp,
                                       (bw_lds_void_t*)(lds + kBwLds + stage * 256), 4, 0, 0);
    }
  };
  issue_tile(0);
  if (NT > 1) issue_tile(1);

  f32x4_t dK[NJ], dV[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) { dK[j] = f32x4_t{0.f, 0.f, 0.f, 0.f}; dV[j] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }

  int stage = 0, cur_rt = ntile - 1;
  for (int it = 0; it < NT; ++it) {
    if (it + 1 >= NT) wait_vmcnt<0>();
    else if (wave == 0) wait_vmcnt<2 * NLD + 1>();     // one more load per tile
    else wait_vmcnt<2 * NLD>();
    __syncthreads();
    if (it + 2 < NT) issue_tile(stage >= 1 ? stage - 1 : kBwStages - 1);
    const char* tq = lds + stage * (2 * kBwTile);
    const char* tdo = tq + kBwTile;
    const float* tstat = reinterpret_cast<const float*>(lds + kBwLds + stage * 256);
    stage = stage + 1 == kBwStages ? 0 : stage + 1;
    const int rt = cur_rt;
    if (--cur_rt < 0) cur_rt = ntile - 1;
    // a row tile that ends in front of this wave's first key, or starts behind the last row any
    // of its keys is seen from (the end of a response token's window), adds nothing here
    if (rs + rt * kBwBN + kBwBN - 1 < wave_first_key || rs + rt * kBwBN > wave_last_row) continue;
    const int row0 = rs + rt * kBwBN + 8 * kb;          // this lane's 8 rows: row0 + e

    // per-row statistics of this lane's rows (head-major, 8 rows = 64 contiguous bytes)
    float st[16];
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      const f32x4_t x = *reinterpret_cast<const f32x4_t*>(tstat + 16 * kb + 4 * e4);
      st[4 * e4] = x[0]; st[4 * e4 + 1] = x[1]; st[4 * e4 + 2] = x[2]; st[4 * e4 + 3] = x[3];
    }
    // dense blocks: once the streamed rows lie behind every key of the block, nothing is hidden
    const bool MASKED = rt < dense_from_rt || rs + rt * kBwBN + kBwBN - 1 > re;
    bool vis[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vis[e] = true;
    if (MASKED) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int r = row0 + e;
      bool ok = key_ok && r <= re && r >= jkey;
      if (kind == 2 && ok) {
        // a response token is seen inside its own window (the closing beacon included)
        const int wr = (int)window_of(ws, (uint32_t)(r - Pk));
        ok = wr == win_j;
      }
      vis[e] = ok;
    }
    }

    f32x4_t Sx[2], dPx[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      Sx[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      dPx[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        Sx[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bw_rows_operand<D>(tq, t, i, n, kb), kop[i], Sx[t], 0, 0, 0);
        dPx[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bw_rows_operand<D>(tdo, t, i, n, kb), vop[i], dPx[t], 0, 0, 0);
      }
    }
    float a[8], ds[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[e] = fast_exp2(fmaf(Sx[e >> 2][e & 3], p.qscale, -st[2 * e]));
      if (MASKED) a[e] = vis[e] ? a[e] : 0.f;
      ds[e] = a[e] * (dPx[e >> 2][e & 3] - st[2 * e + 1]);
    }
    bf16x8_t ahi, alo, dshi, dslo;
    bw_split(a, ahi, alo, sel);
    bw_split(ds, dshi, dslo, sel);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const bf16x8_t dot = bw_cols_operand<D>(tdo, j, lane);      // dO^T
      dV[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dot, ahi, dV[j], 0, 0, 0);
      dV[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dot, alo, dV[j], 0, 0, 0);
      const bf16x8_t qt_op = bw_cols_operand<D>(tq, j, lane);     // Q^T
      dK[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt_op, dshi, dK[j], 0, 0, 0);
      dK[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt_op, dslo, dK[j], 0, 0, 0);
    }
  }
  __syncthreads();

  // every key row is owned by exactly one lane column of one block: plain stores
  float* my = reinterpret_cast<float*>(lds + wave * (16 * D * 4));
  // key row and validity of entry t of this wave, taken from the lane that owns it
  auto dst_of = [&](float* base, int t) -> float* {
    const int jk = __shfl(jkey, t, 64);
    const int ok = __shfl((int)key_ok, t, 64);
    return ok ? base + ((off0 + jk) * p.Hkv + kvh) * D : nullptr;
  };
  float* dk_base = p.dk;
  float* dv_base = p.dv;
  if (split >= 0) {
    const int64_t plane = p.total_rows * p.Hkv * D;
    dk_base = p.part + (int64_t)(2 * split) * plane;
    dv_base = dk_base + plane;
  }
  bw_store_tile<D>(my, dK, p.scale, lane, [&](int t) { return dst_of(dk_base, t); });
  bw_store_tile<D>(my, dV, 1.0f, lane, [&](int t) { return dst_of(dv_base, t); });
}

// Sum of the head-split partials of the dense keys (prompt rows and beacons), in split order.
// One thread per 16 bytes of one (row, KV head); rows that are not dense were written directly.
__global__ __launch_bounds__(256) void prefill_bwd_reduce_kernel(BwdParams p, int B) {
  const int upr = p.D / 4;                       // 16-byte units of one (row, KV head)
  const int64_t units = p.total_rows * p.Hkv * upr;
  const int64_t plane = p.total_rows * p.Hkv * p.D;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < units;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = i / (p.Hkv * upr);
    int lo = 0, hi = B;                        // largest b with row_off[b] <= row
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.row_off[mid] <= row) lo = mid; else hi = mid;
    }
    const int j = (int)(row - p.row_off[lo]);
    const int P0 = p.P[lo], c = p.c[lo];
    const bool dense = c <= 0 || j < P0 || (j - P0) % (c + 1) == c;
    if (!dense) continue;
    f32x4_t sk = f32x4_t{0.f, 0.f, 0.f, 0.f}, sv = sk;
    for (int sp = 0; sp < p.hsplit; ++sp) {
      sk += *reinterpret_cast<const f32x4_t*>(p.part + (int64_t)(2 * sp) * plane + i * 4);
      sv += *reinterpret_cast<const f32x4_t*>(p.part + (int64_t)(2 * sp + 1) * plane + i * 4);
    }
    *reinterpret_cast<f32x4_t*>(p.dk + i * 4) = sk;
    *reinterpret_cast<f32x4_t*>(p.dv + i * 4) = sv;
  }
}

// head splits of the dense key blocks: two when the group has several heads
static int bwd_head_splits(int g) { return g >= 2 ? 2 : 1; }

}  // namespace bc

using namespace bc;

extern "C" size_t bc_prefill_bwd_workspace_bytes(const bc_shape* shape, int64_t total_rows) {
  if (check_shape(shape) != BC_OK || total_rows < 1) return 0;
  const int g = shape->Hq / shape->Hkv;
  const int hs = bwd_head_splits(g);
  size_t bytes = (size_t)total_rows * shape->Hq * 2 * sizeof(float);
  if (hs > 1) bytes += (size_t)hs * 2 * total_rows * shape->Hkv * shape->d * sizeof(float);
  return bytes;
}

extern "C" int32_t bc_prefill_attn_bwd(const bc_shape* shape, const void* q, const void* k,
                                       const void* v, const float* out, const float* lse,
                                       const void* dout, const int64_t* row_offsets,
                                       const int32_t* P, const int32_t* c, int32_t max_rows,
                                       int64_t total_rows, float* dq, float* dk, float* dv,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  if (shape->kv_dtype != BC_BF16) return BC_ERR_SHAPE;
  if (!q || !k || !v || !out || !lse || !dout || !row_offsets || !P || !c || !dq || !dk || !dv)
    return BC_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(dout) ||
      !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
    return BC_ERR_ARG;
  if (max_rows < 1 || max_rows >= (1 << 26) || total_rows < max_rows) return BC_ERR_ARG;
  if (!positive_finite(shape->scale)) return BC_ERR_ARG;
  if (!workspace || !aligned16(workspace) ||
      workspace_bytes < bc_prefill_bwd_workspace_bytes(shape, total_rows))
    return BC_ERR_WORKSPACE;
  BwdParams p;
  p.q = static_cast<const char*>(q); p.k = static_cast<const char*>(k);
  p.v = static_cast<const char*>(v); p.out = out; p.lse = lse;
  p.dout = static_cast<const char*>(dout);
  p.row_off = row_offsets; p.P = P; p.c = c;
  p.dq = dq; p.dk = dk; p.dv = dv;
  p.stat = static_cast<float*>(workspace);
  p.part = p.stat + (size_t)total_rows * shape->Hq * 2;
  p.hsplit = bwd_head_splits(shape->Hq / shape->Hkv);
  p.total_rows = total_rows;
  p.D = shape->d;
  p.Hq = shape->Hq; p.Hkv = shape->Hkv; p.g = shape->Hq / shape->Hkv;
  p.scale = shape->scale;
  p.qscale = shape->scale * kLog2e;
  hipStream_t hs = as_stream(stream);
  const int tiles = (max_rows + kBwBM - 1) / kBwBM;
  const int nhg = (p.g + kDqHeads - 1) / kDqHeads;
  p.npairs = shape->B * shape->Hkv;
  p.pstride = (p.npairs + 7) & ~7;
  // key blocks: at most `tiles` dense-causal blocks + the gathered beacons + `tiles` response blocks
  const dim3 dq_grid(p.pstride * nhg, tiles), dkv_grid(p.pstride, (2 * tiles + 2) * p.hsplit + tiles);
  if (shape->d == 128) {
    prefill_bwd_dq_kernel<128><<<dq_grid, kBwWaves * 64, 0, hs>>>(p);
    prefill_bwd_dkv_kernel<128><<<dkv_grid, kBwWaves * 64, 0, hs>>>(p);
  } else {
    prefill_bwd_dq_kernel<64><<<dq_grid, kBwWaves * 64, 0, hs>>>(p);
    prefill_bwd_dkv_kernel<64><<<dkv_grid, kBwWaves * 64, 0, hs>>>(p);
  }
  if (p.hsplit > 1) {
    const int64_t blocks = (total_rows * shape->Hkv * (shape->d / 4) + 255) / 256;
    prefill_bwd_reduce_kernel<<<(int)(blocks < 65536 ? blocks : 65536), 256, 0, hs>>>(p, shape->B);
  }
  return launch_status();
}
