// bc_prefill_attn: beacon-masked prefill attention, forward (Fig. 2, Sec. 3.2 of the paper).
//
// Training keeps every row and hides what eviction would have removed.  Seen from a tile of
// 64 query rows that lies in the response, the visible keys are three runs:
//   A  the prompt rows                                   (dense, nothing masked)
//   B  the beacons of every window that ended before the tile's first window
//      (one row every c+1 rows: a strided gather,         dense, nothing masked)
//   C  the band from the start of the tile's first window to the tile's last row
//      (block-diagonal windows plus the beacons inside:   masked by integer arithmetic)
// so the kernel walks a compacted key list of about P + r/(c+1) + 64 + c rows per tile
// instead of the r rows of causal attention, and never materialises a mask.  Tiles that
// touch the prompt use run C alone with the same predicate (which is then plain causal).
//
// One workgroup = 64 query rows x up to three query heads of one KV head, 4 waves of 16 rows
// each; two workgroups share a CU (matrix and vector instructions of one SIMD overlap only
// partly on this chip, so the tile body is bound by the sum of the two).  K/V tiles of 32 keys
// are gathered from HBM into LDS by 16-byte LDS-DMA loads (3-stage ring, one barrier per tile,
// each row d * 2 contiguous bytes), shared by the 4 waves and fed to 16x16x32 MFMA: S^T = K.Q^T
// in bf16, O^T += V^T.P^T with P split into two bf16 parts so that the softmax weights keep
// about 16 bits (or, in the workspace form, as one half-precision part against a half-precision
// copy of V).  Softmax runs online in registers in the accumulator layout.  The output tile
// goes through LDS so that every row of d floats is written to HBM as one burst.  Head
// dimension 128 or 64 (a template parameter).
#include <type_traits>

#include "bc_common.h"

namespace bc {

constexpr int kPfWaves = 4;
constexpr int kPfBM = 64;                 // query rows per workgroup
constexpr int kPfBN = 32;                 // keys per tile
constexpr int kPfStages = 3;

typedef __attribute__((address_space(3))) void pf_lds_void_t;
typedef __attribute__((address_space(1))) const void pf_global_void_t;
typedef __attribute__((ext_vector_type(4))) short pf_s16x4_t;
typedef __attribute__((ext_vector_type(8))) short pf_s16x8_t;
typedef __attribute__((address_space(3))) pf_s16x4_t pf_lds_s16x4_t;
typedef __attribute__((ext_vector_type(2))) float pf_f32x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 pf_f16x2_t;
typedef __attribute__((ext_vector_type(8))) _Float16 pf_f16x8_t;

struct PrefillParams {
  const char* q;
  const char* k;
  const char* v;
  const char* v16;         // V rounded to half precision, same layout (workspace form only)
  const int32_t* flag;     // workspace form: 0 = every V entry fits half precision, 1 = not; else NULL
  const int64_t* row_off;
  const int32_t* P;
  const int32_t* c;
  float* out;
  float* lse;
  int32_t Hq, Hkv, g;
  int32_t hsplit;     // the group's heads are split over this many workgroups (HPW heads each)
  int32_t npairs;     // (trajectory, KV head) pairs
  int32_t pstride;    // npairs rounded up to a multiple of 8
  float qscale;       // softmax scale * log2(e)
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {      // RNE, a in the low half
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(pf_f32x2_t{a, b}, bf16x2_t));
}

constexpr float kPfLazy = 5.0f;

// HPW: query heads per wave (the group's heads are split over p.hsplit workgroups); D: head
// dimension, 128 or 64 (rows of 256 or 128 bytes: 16 or 8 units of 16 bytes, four or eight rows
// per 1 KB LDS-DMA instruction, four or two 32-wide steps of the score product, eight or four
// 16-column blocks of the output).
// HALF: the weights enter the value product as one half-precision part (11 bits) against V in
// half precision, instead of two bf16 parts against V in bf16: a third fewer matrix instructions
// and no split.  V's copy in half precision is exact for entries between 2^-14 and 65504 in
// magnitude (bf16 has fewer mantissa bits), which a conversion pass checks; both forms of the
// kernel are launched and each leaves at once when the pass's verdict is for the other.
template <int HPW, int D, bool HALF>
__global__ __launch_bounds__(kPfWaves * 64, 2) void prefill_kernel(PrefillParams p) {
  if (p.flag != nullptr && (p.flag[0] != 0) == HALF) return;
  constexpr int ROWB = D * 2;                 // bytes of a K or V row
  constexpr int UPR = ROWB / 16;              // 16-byte units per row
  constexpr int KS = D / 32;                  // k-steps of the score product
  constexpr int NJ = D / 16;                  // 16-column blocks of the output
  constexpr int kPfTile = kPfBN * ROWB;       // bytes of one K (or V) tile
  constexpr int RPI = 1024 / ROWB;            // rows per LDS-DMA instruction
  constexpr int NLD = kPfBN / (RPI * kPfWaves);   // instructions per wave, tile and tensor
  constexpr int kPfLds = kPfStages * 2 * kPfTile;   // the epilogue's 4 x 16 x D floats fit inside
  static_assert(kPfLds >= kPfWaves * 16 * D * 4, "the output tiles fit the ring's LDS");
  __shared__ __attribute__((aligned(1024))) char lds[kPfLds];
  // grid: x = (head split, trajectory, KV head), y = query tile; workgroups are dispatched
  // x-fastest, so the longest tiles of every trajectory start first
  // (the head splits of a pair are `pstride` workgroups apart, a multiple of 8: workgroups go to the
  // XCDs in turn, so the splits - which read the same K/V tiles - share an L2)
  const int hh = blockIdx.x / p.pstride, pair = blockIdx.x - hh * p.pstride;
  if (pair >= p.npairs) return;
  const int kvh = pair % p.Hkv, b = pair / p.Hkv;
  const int64_t off0 = p.row_off[b];
  const int S = (int)(p.row_off[b + 1] - off0);
  const int qt = gridDim.y - 1 - blockIdx.y;        // long tiles first
  const int r0 = qt * kPfBM;
  if (r0 >= S) return;
  const int r1 = min(r0 + kPfBM - 1, S - 1);
  const int P = p.P[b];
  const WindowStride ws = window_stride(p.c[b], S);
  const int c = ws.c, cp1 = ws.stride;

  // compacted key list of this tile
  int nA = 0, nB = 0, band_start = 0;
  if (c > 0 && r0 >= P) {
    const int m0 = (int)window_of(ws, (uint32_t)(r0 - P));
    nA = P; nB = m0; band_start = P + m0 * cp1;
  }
  const int nC = r1 - band_start + 1;
  const int TA = (nA + kPfBN - 1) / kPfBN, TB = (nB + kPfBN - 1) / kPfBN;
  const int NT = TA + TB + (nC + kPfBN - 1) / kPfBN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, kb = lane >> 4;
  const int tg = wave;
  const HalfSelectors sel = half_selectors();
  const int64_t kv_row_bytes = (int64_t)p.Hkv * ROWB;
  const char* kbase = p.k + (off0 * p.Hkv + kvh) * ROWB;
  const char* vbase = (HALF ? p.v16 : p.v) + (off0 * p.Hkv + kvh) * ROWB;

  // Key tile kt covers 32 consecutive entries of one run.  Entry rr is row j0 + rr*step;
  // entries at and beyond nvalid do not exist (their loads are redirected to row r1).
  struct TileDesc { int j0, step, nvalid; bool predicate; };
  auto tile_desc = [&](int kt) -> TileDesc {
    TileDesc t;
    if (kt < TA) { t.j0 = kt * kPfBN; t.step = 1; t.nvalid = nA - kt * kPfBN; t.predicate = false; }
    else if (kt < TA + TB) {
      const int m = (kt - TA) * kPfBN;
      t.j0 = P + m * cp1 + c; t.step = cp1; t.nvalid = nB - m; t.predicate = false;
    } else {
      const int x = (kt - TA - TB) * kPfBN;
      t.j0 = band_start + x; t.step = 1; t.nvalid = nC - x; t.predicate = true;
    }
    t.nvalid = min(t.nvalid, kPfBN);
    return t;
  };
  // HBM -> LDS gather of tile kt: one instruction moves RPI whole rows; this wave brings entries
  // RPI*wave .. RPI*wave + RPI-1 of K and of V (and, d = 128, the same 16 entries further on)
  const int ld_rr = RPI * wave + lane / UPR;
  auto issue_tile = [&](int kt, int stage) {
    const TileDesc t = tile_desc(kt);
#pragma unroll
    for (int half = 0; half < NLD; ++half) {
      const int rr = ld_rr + RPI * kPfWaves * half;
      const int j = rr < t.nvalid ? t.j0 + rr * t.step : r1;
      const int64_t goff = (int64_t)j * kv_row_bytes + (((lane & (UPR - 1)) ^ tile_swz<D>(rr)) << 4);
      char* dst = lds + stage * (2 * kPfTile) + (wave + kPfWaves * half) * 1024;
      __builtin_amdgcn_global_load_lds((pf_global_void_t*)(kbase + goff), (pf_lds_void_t*)dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((pf_global_void_t*)(vbase + goff),
                                       (pf_lds_void_t*)(dst + kPfTile), 16, 0, 0);
    }
  };

  issue_tile(0, 0);
  if (NT > 1) issue_tile(1, 1);

  // this lane's query row and heads; Q^T as the B operand (column n = row, k = head-dim index)
  const int r = r0 + 16 * tg + n;
  const bool row_ok = r <= r1;
  const int rq = row_ok ? r : r1;
  bf16x8_t qb[HPW][KS];
#pragma unroll
  for (int h = 0; h < HPW; ++h) {
    const int head = hh * HPW + h;
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      uint4 x = make_uint4(0u, 0u, 0u, 0u);
      if (head < p.g)
        x = *reinterpret_cast<const uint4*>(
            p.q + (((off0 + rq) * p.Hq + kvh * p.g + head) * D + 32 * i + 8 * kb) * 2);
      qb[h][i] = __builtin_bit_cast(bf16x8_t, x);
    }
  }
  const int win_r = (c > 0 && r >= P) ? (int)window_of(ws, (uint32_t)(r - P)) : -1;

  f32x4_t O[HPW][NJ];
  float m_run[HPW], l_run[HPW], grow_at[HPW];
  // HALF: the denominators are summed by the matrix cores from the same rounded weights that
  // enter the value product (a row of ones as the other operand), so that numerator and
  // denominator carry the same rounding: what is left of it in o is second order, and a row
  // with one dominant key is as exact as in the two-part form.
  f32x4_t Lacc[HPW];
  const pf_f16x8_t ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f,
                           (_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f};
  const float inv_qscale = 1.0f / p.qscale;
#pragma unroll
  for (int h = 0; h < HPW; ++h) {
    m_run[h] = kNegBig; l_run[h] = 0.f; grow_at[h] = (kNegBig + kPfLazy) * inv_qscale;
    Lacc[h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NJ; ++j) O[h][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }

  // Body of one key tile.  Scores stay unscaled; the softmax scale enters through one fused
  // multiply-add per key: p = 2^(s*qs - m), qs > 0.
  const bool full_rows = r0 + kPfBM - 1 <= r1;
  auto tile_body = [&](const char* tk, const char* tv, const TileDesc& td) {
    // a full tile of the prompt or beacon run under a full query tile needs no per-key tests;
    // the flag is uniform over the workgroup, so the tests are skipped by cheap scalar branches
    const bool MASKED = td.predicate || td.nvalid < kPfBN || !full_rows;
    bool vis[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vis[e] = true;
    if (MASKED) {
      const int lim = row_ok ? td.nvalid - 8 * kb : 0;      // entries e < lim exist
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

    // S^T = K . Q^T ; row m of sub-tile t is tile entry 8*(m/4) + 4*t + m%4
    bf16x8_t ka[2][KS];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = ((n >> 2) << 3) + 4 * t + (n & 3);
#pragma unroll
      for (int i = 0; i < KS; ++i)
        ka[t][i] = *reinterpret_cast<const bf16x8_t*>(tk + row * ROWB + (((4 * i + kb) ^ tile_swz<D>(row)) << 4));
    }
    bf16x8_t phi[HPW], plo[HPW];
    // the scores of every head first: 2 * HPW independent accumulation chains keep the matrix
    // pipe full, and the first head's scores are back when its softmax starts
    f32x4_t Sx[HPW][2];
#pragma unroll
    for (int h = 0; h < HPW; ++h)
#pragma unroll
      for (int t = 0; t < 2; ++t) Sx[h][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < KS; ++i)
#pragma unroll
      for (int h = 0; h < HPW; ++h)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          Sx[h][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][i], qb[h][i], Sx[h][t], 0, 0, 0);
#pragma unroll
    for (int h = 0; h < HPW; ++h) {
      float sv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sv[e] = Sx[h][e >> 2][e & 3];
      }
      if (MASKED) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sv[e] = vis[e] ? sv[e] : kNegBig;
      }
      float tmax = fmaxf(fmaxf(fmaxf(fmaxf(sv[0], sv[1]), sv[2]), fmaxf(fmaxf(sv[3], sv[4]), sv[5])),
                         fmaxf(sv[6], sv[7]));
      // Lazy reference: the running reference m only moves when the tile's maximum exceeds it by
      // more than kPfLazy (log2 units); until then weights are at most 2^kPfLazy, which fp32 sums
      // and the two-part bf16 weights carry without loss, and the accumulators need no rescale.
      // The test runs on the unscaled maximum against grow_at = (m + kPfLazy) / qs - on each
      // lane's own eight keys: only when some lane passes the mark are the row maxima needed.
      if (__any(tmax > grow_at[h])) {
        tmax = rows_allreduce_max(tmax);
        const float m_cand = tmax * p.qscale;                   // kNegBig * qs stays hugely negative
        const float m_new = m_cand > m_run[h] + kPfLazy ? m_cand : m_run[h];
        const float alpha = fast_exp2(m_run[h] - m_new);
        m_run[h] = m_new;
        grow_at[h] = (m_new + kPfLazy) * inv_qscale;
        l_run[h] *= alpha;
        if constexpr (HALF) Lacc[h] *= alpha;
#pragma unroll
        for (int j = 0; j < NJ; ++j) O[h][j] *= alpha;
      }
      const float m_new = m_run[h];
      float pe[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pe[e] = fast_exp2(fmaf(sv[e], p.qscale, -m_new));
      }
      if (MASKED) {
#pragma unroll
        for (int e = 0; e < 8; ++e) pe[e] = vis[e] ? pe[e] : 0.f;
      }
      const float psum = ((pe[0] + pe[1]) + (pe[2] + pe[3])) + ((pe[4] + pe[5]) + (pe[6] + pe[7]));
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        if constexpr (HALF) {
          hi[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pf_f32x2_t{pe[e], pe[e + 1]}, pf_f16x2_t));
          lo[e >> 1] = 0u;
        } else {
          const uint32_t hp = pack_bf16(pe[e], pe[e + 1]);
          hi[e >> 1] = hp;
          lo[e >> 1] = pack_bf16(minus_half(pe[e], hp, sel.low), minus_half(pe[e + 1], hp, sel.high));
        }
      }
      phi[h] = __builtin_bit_cast(bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
      plo[h] = __builtin_bit_cast(bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
      if constexpr (HALF)
        Lacc[h] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, __builtin_bit_cast(pf_f16x8_t, phi[h]), Lacc[h], 0, 0, 0);
      else
        l_run[h] += psum;
    }
    // O^T += V^T . P^T ; V^T through the transposing LDS read
    {
      const int rl = lane & 15;
      const int rowa = 8 * kb + (rl >> 2), rowb = rowa + 4;
      const int sub = (rl & 1) << 3;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int u = 2 * j + ((rl & 3) >> 1);
        const pf_s16x4_t a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (pf_lds_s16x4_t*)(tv + rowa * ROWB + ((u ^ tile_swz<D>(rowa)) << 4) + sub));
        const pf_s16x4_t a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (pf_lds_s16x4_t*)(tv + rowb * ROWB + ((u ^ tile_swz<D>(rowb)) << 4) + sub));
        const bf16x8_t av = __builtin_bit_cast(
            bf16x8_t, (pf_s16x8_t)__builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int h = 0; h < HPW; ++h) {
          if constexpr (HALF) {
            O[h][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(pf_f16x8_t, av),
                                                             __builtin_bit_cast(pf_f16x8_t, phi[h]), O[h][j], 0, 0, 0);
          } else {
            O[h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phi[h], O[h][j], 0, 0, 0);
            O[h][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plo[h], O[h][j], 0, 0, 0);
          }
        }
      }
    }
  };

  int stage = 0;
  for (int kt = 0; kt < NT; ++kt) {
    // tile kt has landed (this wave's part); after the barrier everyone's part has, and
    // everyone has finished tile kt-1, whose stage is the one tile kt+2 goes into
    if (kt + 1 < NT) wait_vmcnt<2 * NLD>();         // (the next tile's loads may stay out)
    else wait_vmcnt<0>();
    __syncthreads();
    if (kt + 2 < NT) issue_tile(kt + 2, stage >= 1 ? stage - 1 : kPfStages - 1);
    const char* tk = lds + stage * (2 * kPfTile);
    const char* tv = tk + kPfTile;
    stage = stage + 1 == kPfStages ? 0 : stage + 1;
    const TileDesc td = tile_desc(kt);
    // a band tile that starts behind the last of this wave's 16 rows holds nothing they may see
    if (td.predicate && td.j0 > r0 + 16 * tg + 15) continue;
    tile_body(tk, tv, td);
  }
  __syncthreads();          // the tile stages are free: the epilogue reuses LDS

  // ---- epilogue: normalise, transpose through LDS, write each row of D floats as one burst
  constexpr int OLPR = D / 4;                 // lanes that cover one output row, 16 bytes each
  constexpr int ORPP = 64 / OLPR;             // rows per pass
  float* my = reinterpret_cast<float*>(lds + wave * (16 * D * 4));        // [16 rows][D] fp32, swizzled
#pragma unroll
  for (int h = 0; h < HPW; ++h) {
    const int head = hh * HPW + h;
    float l;
    if constexpr (HALF) l = Lacc[h][0];            // (already the sum over all keys of the lane's row)
    else l = rows_allreduce_sum(l_run[h]);
    const float inv = 1.0f / l;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int unit = (4 * j + kb) ^ n;                // 16-byte units of an output row
      *reinterpret_cast<f32x4_t*>(my + n * D + unit * 4) = O[h][j] * inv;
    }
    if (head < p.g) {
      // OLPR lanes cover one row (16 bytes each), ORPP rows per pass
#pragma unroll
      for (int pass = 0; pass < 16 / ORPP; ++pass) {
        const int t = ORPP * pass + lane / OLPR, unit = lane & (OLPR - 1);
        const f32x4_t val = *reinterpret_cast<const f32x4_t*>(my + t * D + ((unit ^ t) << 2));
        const int rr = r0 + 16 * tg + t;
        if (rr <= r1)     // written once, not read again by this launch: streaming store
          __builtin_nontemporal_store(val, reinterpret_cast<f32x4_t*>(
              p.out + ((off0 + rr) * p.Hq + kvh * p.g + head) * D + unit * 4));
      }
      if (p.lse && kb == 0 && row_ok)
        p.lse[(off0 + r) * p.Hq + kvh * p.g + head] = (m_run[h] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    }
  }
}

// V in half precision for the workspace form: 8 entries per thread and pass; the verdict word is
// set when a finite entry does not fit (65520 and beyond rounds to infinity).
__global__ __launch_bounds__(256) void prefill_v16_kernel(const uint4* __restrict__ v, uint4* __restrict__ v16,
                                                          int64_t units, int32_t* flag) {
  bool over = false;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < units; i += (int64_t)gridDim.x * blockDim.x) {
    float f[8];
    unpack16(v[i], f, bf16_t{});
    uint32_t h[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      over = over || (fabsf(f[e]) >= 65520.f && fabsf(f[e]) < __builtin_inff()) ||
             (fabsf(f[e + 1]) >= 65520.f && fabsf(f[e + 1]) < __builtin_inff());
      h[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pf_f32x2_t{f[e], f[e + 1]}, pf_f16x2_t));
    }
    v16[i] = make_uint4(h[0], h[1], h[2], h[3]);
  }
  if (__any(over) && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}
__global__ void prefill_clear_flag_kernel(int32_t* flag) { flag[0] = 0; }

constexpr size_t kPfFlagBytes = 256;

template <bool HALF>
static void launch_prefill(const PrefillParams& p, int d, int hpw, dim3 grid, hipStream_t hs) {
  if (d == 128) {
    switch (hpw) {
      case 1: prefill_kernel<1, 128, HALF><<<grid, kPfWaves * 64, 0, hs>>>(p); break;
      case 2: prefill_kernel<2, 128, HALF><<<grid, kPfWaves * 64, 0, hs>>>(p); break;
      default: prefill_kernel<3, 128, HALF><<<grid, kPfWaves * 64, 0, hs>>>(p); break;
    }
  } else {
    switch (hpw) {
      case 1: prefill_kernel<1, 64, HALF><<<grid, kPfWaves * 64, 0, hs>>>(p); break;
      case 2: prefill_kernel<2, 64, HALF><<<grid, kPfWaves * 64, 0, hs>>>(p); break;
      default: prefill_kernel<3, 64, HALF><<<grid, kPfWaves * 64, 0, hs>>>(p); break;
    }
  }
}

// Shared by the two entry points.  workspace == nullptr: the two-part form alone.
static int32_t prefill_forward(const bc_shape* shape, const void* q, const void* k, const void* v,
                               const int64_t* row_offsets, const int32_t* P, const int32_t* c,
                               int32_t max_rows, int64_t total_rows, float* out, float* lse,
                               void* workspace, void* stream) {
  PrefillParams p;
  p.q = static_cast<const char*>(q);
  p.k = static_cast<const char*>(k);
  p.v = static_cast<const char*>(v);
  p.v16 = nullptr; p.flag = nullptr;
  p.row_off = row_offsets; p.P = P; p.c = c;
  p.out = out; p.lse = lse;
  p.Hq = shape->Hq; p.Hkv = shape->Hkv; p.g = shape->Hq / shape->Hkv;
  p.qscale = shape->scale * kLog2e;
  // at most three heads per workgroup (the accumulators of a fourth do not fit the register
  // file): one workgroup for a single head, two for groups up to six, three for seven and eight
  p.hsplit = p.g == 1 ? 1 : (p.g <= 6 ? 2 : 3);
  const int hpw = (p.g + p.hsplit - 1) / p.hsplit;
  p.npairs = shape->Hkv * shape->B;
  p.pstride = (p.npairs + 7) & ~7;
  const dim3 grid(p.hsplit * p.pstride, (max_rows + kPfBM - 1) / kPfBM);
  hipStream_t hs = as_stream(stream);
  if (workspace) {
    int32_t* flag = static_cast<int32_t*>(workspace);
    char* v16 = static_cast<char*>(workspace) + kPfFlagBytes;
    const int64_t units = total_rows * shape->Hkv * shape->d / 8;
    const int64_t blocks = (units + 255) / 256;
    prefill_clear_flag_kernel<<<1, 1, 0, hs>>>(flag);
    prefill_v16_kernel<<<(int)(blocks < 4096 ? blocks : 4096), 256, 0, hs>>>(
        static_cast<const uint4*>(v), reinterpret_cast<uint4*>(v16), units, flag);
    p.v16 = v16; p.flag = flag;
    launch_prefill<true>(p, shape->d, hpw, grid, hs);
  }
  launch_prefill<false>(p, shape->d, hpw, grid, hs);
  return launch_status();
}

}  // namespace bc

using namespace bc;

extern "C" size_t bc_prefill_workspace_bytes(const bc_shape* shape, int64_t total_rows) {
  if (check_shape(shape) != BC_OK || total_rows < 1) return 0;
  return kPfFlagBytes + (size_t)total_rows * shape->Hkv * shape->d * 2;
}

extern "C" int32_t bc_prefill_attn_ws(const bc_shape* shape, const void* q, const void* k,
                                      const void* v, const int64_t* row_offsets, const int32_t* P,
                                      const int32_t* c, int32_t max_rows, int64_t total_rows,
                                      float* out, float* lse, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  if (shape->kv_dtype != BC_BF16) return BC_ERR_SHAPE;
  if (!q || !k || !v || !row_offsets || !P || !c || !out) return BC_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return BC_ERR_ARG;
  if (max_rows < 1 || max_rows >= (1 << 26) || total_rows < max_rows) return BC_ERR_ARG;
  if (!positive_finite(shape->scale)) return BC_ERR_ARG;
  if (!workspace || !aligned16(workspace) || workspace_bytes < bc_prefill_workspace_bytes(shape, total_rows))
    return BC_ERR_WORKSPACE;
  return prefill_forward(shape, q, k, v, row_offsets, P, c, max_rows, total_rows, out, lse, workspace, stream);
}

extern "C" int32_t bc_prefill_attn(const bc_shape* shape, const void* q, const void* k,
                                   const void* v, const int64_t* row_offsets, const int32_t* P,
                                   const int32_t* c, int32_t max_rows, float* out, float* lse,
                                   void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  if (shape->kv_dtype != BC_BF16) return BC_ERR_SHAPE;
  if (!q || !k || !v || !row_offsets || !P || !c || !out) return BC_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return BC_ERR_ARG;
  if (max_rows < 1 || max_rows >= (1 << 26)) return BC_ERR_ARG;
  if (!positive_finite(shape->scale)) return BC_ERR_ARG;       // the kernel takes maxima of unscaled scores
  return prefill_forward(shape, q, k, v, row_offsets, P, c, max_rows, 0, out, lse, nullptr, stream);
}
