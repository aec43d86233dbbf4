// bc_decode_attn: single-token grouped-query attention over the ragged compressed cache
// (Sec. 2 and Sec. 3.1 of the paper: standard attention over whatever is resident).
//
// Split-K flash decoding.  Work item = (sequence, KV head) pair x chunk of rows; grid =
// (max chunks, pairs).  With 128 pairs or more a pair is one chunk and its workgroup finishes
// it.  With fewer pairs the resident rows of a sequence are spread evenly over up to 64
// workgroups (sequences under 1024 rows stay whole); every chunk writes an (m, l, o) partial
// and a second, small kernel folds the partials of each pair in chunk order.  No float atomics
// and no fences: results are bit-reproducible.  Large ragged batches (more pairs than compute
// units) can dispatch the longest sequences first (bc_sort_by_length).  Batches of at most 128
// pairs with short caches use two workgroups per pair, each with all K rows and one half of the
// V columns, so that all compute units pull data and nothing has to be merged.
//
// Two main kernels:
//  * decode_lds_kernel (bf16, d = 128 or 64): every wave streams 32-row K and V tiles from HBM
//    straight into its own LDS region with 16-byte LDS-DMA loads (1 KB of consecutive bytes
//    per instruction, 16 KB in flight per wave at d = 128), then forms the q.K products and the p.V
//    sums of all query heads of the group with 16x16x32 bf16 MFMA tiles fed from LDS (K by
//    128-bit reads, V by the 16-bit transposing reads), softmax in registers.
//  * decode_valu_kernel (fp32): rows held in registers, 16 bytes per lane, plain
//    FMA dot products completed by a DPP all-reduce.
// Both carry the fused step (append before, eviction after the attention) in the same launch: the
// appended row is read from the caller's tensors, every reader of a sequence takes a ticket when
// it is done with the slab, and the holder of the last ticket moves the beacon and the tables.
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <type_traits>
#include "bc_common.h"

namespace bc {

// Every sequence's ticket counter has a 128-byte line to itself: the workgroups of a launch finish
// close together, and their atomics on a shared line would queue up behind each other.
constexpr int kTicketStride = 32;

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
  float* part_o;       // [pairs][max_chunks][Gp][D]
  float* part_ml;      // [pairs][max_chunks][2][Gp]   (running max in log2 units, denominator)
  int32_t* part_n;     // [pairs] chunks written by this launch (read by the merge kernel)
  // fused step (all nullable): append this token row first, evict with this beacon afterwards
  const int32_t* c;
  int32_t* nb_rw;
  int32_t* w_rw;
  const char* new_k;
  const char* new_v;
  const char* bk;
  const char* bv;
  int32_t* tickets;    // [B] counters kTicketStride ints apart, zero between launches
  const int32_t* order;     // [B] dispatch order (workgroup i serves sequence order[i]) or null
  const int32_t* budget;   // [B] cap on nb + w (nullable), with
  uint8_t* live;           // [B] cleared when the cap is reached
  int32_t beacon_row;  // the fused row is the beacon closing a full window (bk = new_k, bv = new_v)
  int32_t B;
  int32_t spec_P, spec_cap;   // bc_cache::uniform_P, uniform_cap (0 = no promise)
  int32_t Hq, Hkv, g;  // g = real group size
  int32_t Gp;          // padded group size of the partial layout
  int32_t D;
  int32_t rows_per_wg; // R: rows per workgroup when a chunk size is forced; otherwise (0) the
                       // resident rows of a sequence are spread evenly over its chunks
  int32_t max_chunks;
  float qscale;        // softmax scale * log2(e)
};

struct PairInfo {
  int s, kvh, L, nchunks, chunk, row0, row_end;
  int P, nb, w_att, cap, c;   // tables as the attention of this launch sees them
  int64_t base;               // first entry of the sequence in the slabs
  int new_row;                // slot of the row appended by this launch, or -1
  bool evict_due;             // this launch ends with beacon append + eviction
  bool store_new_row;         // the appended row outlives this launch: write it to the slab
  bool update;                // tables change at the end of this launch
  bool live;
};

// Common prologue: which rows does this workgroup own?  Uniform across the workgroup.  All
// table loads are issued together.  With a fused append the state rules of bc_append_kv are
// applied here, identically in every workgroup of the sequence.
constexpr int kMinChunkRows = 128;   // a chunk smaller than this is not worth a workgroup
constexpr int kMinSplitRows = 1024;  // sequences shorter than this are not split at all
constexpr int kLptMaxB = 4096;       // sort key: length * 4096 + index
constexpr int kLptMaxLen = 1 << 19;
constexpr int kLptMinPairs = 256;    // compute units of the chip: below this every workgroup starts at once

// Longest sequence first: with more workgroups than the chip holds at once and ragged lengths,
// the dispatch order decides the tail.  bc_sort_by_length ranks the B sequences by resident
// length (keys made unique by the index, so the ranks are a permutation) into an array the
// caller owns; with that array in bc_cache::order, workgroup number i of a decode launch (in
// dispatch order) serves sequence order[i].  The array is only read by the decode launches, so
// every workgroup sees the same permutation even while a fused step updates the tables, and it
// may be as old as the caller likes.
struct SortParams {
  const uint8_t* active;
  const int32_t *P, *nb, *w;
  int32_t* order;
  int32_t B;
};

__global__ __launch_bounds__(256) void sort_by_length_kernel(SortParams p) {
  __shared__ int s_key[kLptMaxB];
  for (int t = threadIdx.x; t < p.B; t += blockDim.x) {
    const int act = p.active ? p.active[t] : 1;
    int len = act ? p.P[t] + p.nb[t] + p.w[t] + 1 : 0;         // inactive sequences rank last
    len = min(max(len, 0), kLptMaxLen - 1);
    s_key[t] = (len << 12) | (kLptMaxB - 1 - t);
  }
  for (int t = p.B + threadIdx.x; t < ((p.B + 3) & ~3); t += blockDim.x) s_key[t] = -1;
  __syncthreads();
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= p.B) return;
  const int mine = s_key[t];
  int rank = 0;                                               // number of larger keys
  for (int u = 0; u < p.B; u += 4) {
    const int4 o = *reinterpret_cast<const int4*>(s_key + u);
    rank += (o.x > mine) + (o.y > mine) + (o.z > mine) + (o.w > mine);
  }
  p.order[rank] = t;
}

// The kernel arguments span four 64-byte lines that the code below would touch one after the
// other, each a miss of the scalar cache on the way to the first tile request: ask for all four
// at once.
__device__ __forceinline__ void touch_kernel_arguments() {
  typedef __attribute__((address_space(4))) const int const_int_t;
  const_int_t* ka = (const_int_t*)__builtin_amdgcn_kernarg_segment_ptr();
  static_assert(sizeof(DecodeParams) > 48 * 4, "the last line touched lies inside the arguments");
  const int a = ka[0], b = ka[16], c = ka[32], d = ka[48];
  asm volatile("" : : "s"(a), "s"(b), "s"(c), "s"(d));
}

// slot: the sequence's index, or its rank in the dispatch order when there is one.  The grid
// carries (chunk, KV head, slot) in its three dimensions, so that nothing has to be divided
// before the tables can be requested; all of them are requested together.
struct NoEarlyWork { __device__ __forceinline__ void operator()() const {} };
template <typename F = NoEarlyWork>
__device__ __forceinline__ PairInfo pair_info(const DecodeParams& p, int slot, int kvh, int chunk,
                                              const F& while_tables_travel = F()) {
  PairInfo pi;
  int act, w;
  int s = slot;
  bool bad_order = false;
  // (values that are the same for the whole workgroup are moved to scalar registers where the
  // compiler cannot see that itself - anything it loads through the vector path - so that the
  // conditions on them become real branches instead of lane masks)
  if (p.order) {
    s = __builtin_amdgcn_readfirstlane(p.order[slot]);
    bad_order = (unsigned)s >= (unsigned)p.B;        // not written by bc_sort_by_length
    if (bad_order) s = 0;
  }
  pi.s = s;
  pi.kvh = kvh;
  // The six table entries travel through the scalar cache, requested by hand: their counter is
  // not the vector loads' one, so work started in the meantime (the first tile, when the caller
  // has promised the slab geometry) does not have to be back before they are.
  {
    int32_t tP, tnb, tw, tcap, tc;
    int64_t tbase;
    asm volatile("s_load_dword %0, %1, 0x0" : "=s"(tP) : "s"(p.P + pi.s) : "memory");
    asm volatile("s_load_dword %0, %1, 0x0" : "=s"(tnb) : "s"(p.nb + pi.s) : "memory");
    asm volatile("s_load_dword %0, %1, 0x0" : "=s"(tw) : "s"(p.w + pi.s) : "memory");
    asm volatile("s_load_dword %0, %1, 0x0" : "=s"(tcap) : "s"(p.cap + pi.s) : "memory");
    asm volatile("s_load_dwordx2 %0, %1, 0x0" : "=s"(tbase) : "s"(p.base + pi.s) : "memory");
    asm volatile("s_load_dword %0, %1, 0x0" : "=s"(tc) : "s"(p.c + pi.s) : "memory");
    while_tables_travel();
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(tP), "+s"(tnb), "+s"(tw), "+s"(tcap), "+s"(tbase), "+s"(tc) : : "memory");
    pi.P = tP; pi.nb = tnb; w = tw; pi.cap = tcap; pi.base = tbase; pi.c = tc;
  }
  act = p.active ? __builtin_amdgcn_readfirstlane((int)p.active[pi.s]) : 1;
  if (bad_order) {
    if (chunk == 0 && threadIdx.x == 0) atomicOr(p.err, BC_ERRBIT_STATE);
    act = 0;
  }
  const bool herald = chunk == 0 && pi.kvh == 0 && threadIdx.x == 0;   // reports errors
  pi.live = false;
  pi.update = false; pi.evict_due = false; pi.new_row = -1; pi.store_new_row = false;
  pi.L = 0; pi.nchunks = 0; pi.chunk = chunk; pi.row0 = 0; pi.row_end = 0; pi.w_att = w;
  // beacon step: only sequences whose window is full take part; one that has no room for the
  // beacon at the tail is reported and left alone
  bool take = act != 0;
  if (take && p.beacon_row) {
    take = pi.c > 0 && w == pi.c;
    if (take && pi.P + pi.nb + w >= pi.cap) {
      if (herald) atomicOr(p.err, BC_ERRBIT_CAPACITY);
      take = false;
    }
  }
  if (take) {
    const int L_old = pi.P + pi.nb + w;
    bool append_ok = false;
    if (p.beacon_row) {
      append_ok = true;
    } else if (p.new_k) {
      if (pi.c > 0 && w >= pi.c) { if (herald) atomicOr(p.err, BC_ERRBIT_STATE); }
      else if (L_old >= pi.cap)  { if (herald) atomicOr(p.err, BC_ERRBIT_CAPACITY); }
      else append_ok = true;
    }
    pi.L = L_old + (append_ok ? 1 : 0);
    pi.w_att = w + (append_ok ? 1 : 0);
    if (append_ok) pi.new_row = L_old;
    if (p.beacon_row) {
      pi.evict_due = true;          // the row just attended to moves behind the earlier beacons
    } else if (p.bk && pi.c > 0) {
      if (pi.w_att == pi.c + 1) { if (herald) atomicOr(p.err, BC_ERRBIT_STATE); }
      else if (pi.w_att == pi.c) pi.evict_due = true;
    }
    // a row that this step's eviction drops at once (c = 1, or the beacon itself, which goes
    // straight to its slot behind the earlier beacons) is never written at the tail
    pi.store_new_row = append_ok && !(pi.evict_due && (pi.w_att == 1 || p.beacon_row));
    if (pi.L <= 0) {
      if (herald) atomicOr(p.err, BC_ERRBIT_STATE);
    } else {
      // rows per chunk: the forced size, or the sequence's rows spread evenly over as many of
      // the max_chunks workgroups as have at least kMinChunkRows rows to read
      int rpc = p.rows_per_wg;
      if (rpc <= 0 && p.max_chunks == 1) {
        rpc = (pi.L + 31) & ~31;              // one workgroup has the whole sequence
        pi.nchunks = 1;
      } else {
        if (rpc <= 0) {
          // (a short sequence stays whole: its partial would cost more than the split saves)
          const int nc = pi.L < kMinSplitRows ? 1 : min(p.max_chunks, pi.L / kMinChunkRows);
          rpc = (((pi.L + nc - 1) / nc) + 31) & ~31;
        }
        pi.nchunks = (pi.L + rpc - 1) / rpc;
      }
      // the evaluation cap is tested on what this step's attention sees, whether or not the
      // append went through
      pi.update = append_ok || pi.evict_due ||
                  (p.budget && pi.nb + pi.w_att >= __builtin_amdgcn_readfirstlane(p.budget[pi.s]));
      if (pi.chunk < pi.nchunks) {
        pi.row0 = pi.chunk * rpc;
        pi.row_end = min(pi.L, pi.row0 + rpc);
        pi.live = true;
      }
    }
  }
  if (p.part_n && chunk == 0 && threadIdx.x == 0) p.part_n[pi.s * p.Hkv + pi.kvh] = pi.nchunks;
  // (uniform by construction; said explicitly for what went through vector arithmetic)
  pi.L = __builtin_amdgcn_readfirstlane(pi.L);
  pi.nchunks = __builtin_amdgcn_readfirstlane(pi.nchunks);
  pi.row0 = __builtin_amdgcn_readfirstlane(pi.row0);
  pi.row_end = __builtin_amdgcn_readfirstlane(pi.row_end);
  pi.new_row = __builtin_amdgcn_readfirstlane(pi.new_row);
  pi.live = __builtin_amdgcn_readfirstlane((int)pi.live) != 0;
  pi.update = __builtin_amdgcn_readfirstlane((int)pi.update) != 0;
  pi.evict_due = __builtin_amdgcn_readfirstlane((int)pi.evict_due) != 0;
  pi.store_new_row = __builtin_amdgcn_readfirstlane((int)pi.store_new_row) != 0;
  return pi;
}

// What the holder of a sequence's last ticket does, as one wave, once every reader of the
// sequence's rows is done with them: the beacon entry goes to its slot behind the earlier beacons
// (the evicted window's first row), the tables move on, the ticket counter returns to zero.
template <int ROWB>
__device__ __forceinline__ void finish_step(const DecodeParams& p, const PairInfo& pi, int lane) {
  constexpr int UPR = ROWB / 16;                   // 16-byte units per row
  if (pi.evict_due) {
    const int n16 = p.Hkv * UPR;                   // 16-byte units of one K (or V) entry
    for (int i = lane; i < 2 * n16; i += 64) {
      const int which = i >= n16, r = which ? i - n16 : i;
      const int h = r / UPR, u = r & (UPR - 1);
      const char* src = (which ? p.bv : p.bk) + (int64_t)(pi.s * p.Hkv + h) * ROWB + (u << 4);
      char* slab = const_cast<char*>(which ? p.v_slab : p.k_slab);
      const int64_t dst =
          (pi.base * p.Hkv + (int64_t)h * pi.cap + pi.P + pi.nb) * ROWB + (u << 4);
      *reinterpret_cast<uint4*>(slab + dst) = *reinterpret_cast<const uint4*>(src);
    }
  }
  if (lane == 0) {
    p.tickets[pi.s * kTicketStride] = 0;
    p.nb_rw[pi.s] = pi.nb + (pi.evict_due ? 1 : 0);
    p.w_rw[pi.s] = pi.evict_due ? 0 : pi.w_att;
    if (p.budget && pi.nb + pi.w_att >= p.budget[pi.s]) p.live[pi.s] = 0;   // generation interrupted
  }
}

// Epilogue shared by both kernels: s_m/s_l/s_acc hold one (m, l, o) per wave in LDS;
// merge them in wave order and write the result or the chunk partial.
template <int NW, int D, int DOUT = D, int APITCH = D>
__device__ __forceinline__ void merge_waves_and_store(const DecodeParams& p, const PairInfo& pi,
                                                      const float* s_m, const float* s_l,
                                                      const float* s_acc, int ml_stride,
                                                      int acc_stride, int col0 = 0) {
  // APITCH: floats between the accumulator rows of two heads in s_acc
  // ml_stride, acc_stride: floats between the entries of two waves in s_m / s_l and in s_acc
  // D: columns this workgroup holds (all DOUT of a head, or one half starting at col0)
  const int nout = p.g * D;
  const int pair = pi.s * p.Hkv + pi.kvh;
  float* po = p.part_o + ((int64_t)pair * p.max_chunks + pi.chunk) * (p.Gp * D);
  float* pml = p.part_ml + ((int64_t)pair * p.max_chunks + pi.chunk) * (2 * p.Gp);
  float* outp = p.out + (int64_t)(pi.s * p.Hq + pi.kvh * p.g) * DOUT + col0;
  // (NW * 64 threads: the block size read from the launch descriptor would be one more scalar-cache miss)
  for (int i = threadIdx.x; i < nout; i += NW * 64) {
    const int h = i / D, x = i - h * D;
    float mx = s_m[h];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) mx = fmaxf(mx, s_m[wv * ml_stride + h]);
    float lsum = 0.f, o = 0.f;
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      const float a = fast_exp2(s_m[wv * ml_stride + h] - mx);
      lsum += s_l[wv * ml_stride + h] * a;
      o += s_acc[wv * acc_stride + h * APITCH + x] * a;
    }
    if (pi.nchunks == 1) {
      __builtin_nontemporal_store(o / lsum, outp + (D == DOUT ? i : h * DOUT + x));   // streamed out: nothing left dirty in L2
    } else {
      __builtin_nontemporal_store(o, po + i);
      if (x == 0) {
        __builtin_nontemporal_store(mx, pml + h);
        __builtin_nontemporal_store(lsum, pml + p.Gp + h);
      }
    }
  }
}

// The same merge, four output columns per thread (128-bit LDS reads and stores): fewer waves
// take part, which shortens this serial tail of the matrix-core kernel.
template <int NW, int D, int DOUT, int APITCH>
__device__ __forceinline__ void merge_waves_and_store4(const DecodeParams& p, const PairInfo& pi,
                                                       const float* s_m, const float* s_l,
                                                       const float* s_acc, int wave_stride, int col0) {
  constexpr int Q = D / 4;                       // column quads per head
  const int nitems = p.g * Q;
  const int pair = pi.s * p.Hkv + pi.kvh;
  float* po = p.part_o + ((int64_t)pair * p.max_chunks + pi.chunk) * (p.Gp * D);
  float* pml = p.part_ml + ((int64_t)pair * p.max_chunks + pi.chunk) * (2 * p.Gp);
  float* outp = p.out + (int64_t)(pi.s * p.Hq + pi.kvh * p.g) * DOUT + col0;
  for (int i = threadIdx.x; i < nitems; i += NW * 64) {
    const int h = i / Q, x = (i - h * Q) * 4;
    // all reads first: the merge is one LDS round trip, not one per wave
    float mw[NW], lw[NW];
    f32x4_t ow[NW];
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      mw[wv] = s_m[wv * wave_stride + h];
      lw[wv] = s_l[wv * wave_stride + h];
      ow[wv] = *reinterpret_cast<const f32x4_t*>(s_acc + wv * wave_stride + h * APITCH + x);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    float mx = mw[0];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) mx = fmaxf(mx, mw[wv]);
    float lsum = 0.f;
    f32x4_t o = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      const float a = fast_exp2(mw[wv] - mx);
      lsum += lw[wv] * a;
      o += ow[wv] * a;
    }
    if (pi.nchunks == 1) {
      const float inv = __builtin_amdgcn_rcpf(lsum);      // (one rounding error of the hardware reciprocal)
      __builtin_nontemporal_store(o * inv, reinterpret_cast<f32x4_t*>(outp + h * DOUT + x));
    } else {
      __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(po + h * D + x));
      if (x == 0) {
        __builtin_nontemporal_store(mx, pml + h);
        __builtin_nontemporal_store(lsum, pml + p.Gp + h);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// bf16, d = 128 or 64: LDS-DMA tiles + MFMA
// ---------------------------------------------------------------------------
constexpr int kLdsWaves = 8;           // waves per workgroup
constexpr int kLdsWavesSplit = 12;     // ... of the two-workgroups-per-pair form on short caches (12 KB of LDS per wave)
constexpr int kSplitWaves12MaxCap = 1100;   // rows: beyond this eight waves are as fast or faster (measured)
constexpr int kTileRows = 32;          // rows per wave tile
constexpr int kLdsBytes = kLdsWaves * 2 * kTileRows * 256;   // d = 128: 128 KB (half of it for d = 64)
constexpr int kLdsBytesSplit = kLdsWavesSplit * 3 * kTileRows * 128;   // K tile + half a V tile per wave: 144 KB
constexpr int kLdsBytesMax = kLdsBytesSplit > kLdsBytes ? kLdsBytesSplit : kLdsBytes;

typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

// K/V rows are read exactly once per launch: they are loaded with the non-temporal cache policy
// (the `nt` bit of the load instructions), which measured 5 % faster per step than the default
// policy at config 2.
constexpr int kStreamMinWorkgroups = 48;

template <bool STREAM> __device__ __forceinline__ uint4 load16(const char* p);
template <> __device__ __forceinline__ uint4 load16<false>(const char* p) {
  return *reinterpret_cast<const uint4*>(p);
}
__device__ __forceinline__ uint4 load16_stream(const char* p) {
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
  const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(r.x, r.y, r.z, r.w);
}

template <> __device__ __forceinline__ uint4 load16<true>(const char* p) { return load16_stream(p); }

// STREAM: 1 = load K and V with the non-temporal policy (large launches; small ones are
// latency-bound and about a microsecond faster with the default policy, 0); 2 = V only: with two
// workgroups per pair and long caches the K lines, which the partner reads a little later, are
// better kept cacheable.
// VS: workgroups per (sequence, KV head) pair.  With VS = 2 (batches of at most 128 pairs, which
// would leave half of the compute units idle) two workgroups serve a pair: both read all K rows
// and compute the same scores and weights, each reads one half of every V row and produces that
// half of the output columns - no partial results to merge.  The partner's workgroup index is
// larger by the number of pairs, which is the same XCD (same L2) when that number is a
// multiple of 8: the K rows then come from HBM once.
// NW: waves per workgroup, 8 or (two workgroups per pair, short caches: every wave then has one or
// two tiles, and twelve waves finish a sequence of up to 384 rows in one pass) 12.
// SHORT: every wave has at most two tiles (the caller's max_cap is at most 2 * NW * 32 rows, one
// chunk per pair, no dispatch order).  The code is then a straight line: query and appended row
// are requested first (their addresses do not need the tables), then the K part of the first
// tile, its V part, and the second tile's K and V parts into registers - everything in flight
// from the start, in the order it is needed - and every stage waits only for what it is about to
// read: scores and softmax of a tile run while its V rows are still on their way, so that behind
// the last byte only one value product is left.
template <int STREAM, int D, int VS, int NW, bool SHORT = false>
__global__ __launch_bounds__(NW * 64) void decode_lds_kernel(DecodeParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  constexpr bool KSTREAM = STREAM == 1, VSTREAM = STREAM >= 1;
  constexpr int DV = D / VS;               // V (and output) columns of this workgroup
  constexpr int VROWB = DV * 2;            // bytes of its part of a V row, = row pitch of the V tile in LDS
  constexpr int VUPR = VROWB / 16;
  constexpr int VRPI = 1024 / VROWB;
  constexpr int VNDMA = kTileRows / VRPI;
  constexpr int VTILEB = kTileRows * VROWB;
  constexpr int ROWB = D * 2;              // bytes of one row of one KV head: 256 or 128
  constexpr int UPR = ROWB / 16;           // 16-byte units per row: 16 or 8
  constexpr int RPI = 1024 / ROWB;         // rows one 1 KB LDS-DMA instruction brings: 4 or 8
  constexpr int NDMA = kTileRows / RPI;    // such instructions per K (or V) tile: 8 or 4
  constexpr int NI = D / 32;               // MFMAs (k = 32) along the head dimension: 4 or 2
  constexpr int NJ = DV / 16;              // 16-column blocks of the output held here: 8 or 4
  constexpr int TILEB = kTileRows * ROWB;  // one K (or V) tile: 8 or 4 KB
  touch_kernel_arguments();
  // grid: VS = 1: (chunk, KV head, slot); VS = 2: (KV head, slot, V half), the slots padded so
  // that a pair's two workgroups are 8k apart in dispatch order (workgroups go to the XCDs in turn)
  const int vhalf = VS == 1 ? 0 : (int)blockIdx.z;
  const int slot = VS == 1 ? (int)blockIdx.z : (int)blockIdx.y;
  const int kvh0 = VS == 1 ? (int)blockIdx.y : (int)blockIdx.x;
  if (VS != 1 && slot >= p.B) return;
  // (the wave's number as a scalar: conditions on it become real branches, not lane masks)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r4 = lane / UPR, pos = lane & (UPR - 1);   // row within a 1 KB load, unit within the row
  const int r4v = lane / VUPR, posv = lane & (VUPR - 1);   // the same for this workgroup's part of V
  const int n = lane & 15, kb = lane >> 4;       // MFMA column / k-block of this lane
  char* wk = lds + wave * (TILEB + VTILEB);
  char* wv = wk + TILEB;

  // B operand of the score product: Q^T, column n = query head, k = head-dim index.
  // The loads are written out by hand so that the compiler does not count them: it cannot tell
  // the order in which they and the LDS-DMA loads complete, and would put a wait for ALL
  // outstanding loads - the next tile's among them - in front of the first use in every pass of
  // the tile loop.  They are older than any tile load the wave waits for.
  bf16x8_t qb[NI];
  auto request_query = [&](int s_) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      __attribute__((ext_vector_type(4))) uint32_t r = {0u, 0u, 0u, 0u};
      if (n < p.g) {
        const char* src = p.q + ((int64_t)(s_ * p.Hq + kvh0 * p.g + n) * D + 32 * i + 8 * kb) * 2;
        asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(r) : "v"(src) : "memory");
      }
      qb[i] = __builtin_bit_cast(bf16x8_t, r);
    }
  };
  // Fused append: lanes 0..UPR-1 carry the new K row, the next VUPR lanes this workgroup's part of
  // the new V row (16 bytes each); loaded by hand like the query, for the same reason.  The
  // instruction is issued whether or not a row is appended (the other lanes, and all lanes of a
  // plain attention call, read the head of the query tensor instead): the waits below count it.
  u32x4_t newrow_v;
  auto request_new_row = [&](int s_) {
    const char* src = p.q + ((lane & 7) << 4);      // (128 bytes: inside the smallest query tensor)
    if (p.new_k != nullptr && lane < UPR + VUPR) {
      if constexpr (VS == 1)
        src = (lane < UPR ? p.new_k : p.new_v) + (int64_t)(s_ * p.Hkv + kvh0) * ROWB + ((lane & (UPR - 1)) << 4);
      else
        src = lane < UPR
            ? p.new_k + (int64_t)(s_ * p.Hkv + kvh0) * ROWB + (lane << 4)
            : p.new_v + (int64_t)(s_ * p.Hkv + kvh0) * ROWB + vhalf * VROWB + ((lane - UPR) << 4);
    }
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(newrow_v) : "v"(src) : "memory");
  };
  // HBM -> LDS: the K part of a tile (NDMA instructions, each RPI whole rows = 1 KB), then this
  // workgroup's V part, 16-byte units XOR-swizzled by the row.  Addresses are a base in scalar
  // registers plus a 32-bit offset per lane.  CLAMP: rows beyond `last_row` are read from
  // `last_row` instead (they are masked later; the loads stay inside the resident rows); without
  // it the tile's rows must all exist, and the lane offsets do not depend on the tile.
  const uint32_t wk_lds = lds_address(lds) + wave * (TILEB + VTILEB), wv_lds = wk_lds + TILEB;
  auto request_tile_dma = [&](auto clamp, uint64_t kb_, uint64_t vb_, int trow0, int last_row) {
    constexpr bool CLAMP = decltype(clamp)::value;
#pragma unroll
    for (int j = 0; j < NDMA; ++j) {
      const int row = RPI * j + r4;
      const uint32_t unit = (uint32_t)(pos ^ tile_swz<D>(row)) << 4;
      if constexpr (CLAMP)
        lds_dma16_s<KSTREAM>((uint32_t)min(trow0 + row, last_row) * ROWB + unit, kb_, wk_lds + j * 1024);
      else
        lds_dma16_s<KSTREAM>((uint32_t)r4 * ROWB + unit, kb_ + (uint64_t)(trow0 + RPI * j) * ROWB, wk_lds + j * 1024);
    }
#pragma unroll
    for (int j = 0; j < VNDMA; ++j) {
      const int vrow = VRPI * j + r4v;
      const uint32_t unit = (uint32_t)(posv ^ tile_swz<DV>(vrow)) << 4;
      if constexpr (CLAMP)
        lds_dma16_s<VSTREAM>((uint32_t)min(trow0 + vrow, last_row) * ROWB + unit, vb_, wv_lds + j * 1024);
      else
        lds_dma16_s<VSTREAM>((uint32_t)r4v * ROWB + unit, vb_ + (uint64_t)(trow0 + VRPI * j) * ROWB, wv_lds + j * 1024);
    }
  };
  // (not initialised, and written by request_tile_regs only: the loads are invisible to the
  // compiler, so a register-to-register copy between a load and its wait would copy what is not
  // there yet; the check of the generated code looks for exactly that)
  u32x4_t kreg[NDMA], vreg[VNDMA];
  auto request_tile_regs = [&](uint64_t kb_, uint64_t vb_, int trow0, int last_row) {
#pragma unroll
    for (int j = 0; j < NDMA; ++j)
      load16_uncounted_s<KSTREAM>(kreg[j], (uint32_t)min(trow0 + RPI * j + r4, last_row) * ROWB + (pos << 4), kb_);
#pragma unroll
    for (int j = 0; j < VNDMA; ++j)
      load16_uncounted_s<VSTREAM>(vreg[j], (uint32_t)min(trow0 + VRPI * j + r4v, last_row) * ROWB + (posv << 4), vb_);
  };
  if constexpr (SHORT) {            // the sequence is the slot: nothing here needs the tables
    request_query(slot);
    request_new_row(slot);
  }
  // Prompt rows never change and are always resident.  When the caller has promised the slab
  // geometry (every sequence: P = spec_P, cap = spec_cap, base = index * spec_cap), a wave whose
  // first tile lies inside the prompt requests it before the tables are back; whatever the
  // tables say afterwards decides: if the geometry is another, the tile is requested again.
  // (Requesting the tiles behind the prompt early as well, under a promised number of resident
  // rows, was measured: with everything asked for at once the step is 2 % slower.)
  bool early_tile = false;
  auto request_early_tiles = [&]() {
    if (p.spec_P > 0 && p.order == nullptr && p.max_chunks == 1 && (wave + 1) * kTileRows <= p.spec_P) {
      const int64_t off_ = ((int64_t)slot * p.spec_cap * p.Hkv + (int64_t)kvh0 * p.spec_cap) * ROWB;
      request_tile_dma(std::false_type{}, (uint64_t)(p.k_slab + off_), (uint64_t)(p.v_slab + off_ + vhalf * VROWB),
                       wave * kTileRows, 0);
      early_tile = true;
    }
  };
  const PairInfo pi = VS == 1 && !SHORT ? pair_info(p, slot, kvh0, (int)blockIdx.x)
                                        : pair_info(p, slot, kvh0, 0, request_early_tiles);
  // Tiles wave, wave + NW, ... of the chunk belong to this wave.
  const int ntiles = (pi.row_end - pi.row0 + kTileRows - 1) / kTileRows;
  bool nothing_to_do = !pi.live;
  if constexpr (SHORT) {
    // more rows than the caller's max_cap allows: no wave of the sequence goes on (none takes
    // a ticket, so its tables and the counters stay as they were)
    if (ntiles > 2 * NW) {
      if (pi.kvh == 0 && vhalf == 0 && tid == 0) atomicOr(p.err, BC_ERRBIT_STATE);
      nothing_to_do = true;
    }
  }
  if (nothing_to_do) { wait_vmcnt<0>(); return; }
  // rows the tile loads may touch: the resident rows that are already in the slab
  const int last_slab_row = max((pi.new_row >= 0 ? pi.new_row : pi.L) - 1, 0);
  if (early_tile && (pi.P != p.spec_P || pi.cap != p.spec_cap || pi.base != (int64_t)pi.s * p.spec_cap))
    early_tile = false;      // the promise does not hold here: the tile is requested again below

  const HalfSelectors sel = half_selectors();
  const int64_t stream_off = (pi.base * p.Hkv + (int64_t)pi.kvh * pi.cap) * ROWB;
  const char* kbase = p.k_slab + stream_off;
  const char* vbase = p.v_slab + stream_off + vhalf * VROWB;
  const uint64_t kbase_s = (uint64_t)kbase, vbase_s = (uint64_t)vbase;      // (uniform: scalar registers)
  if constexpr (!SHORT) {           // the sequence may come from the dispatch order: after the tables
    request_query(pi.s);
    request_new_row(pi.s);
  }

  f32x4_t O[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) O[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = kNegBig, l_run = 0.f;

  // A wave's first tile goes from HBM to LDS by LDS-DMA; the second is requested at the same
  // time into registers, so both are in flight from the start.  Afterwards: copy the register
  // tile to LDS, request the next tile into the freed registers, compute - one tile always in
  // flight behind the one in use.
  auto k_regs_to_lds = [&]() {
#pragma unroll
    for (int j = 0; j < NDMA; ++j) {
      const int row = RPI * j + r4;
      *reinterpret_cast<u32x4_t*>(wk + row * ROWB + ((pos ^ tile_swz<D>(row)) << 4)) = kreg[j];
    }
  };
  auto v_regs_to_lds = [&]() {
#pragma unroll
    for (int j = 0; j < VNDMA; ++j) {
      const int vrow = VRPI * j + r4v;
      *reinterpret_cast<u32x4_t*>(wv + vrow * VROWB + ((posv ^ tile_swz<DV>(vrow)) << 4)) = vreg[j];
    }
  };
  auto query_landed = [&]() {
#pragma unroll
    for (int i = 0; i < NI; ++i) landed(qb[i]);
    landed(newrow_v);
  };
  auto k_regs_landed = [&]() {
#pragma unroll
    for (int j = 0; j < NDMA; ++j) landed(kreg[j]);
  };
  auto v_regs_landed = [&]() {
#pragma unroll
    for (int j = 0; j < VNDMA; ++j) landed(vreg[j]);
  };
  if (wave < ntiles && !early_tile) {
    const int trow0 = pi.row0 + wave * kTileRows;
    if (trow0 + kTileRows <= last_slab_row + 1) request_tile_dma(std::false_type{}, kbase_s, vbase_s, trow0, 0);
    else request_tile_dma(std::true_type{}, kbase_s, vbase_s, trow0, last_slab_row);
  }

  // Fused step: every wave of every workgroup of the sequence takes a ticket as soon as its last
  // load from the slab has landed (the tables were read at the start); whoever draws the last one
  // may write the beacon row and update the tables.  The answer is only looked at after the wave
  // merge, so the atomic's round trip (about a microsecond) hides behind the remaining compute.
  int ticket = -1;
  auto take_ticket = [&]() {
    if (pi.update && lane == 0) {
      const int one_ = 1;
      asm volatile("global_atomic_add %0, %1, %2, off sc0"
                   : "=v"(ticket) : "v"(p.tickets + pi.s * kTicketStride), "v"(one_) : "memory");
    }
  };
  // The appended row is not in the slab yet: place it in the tile (K part before the scores, V
  // part before the value product), clear the V rows behind it, store it for later steps (unless
  // this step's eviction drops it at once).  Only the sequence's last tile can hold it.
  auto patch_k_row = [&](int trow0) {
    const int ra = pi.new_row - trow0;
    if (ra >= 0 && ra < kTileRows && lane < UPR)
      *reinterpret_cast<u32x4_t*>(wk + ra * ROWB + ((lane ^ tile_swz<D>(ra)) << 4)) = newrow_v;
  };
  auto patch_v_row_and_store = [&](int trow0) {
    const int ra = pi.new_row - trow0;
    if (ra < 0 || ra >= kTileRows) return;
    if (lane >= UPR && lane < UPR + VUPR) {
      const int u = lane - UPR;
      *reinterpret_cast<u32x4_t*>(wv + ra * VROWB + ((u ^ tile_swz<DV>(ra)) << 4)) = newrow_v;
      if (pi.store_new_row)
        *reinterpret_cast<u32x4_t*>(const_cast<char*>(vbase) + (int64_t)pi.new_row * ROWB + (u << 4)) = newrow_v;
    } else if (lane < UPR) {
      if (pi.store_new_row && vhalf == 0)
        *reinterpret_cast<u32x4_t*>(const_cast<char*>(kbase) + (int64_t)pi.new_row * ROWB + (lane << 4)) = newrow_v;
    }
    for (int rr = ra + 1 + r4v; rr < kTileRows; rr += VRPI)
      *reinterpret_cast<uint4*>(wv + rr * VROWB + (posv << 4)) = make_uint4(0u, 0u, 0u, 0u);
  };

  // ---- scores, transposed: S^T[key][head] = K . Q^T.  Row m of sub-tile t is key
  //      8*(m/4) + 4*t + m%4, so that a lane ends up with 8 consecutive keys of one head:
  //      lane (n, kb) holds head n, keys trow0 + 8*kb + e, e = 4*t + r.
  // ---- softmax: the scores stay unscaled; the softmax scale (>= 0) enters through one fused
  //      multiply-add per key, p = 2^(s*qs - m).  Only a sequence's last tile has rows beyond its
  //      end; the tests for them sit behind a branch that is uniform over the wave.  The weights
  //      leave as p = hi + lo with both parts bf16: the p.V product keeps ~16 bits of p.
  bf16x8_t phi, plo;
  auto scores_and_softmax = [&](int trow0, bool first) {
    f32x4_t S[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      S[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      const int row = ((n >> 2) << 3) + 4 * t + (n & 3);
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int u = 4 * i + kb;
        const bf16x8_t a =
            *reinterpret_cast<const bf16x8_t*>(wk + row * ROWB + ((u ^ tile_swz<D>(row)) << 4));
        S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[i], S[t], 0, 0, 0);
      }
    }
    const bool partial = trow0 + kTileRows > pi.row_end;
    const int nvalid = pi.row_end - trow0 - 8 * kb;        // keys e < nvalid of this lane exist
    float sv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sv[e] = S[e >> 2][e & 3];
    if (partial) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sv[e] = e < nvalid ? sv[e] : kNegBig;
    }
    float tmax = fmaxf(fmaxf(fmaxf(fmaxf(sv[0], sv[1]), sv[2]), fmaxf(fmaxf(sv[3], sv[4]), sv[5])),
                       fmaxf(sv[6], sv[7]));
    tmax = rows_allreduce_max(tmax);
    const float m_new = fmaxf(m_run, tmax * p.qscale);
    float pe[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) pe[e] = fast_exp2(fmaf(sv[e], p.qscale, -m_new));
    if (partial) {      // (with a scale of zero the fused form gives 1 for the missing keys, not 0)
#pragma unroll
      for (int e = 0; e < 8; ++e) pe[e] = e < nvalid ? pe[e] : 0.f;
    }
    const float psum = ((pe[0] + pe[1]) + (pe[2] + pe[3])) + ((pe[4] + pe[5]) + (pe[6] + pe[7]));
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const uint32_t hp = pack2_bf16(pe[e], pe[e + 1]);
      hi[e >> 1] = hp;
      lo[e >> 1] = pack2_bf16(minus_half(pe[e], hp, sel.low), minus_half(pe[e + 1], hp, sel.high));
    }
    // a wave's first tile finds empty accumulators: nothing to rescale
    if (!first) {
      const float alpha = fast_exp2(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int j = 0; j < NJ; ++j) O[j] *= alpha;
    }
    m_run = m_new;
    l_run += psum;
    phi = __builtin_bit_cast(bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
    plo = __builtin_bit_cast(bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
  };
  // ---- O^T[dcol][head] += V^T . P^T ; V^T comes from the transposing LDS read: lane r of a
  //      16-lane block points at 4 consecutive dcols of key 8*kb + r/4 (+4 for the 2nd read)
  auto value_product = [&]() {
    const int r = lane & 15;
    const int key0 = 8 * kb + (r >> 2);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int u = 2 * j + ((r & 3) >> 1);
      const int sub = (r & 1) << 3;
      const int rowa = key0, rowb = key0 + 4;
      const s16x4_t a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_t*)(wv + rowa * VROWB + ((u ^ tile_swz<DV>(rowa)) << 4) + sub));
      const s16x4_t a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_t*)(wv + rowb * VROWB + ((u ^ tile_swz<DV>(rowb)) << 4) + sub));
      typedef __attribute__((ext_vector_type(8))) short s16x8_t;
      const s16x8_t a = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8_t av = __builtin_bit_cast(bf16x8_t, a);
      O[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phi, O[j], 0, 0, 0);
      O[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plo, O[j], 0, 0, 0);
    }
  };

  if constexpr (SHORT) {
    // Loads in flight, oldest first: query (NI), appended row (1), K of the first tile (NDMA),
    // its V part (VNDMA) and, with a second tile, its K (NDMA) and V (VNDMA) into registers.
    const int trowA = wave * kTileRows, trowB = trowA + NW * kTileRows;
    if (wave >= ntiles) {
      wait_vmcnt<0>();          // query and row loads, before their registers are reused
      query_landed();
      take_ticket();
    } else if (wave + NW < ntiles) {
      request_tile_regs(kbase_s, vbase_s, trowB, last_slab_row);
      wait_vmcnt<VNDMA + NDMA + VNDMA>();          // K of the first tile is in LDS
      query_landed();
      scores_and_softmax(trowA, true);
      wait_vmcnt<NDMA + VNDMA>();                  // ... and its V part
      value_product();
      wait_vmcnt<VNDMA>();                         // K of the second tile is in registers
      k_regs_landed();
      k_regs_to_lds();
      patch_k_row(trowB);
      scores_and_softmax(trowB, false);
      wait_vmcnt<0>();
      v_regs_landed();
      v_regs_to_lds();
      patch_v_row_and_store(trowB);
      take_ticket();
      value_product();
    } else {
      wait_vmcnt<VNDMA>();
      query_landed();
      patch_k_row(trowA);
      scores_and_softmax(trowA, true);
      wait_vmcnt<0>();
      patch_v_row_and_store(trowA);
      take_ticket();
      value_product();
    }
  } else {
    if (wave >= ntiles) {
      wait_vmcnt<0>();          // the query loads, before their registers are reused
      query_landed();
      take_ticket();
    } else {
      for (int tile = wave;; tile += NW) {
        const int trow0 = pi.row0 + tile * kTileRows;
        if (tile + NW < ntiles) {
          // the next tile of this wave goes to registers while this one is in use; the tile in
          // use has landed once at most those loads are pending
          request_tile_regs(kbase_s, vbase_s, trow0 + NW * kTileRows, last_slab_row);
          wait_vmcnt<NDMA + VNDMA>();
          query_landed();
          scores_and_softmax(trow0, tile == wave);
          value_product();
          wait_vmcnt<0>();
          k_regs_landed();
          v_regs_landed();
          k_regs_to_lds();
          v_regs_to_lds();
        } else {
          // this wave's last tile: nothing between here and the end of the kernel waits for
          // memory, so the ticket's answer can stay out
          wait_vmcnt<0>();
          query_landed();
          patch_k_row(trow0);
          patch_v_row_and_store(trow0);
          take_ticket();
          scores_and_softmax(trow0, tile == wave);
          value_product();
          break;
        }
      }
    }
  }

  // denominators: sum the four k-blocks of each head
  l_run = rows_allreduce_sum(l_run);

  // ---- merge the waves through LDS.  Every wave leaves its (m, l, o) at the start of its own
  // tile region, which nobody else touches, as soon as it is done: one barrier, and the early
  // waves' writes do not wait for the late ones.
  // (rows of DV floats would all start on the same LDS bank: a pitch of DV + 4 floats spreads the
  // 128-bit writes of the up to eight heads over the banks)
  constexpr int APITCH = DV + 4;
  constexpr int WSTRIDE = (TILEB + VTILEB) / 4;                   // floats between two waves' regions
  static_assert((8 * APITCH + 16 + 1) * 4 <= TILEB + VTILEB, "the partial fits the wave's region");
  float* s_acc = reinterpret_cast<float*>(lds);                    // wave w: [8][APITCH] at w * WSTRIDE
  float* s_m = s_acc + 8 * APITCH;                                 //         [8] behind it
  float* s_l = s_m + 8;
  if (n < p.g) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      *reinterpret_cast<f32x4_t*>(s_acc + wave * WSTRIDE + n * APITCH + 16 * j + 4 * kb) = O[j];
    if (kb == 0) { s_m[wave * WSTRIDE + n] = m_run; s_l[wave * WSTRIDE + n] = l_run; }
  }
  __syncthreads();
  merge_waves_and_store4<NW, DV, D, APITCH>(p, pi, s_m, s_l, s_acc, WSTRIDE, vhalf * DV);

  // ---- the wave that drew the sequence's last ticket writes the beacon row and updates the tables
  if (!pi.update) return;
  wait_vmcnt<0>();     // the ticket has arrived
  landed(ticket);
  if (__builtin_amdgcn_readfirstlane(ticket) != p.Hkv * pi.nchunks * VS * NW - 1) return;
  finish_step<ROWB>(p, pi, lane);
}

// ---------------------------------------------------------------------------
// generic VALU kernel: fp32 rows and d = 64
// ---------------------------------------------------------------------------
constexpr int kValuWaves = 4;

template <typename T, int D, int G, int U>
__global__ __launch_bounds__(256) void decode_valu_kernel(DecodeParams p) {
  constexpr int ES = Elem<T>::size;
  constexpr int EPL = Elem<T>::per16;   // elements per lane per row
  constexpr int LPR = D / EPL;          // lanes per row
  constexpr int RPI = 64 / LPR;         // rows per wave load instruction
  constexpr int RB = D * ES;            // row bytes
  constexpr int ROWS_PER_PASS = kValuWaves * RPI * U;

  touch_kernel_arguments();
  const PairInfo pi = pair_info(p, (int)blockIdx.z, (int)blockIdx.y, (int)blockIdx.x);
  if (!pi.live) return;
  const int L = pi.L, row_end = pi.row_end;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane / LPR, ls = lane - lr * LPR;
  const int64_t stream_off = (pi.base * p.Hkv + (int64_t)pi.kvh * pi.cap) * RB + ls * 16;
  const char* kbase = p.k_slab + stream_off;
  const char* vbase = p.v_slab + stream_off;

  // q slice of every head of the group, pre-scaled so that exp() becomes exp2()
  float qf[G][EPL];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    if (h < p.g) {
      const uint4 r = *reinterpret_cast<const uint4*>(
          p.q + ((int64_t)(pi.s * p.Hq + pi.kvh * p.g + h) * D) * ES + ls * 16);
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

  // Fused step: the appended row (always the sequence's last) is not in the slab yet.  The loop
  // below covers the rows that are; the workgroup whose chunk holds the appended row takes it
  // from the caller's tensors in a pass of its own behind the loop and stores it for later steps
  // (unless this step's eviction drops it at once).  No reader touches the slab at that row in
  // this launch, so the store races with nothing.
  const bool new_row_here = pi.new_row >= pi.row0 && pi.new_row < row_end;      // (uniform)
  const int slab_end = new_row_here ? pi.new_row : row_end;

  for (int pr = pi.row0 + wave * (RPI * U); pr < slab_end; pr += ROWS_PER_PASS) {
    uint4 kk[U], vv[U];
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = pr + u * RPI + lr;
      valid[u] = r < slab_end;
      const int rc = valid[u] ? r : (slab_end - 1);  // stay inside the resident rows
      kk[u] = load16_stream(kbase + (int64_t)rc * RB);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = pr + u * RPI + lr;
      const int rc = valid[u] ? r : (slab_end - 1);
      vv[u] = load16_stream(vbase + (int64_t)rc * RB);
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
      const float alpha = fast_exp2(m[h] - mn);
      m[h] = mn;
      l[h] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[h][e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float pw = valid[u] ? fast_exp2(sc[u][h] - mn) : 0.f;
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

  if (new_row_here && wave == 0) {
    // the appended row: one more row for the first lane group of the first wave
    const int64_t at = (int64_t)(pi.s * p.Hkv + pi.kvh) * RB + ls * 16;
    const uint4 kq = *reinterpret_cast<const uint4*>(p.new_k + at);
    const uint4 vq = *reinterpret_cast<const uint4*>(p.new_v + at);
    if (pi.store_new_row && lr == 0) {
      *reinterpret_cast<uint4*>(const_cast<char*>(kbase) + (int64_t)pi.new_row * RB) = kq;
      *reinterpret_cast<uint4*>(const_cast<char*>(vbase) + (int64_t)pi.new_row * RB) = vq;
    }
    float kf[EPL], vf[EPL];
    unpack16(kq, kf, T{});
    unpack16(vq, vf, T{});
    const bool mine = lr == 0;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float a = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) a = fmaf(qf[h][e], kf[e], a);
      a = group_allreduce_sum<LPR>(a);
      const float sc1 = mine ? a : kNegBig;
      const float mn = fmaxf(m[h], sc1);
      const float alpha = fast_exp2(m[h] - mn);
      const float pw = mine ? fast_exp2(sc1 - mn) : 0.f;
      m[h] = mn;
      l[h] = l[h] * alpha + pw;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(pw, vf[e], acc[h][e] * alpha);
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
      const float a = fast_exp2(m[h] - mn), b = fast_exp2(mo - mn);
      m[h] = mn;
      l[h] = l[h] * a + lo * b;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float ao = __shfl_xor(acc[h][e], off, 64);
        acc[h][e] = acc[h][e] * a + ao * b;
      }
    }
  }

  __shared__ float s_acc[kValuWaves * G * D];
  __shared__ float s_m[kValuWaves * G], s_l[kValuWaves * G];
  if (lr == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_acc[(wave * G + h) * D + ls * EPL + e] = acc[h][e];
      if (ls == 0) { s_m[wave * G + h] = m[h]; s_l[wave * G + h] = l[h]; }
    }
  }
  __syncthreads();
  // Fused step: one ticket per workgroup, taken once all its waves have used the rows they read
  // (the barrier above); the answer comes back under the merge.  The workgroup that draws the
  // sequence's last one finishes the step.
  int ticket = -1;
  if (pi.update && tid == 0) ticket = atomicAdd(p.tickets + pi.s * kTicketStride, 1);
  merge_waves_and_store<kValuWaves, D>(p, pi, s_m, s_l, s_acc, G, G * D);
  if (!pi.update || wave != 0) return;
  if (__builtin_amdgcn_readfirstlane(ticket) != p.Hkv * pi.nchunks - 1) return;
  finish_step<RB>(p, pi, lane);
}

// ---------------------------------------------------------------------------
// chunk merge: one workgroup per pair, partials combined in chunk order
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void decode_merge_kernel(DecodeParams p) {
  const int pair = blockIdx.x;
  const int s = pair / p.Hkv, kvh = pair - s * p.Hkv;
  const int nchunks = p.part_n[pair];             // 0: nothing to do, 1: already final
  if (nchunks <= 1) return;
  const int D = p.D;
  const float* ao = p.part_o + (int64_t)pair * p.max_chunks * (p.Gp * D);
  const float* aml = p.part_ml + (int64_t)pair * p.max_chunks * (2 * p.Gp);
  float* outp = p.out + (int64_t)(s * p.Hq + kvh * p.g) * D;
  const int nout = p.g * D;
  // chunks are folded in order, sixteen at a time: the loads of a batch are independent and in
  // flight together (the partials come from memory, not from this compute unit's caches)
  constexpr int kBatch = 16;
  for (int i = threadIdx.x; i < nout; i += 256) {
    const int h = i / D;
    float mx = kNegBig, lsum = 0.f, o = 0.f;
    for (int ch0 = 0; ch0 < nchunks; ch0 += kBatch) {
      float mv[kBatch], lv[kBatch], ov[kBatch];
#pragma unroll
      for (int k = 0; k < kBatch; ++k) {
        const int ch = min(ch0 + k, nchunks - 1);
        mv[k] = __builtin_nontemporal_load(aml + ch * 2 * p.Gp + h);
        lv[k] = __builtin_nontemporal_load(aml + ch * 2 * p.Gp + p.Gp + h);
        ov[k] = __builtin_nontemporal_load(ao + (int64_t)ch * (p.Gp * D) + i);
      }
      float bm = kNegBig;
#pragma unroll
      for (int k = 0; k < kBatch; ++k) {
        if (ch0 + k >= nchunks) mv[k] = kNegBig;
        bm = fmaxf(bm, mv[k]);
      }
      const float mn = fmaxf(mx, bm);
      const float keep = fast_exp2(mx - mn);
      lsum *= keep; o *= keep; mx = mn;
#pragma unroll
      for (int k = 0; k < kBatch; ++k) {
        const float a = (ch0 + k < nchunks) ? fast_exp2(mv[k] - mx) : 0.f;
        lsum += lv[k] * a;
        o += ov[k] * a;
      }
    }
    outp[i] = o / lsum;
  }
}

struct DecodePlan {
  bool lds;           // LDS/MFMA kernel (bf16, d = 128) or the VALU kernel
  int Gp;             // padded group size
  int rows_per_pass;  // rows one pass of a workgroup covers
  int R;              // rows per workgroup
  int max_chunks;
  size_t tickets_bytes, part_n_bytes, part_o_bytes, part_ml_bytes;
  size_t total() const { return tickets_bytes + part_n_bytes + part_o_bytes + part_ml_bytes; }
};

static int padded_group(int g) { return g <= 1 ? 1 : g <= 2 ? 2 : g <= 4 ? 4 : g <= 6 ? 6 : 8; }
static size_t align256(size_t x) { return (x + 255) / 256 * 256; }

constexpr int kPlanForSizing = -1;    // rows_override value: size the workspace (see below)

static DecodePlan make_plan(const bc_shape* sh, int max_cap, int rows_override, int plan_bits) {
  DecodePlan pl;
  pl.lds = sh->kv_dtype == BC_BF16 && !(plan_bits & BC_PLAN_PLAIN_ALU);
  if (pl.lds) {
    pl.Gp = 8;
    pl.rows_per_pass = kLdsWaves * kTileRows;
  } else {
    pl.Gp = padded_group(sh->Hq / sh->Hkv);
    const int epl = 16 / elem_size(sh->kv_dtype);
    const int lpr = sh->d / epl, rpi = 64 / lpr;
    pl.rows_per_pass = kValuWaves * rpi * 8;
  }
  const long npairs = (long)sh->B * sh->Hkv;
  if (rows_override > 0) {
    // forced chunk size (experiments, tests): fixed rows per workgroup
    int R = ((rows_override + pl.rows_per_pass - 1) / pl.rows_per_pass) * pl.rows_per_pass;
    while ((max_cap + R - 1) / R > 64) R += pl.rows_per_pass;   // bound the partials per pair
    pl.R = R;
    pl.max_chunks = (max_cap + R - 1) / R;
  } else {
    // One workgroup per (sequence, KV head) pair when there are enough pairs: a long-running
    // workgroup streams its rows at full rate and needs no merge launch.  With few pairs the
    // rows of a sequence are spread over enough workgroups to fill the chip (256 compute units),
    // at least kMinChunkRows rows each, at most 64 chunks - but only when the longest stream
    // gets shorter by more than the merge launch costs (about 6 us, some 480 rows of one stream).
    long chunks = 1;
    if (npairs < 128) {
      chunks = (256 + npairs - 1) / npairs;
      const long by_rows = max_cap / kMinChunkRows;
      if (chunks > by_rows) chunks = by_rows;
      if (chunks > 64) chunks = 64;
      if (chunks < 1 || max_cap - max_cap / chunks < 480) chunks = 1;
    }
    pl.R = 0;                                        // spread evenly, decided per sequence
    pl.max_chunks = (int)chunks;
  }
  // Workspace sizing: the most chunks the automatic plan can choose (64 with few pairs, one
  // otherwise); a forced chunk size on a large batch may use up to four.
  if (rows_override == kPlanForSizing) pl.max_chunks = npairs < 128 ? 64 : 4;
  const size_t pairs = (size_t)sh->B * sh->Hkv;
  pl.tickets_bytes = align256((size_t)sh->B * kTicketStride * 4);
  pl.part_n_bytes = align256(pairs * 4);
  pl.part_o_bytes = align256(pairs * pl.max_chunks * pl.Gp * sh->d * 4);
  pl.part_ml_bytes = align256(pairs * pl.max_chunks * 2 * pl.Gp * 4);
  return pl;
}

template <typename T, int D>
static void launch_valu(const DecodeParams& p, int G, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: decode_valu_kernel<T, D, 1, 8><<<grid, 256, 0, st>>>(p); break;
    case 2: decode_valu_kernel<T, D, 2, 8><<<grid, 256, 0, st>>>(p); break;
    case 4: decode_valu_kernel<T, D, 4, 8><<<grid, 256, 0, st>>>(p); break;
    case 6: decode_valu_kernel<T, D, 6, 8><<<grid, 256, 0, st>>>(p); break;
    default: decode_valu_kernel<T, D, 8, 8><<<grid, 256, 0, st>>>(p); break;
  }
}

// Which instantiation of the LDS/MFMA kernel serves a call, with its launch shape.  `name` is the
// kernel's name as profilers print it.
struct LdsLaunch {
  void (*fn)(DecodeParams);
  const char* name;
  dim3 grid;
  int threads;
  int lds_bytes;
};
#define BC_LDS_KERNEL(...) decode_lds_kernel<__VA_ARGS__>, "bc::decode_lds_kernel<" #__VA_ARGS__ ">"

static LdsLaunch pick_lds_kernel(const bc_shape* shape, const bc_cache* cache, const DecodePlan& pl,
                                 bool ordered) {
  const int pairs = shape->B * shape->Hkv;
  const dim3 grid(pl.max_chunks, shape->Hkv, shape->B);
  // launches that cannot saturate the memory system are latency-bound: default cache policy
  const bool cacheable = (cache->plan & BC_PLAN_CACHEABLE_LOADS) != 0;
  const bool general = (cache->plan & BC_PLAN_GENERAL_LOOP) != 0;
  const bool stream = (long)pairs * pl.max_chunks >= kStreamMinWorkgroups && !cacheable;
  // at most two tiles per wave of an eight-wave workgroup: the straight-line form of the kernel
  const bool two8 = pl.max_chunks == 1 && !ordered && !general && cache->max_cap <= 2 * kLdsWaves * kTileRows;
  // two workgroups per pair (each one half of the V columns) while that still fits the chip
  int slots = shape->B;                   // padded until the pairs are a multiple of 8
  while ((slots * shape->Hkv) & 7) ++slots;
  const bool vsplit = shape->d == 128 && pl.max_chunks == 1 && 2 * slots * shape->Hkv <= kLptMinPairs &&
                      !(cache->plan & BC_PLAN_ONE_WORKGROUP_PER_PAIR);
  if (vsplit) {
    // K lines are read by both workgroups of a pair: streamed while the batch's K is small
    // enough for the partner's request to find the line still on its way or in the L2
    // (measured up to about 48 MB), cacheable beyond
    const bool stream2 = 2L * pairs >= kStreamMinWorkgroups && !cacheable;
    const bool small_k = (int64_t)pairs * cache->max_cap * 256 <= (48LL << 20);
    // short caches: twelve waves (most sequences then need one pass); long ones: eight
    const bool w12 = cache->max_cap <= kSplitWaves12MaxCap;
    const bool two12 = w12 && cache->max_cap <= 2 * kLdsWavesSplit * kTileRows && !general;
    const dim3 g2(shape->Hkv, slots, 2);
    const int t12 = kLdsWavesSplit * 64, l12 = kLdsBytesSplit, t8 = kLdsWaves * 64, l8 = kLdsWaves * 3 * kTileRows * 128;
    if (two12) return stream2 ? LdsLaunch{BC_LDS_KERNEL(1, 128, 2, 12, true), g2, t12, l12}
                              : LdsLaunch{BC_LDS_KERNEL(0, 128, 2, 12, true), g2, t12, l12};
    if (!stream2) return w12 ? LdsLaunch{BC_LDS_KERNEL(0, 128, 2, 12), g2, t12, l12}
                             : LdsLaunch{BC_LDS_KERNEL(0, 128, 2, 8), g2, t8, l8};
    if (small_k) return w12 ? LdsLaunch{BC_LDS_KERNEL(1, 128, 2, 12), g2, t12, l12}
                            : LdsLaunch{BC_LDS_KERNEL(1, 128, 2, 8), g2, t8, l8};
    return LdsLaunch{BC_LDS_KERNEL(2, 128, 2, 8), g2, t8, l8};
  }
  if (shape->d == 128) {
    // More pairs than the chip holds workgroups, and short caches: workgroups of four waves, two
    // per compute unit (64 KB of LDS each), so that one's start and end phases - tables, first
    // bytes, merge, store - overlap with the other's streaming.  Measured at 512 pairs of 512
    // rows: 28.2 -> 25.4 us; with long ragged sequences (512 pairs of up to 2700 rows) the longest
    // streams set the pace and eight waves are faster (54.5 against 62.5 us).
    const bool four = pairs > kLptMinPairs && cache->max_cap <= kSplitWaves12MaxCap && stream &&
                      !(cache->plan & BC_PLAN_NO_SMALL_WORKGROUPS);
    if (four) return LdsLaunch{BC_LDS_KERNEL(1, 128, 1, 4), grid, 4 * 64, kLdsBytes / 2};
    if (two8) return stream ? LdsLaunch{BC_LDS_KERNEL(1, 128, 1, 8, true), grid, kLdsWaves * 64, kLdsBytes}
                            : LdsLaunch{BC_LDS_KERNEL(0, 128, 1, 8, true), grid, kLdsWaves * 64, kLdsBytes};
    return stream ? LdsLaunch{BC_LDS_KERNEL(1, 128, 1, 8), grid, kLdsWaves * 64, kLdsBytes}
                  : LdsLaunch{BC_LDS_KERNEL(0, 128, 1, 8), grid, kLdsWaves * 64, kLdsBytes};
  }
  if (two8) return stream ? LdsLaunch{BC_LDS_KERNEL(1, 64, 1, 8, true), grid, kLdsWaves * 64, kLdsBytes / 2}
                          : LdsLaunch{BC_LDS_KERNEL(0, 64, 1, 8, true), grid, kLdsWaves * 64, kLdsBytes / 2};
  return stream ? LdsLaunch{BC_LDS_KERNEL(1, 64, 1, 8), grid, kLdsWaves * 64, kLdsBytes / 2}
                : LdsLaunch{BC_LDS_KERNEL(0, 64, 1, 8), grid, kLdsWaves * 64, kLdsBytes / 2};
}

// The LDS kernel needs 128 KB of dynamic LDS: opt in once per device.  Two host threads that get
// here together both set the (same) attributes; the flag only saves the later calls.
static int32_t enable_big_lds() {
  static std::atomic<bool> done[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BC_ERR_HIP;
  if (done[dev].load(std::memory_order_acquire)) return BC_OK;
  const void* kernels[] = {reinterpret_cast<const void*>(decode_lds_kernel<1, 128, 1, 4>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 128, 1, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 128, 1, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 128, 1, 8, true>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 128, 1, 8, true>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 64, 1, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 64, 1, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 64, 1, 8, true>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 64, 1, 8, true>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 128, 2, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 128, 2, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<2, 128, 2, 8>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 128, 2, 12>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 128, 2, 12>),
                           reinterpret_cast<const void*>(decode_lds_kernel<0, 128, 2, 12, true>),
                           reinterpret_cast<const void*>(decode_lds_kernel<1, 128, 2, 12, true>)};
  bool ok = true;
  for (const void* kfn : kernels)
    ok = ok && hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesMax) ==
                   hipSuccess;
  if (!ok)
    return BC_ERR_HIP;
  done[dev].store(true, std::memory_order_release);
  return BC_OK;
}

__global__ void fill_zero_kernel(uint32_t* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    p[i] = 0u;
}

// Batches that need more than one round of workgroups follow the caller's dispatch order
// (bc_sort_by_length), if there is one; with fewer workgroups everything starts at once.
static bool follows_order(const bc_shape* shape, const bc_cache* cache, const DecodePlan& pl) {
  return cache->order && pl.max_chunks == 1 && shape->B * shape->Hkv > kLptMinPairs &&
         !(cache->plan & BC_PLAN_IGNORE_ORDER);
}

// Attention launch shared by bc_decode_attn (k = beacon_k = NULL) and the fused bc_decode_step.
static int32_t launch_attention(const bc_shape* shape, const bc_cache* cache, const DecodePlan& pl,
                                const void* q, float* out, const uint8_t* active, void* workspace,
                                const void* k, const void* v, const void* bk, const void* bv,
                                hipStream_t hs, const int32_t* budget = nullptr,
                                uint8_t* live = nullptr, bool beacon_row = false) {
  DecodeParams p;
  p.k_slab = static_cast<const char*>(cache->k_slab);
  p.v_slab = static_cast<const char*>(cache->v_slab);
  p.base = cache->base; p.cap = cache->cap; p.P = cache->P; p.nb = cache->nb; p.w = cache->w;
  p.err = cache->err;
  p.q = static_cast<const char*>(q);
  p.out = out;
  p.active = active;
  char* ws = static_cast<char*>(workspace);
  p.tickets = reinterpret_cast<int32_t*>(ws);
  char* parts = ws + pl.tickets_bytes;
  p.part_n = pl.max_chunks > 1 ? reinterpret_cast<int32_t*>(parts) : nullptr;
  p.part_o = reinterpret_cast<float*>(parts + pl.part_n_bytes);
  p.part_ml = reinterpret_cast<float*>(parts + pl.part_n_bytes + pl.part_o_bytes);
  p.c = cache->c; p.nb_rw = cache->nb; p.w_rw = cache->w;
  p.new_k = static_cast<const char*>(k); p.new_v = static_cast<const char*>(v);
  p.bk = static_cast<const char*>(bk); p.bv = static_cast<const char*>(bv);
  p.budget = budget; p.live = live;
  p.beacon_row = beacon_row ? 1 : 0;
  p.B = shape->B;
  p.order = follows_order(shape, cache, pl) ? cache->order : nullptr;
  p.Hq = shape->Hq; p.Hkv = shape->Hkv; p.g = shape->Hq / shape->Hkv;
  p.Gp = pl.Gp;
  p.D = shape->d;
  p.rows_per_wg = pl.R;
  p.max_chunks = pl.max_chunks;
  p.qscale = shape->scale * kLog2e;
  p.spec_P = (cache->plan & BC_PLAN_IGNORE_PROMISE) ? 0 : cache->uniform_P;
  p.spec_cap = cache->uniform_cap;

  const int pairs = shape->B * shape->Hkv;
  const dim3 grid(pl.max_chunks, shape->Hkv, shape->B);
  if (pl.lds) {
    const int32_t st = enable_big_lds();
    if (st != BC_OK) return st;
    const LdsLaunch k = pick_lds_kernel(shape, cache, pl, p.order != nullptr);
    k.fn<<<k.grid, k.threads, k.lds_bytes, hs>>>(p);
  } else if (shape->kv_dtype == BC_BF16) {
    if (shape->d == 128) launch_valu<bf16_t, 128>(p, pl.Gp, grid, hs);
    else launch_valu<bf16_t, 64>(p, pl.Gp, grid, hs);
  } else {
    if (shape->d == 128) launch_valu<float, 128>(p, pl.Gp, grid, hs);
    else launch_valu<float, 64>(p, pl.Gp, grid, hs);
  }
  if (pl.max_chunks > 1) decode_merge_kernel<<<pairs, 256, 0, hs>>>(p);
  return launch_status();
}

static int32_t check_attention_args(const bc_shape* shape, const bc_cache* cache, const void* q,
                                    const float* out, const void* workspace, size_t workspace_bytes,
                                    DecodePlan* pl) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return BC_ERR_ARG;
  if (shape->B > 65535 || shape->Hkv > 65535) return BC_ERR_SHAPE;      // grid dimensions
  if (!nonnegative_finite(shape->scale)) return BC_ERR_ARG;   // the kernels take maxima of unscaled scores
  if (cache->rows_per_workgroup < 0 || (cache->plan & ~BC_PLAN_ALL_BITS)) return BC_ERR_ARG;
  *pl = make_plan(shape, cache->max_cap, cache->rows_per_workgroup, cache->plan);
  if ((cache->plan & BC_PLAN_NEED_MATRIX_KERNEL) && !pl->lds) return BC_ERR_SHAPE;
  if (!workspace || !aligned16(workspace) || workspace_bytes < pl->total()) return BC_ERR_WORKSPACE;
  return BC_OK;
}

}  // namespace bc

using namespace bc;

extern "C" int32_t bc_sort_by_length(const bc_shape* shape, const bc_cache* cache,
                                     const uint8_t* active, int32_t* order, void* stream) {
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (!order) return BC_ERR_ARG;
  if (shape->B > kLptMaxB) return BC_ERR_SHAPE;
  SortParams p;
  p.active = active; p.P = cache->P; p.nb = cache->nb; p.w = cache->w;
  p.order = order; p.B = shape->B;
  sort_by_length_kernel<<<(shape->B + 255) / 256, 256, 0, as_stream(stream)>>>(p);
  return launch_status();
}

extern "C" size_t bc_decode_workspace_bytes(const bc_shape* shape, int32_t max_cap) {
  if (check_shape(shape) != BC_OK || max_cap < 1) return 0;
  // sized for the largest number of chunks the automatic plan can select, for either kernel
  const DecodePlan a = make_plan(shape, max_cap, kPlanForSizing, 0),
                   b = make_plan(shape, max_cap, kPlanForSizing, BC_PLAN_PLAIN_ALU);
  return a.total() > b.total() ? a.total() : b.total();
}

extern "C" int32_t bc_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 3u)) return BC_ERR_ARG;
  const int64_t n = (int64_t)(workspace_bytes / 4);
  if (n == 0) return BC_OK;
  const int64_t blocks = (n + 255) / 256;
  fill_zero_kernel<<<(int)(blocks < 4096 ? blocks : 4096), 256, 0, as_stream(stream)>>>(
      static_cast<uint32_t*>(workspace), n);
  return launch_status();
}

extern "C" int32_t bc_decode_plan_describe(const bc_shape* shape, const bc_cache* cache, char* text,
                                           size_t text_bytes) {
  if (!text || text_bytes == 0) return BC_ERR_ARG;
  text[0] = 0;
  int32_t st = check_shape(shape);
  if (st != BC_OK) return st;
  st = check_cache(cache);
  if (st != BC_OK) return st;
  if (cache->rows_per_workgroup < 0 || (cache->plan & ~BC_PLAN_ALL_BITS)) return BC_ERR_ARG;
  const DecodePlan pl = make_plan(shape, cache->max_cap, cache->rows_per_workgroup, cache->plan);
  if ((cache->plan & BC_PLAN_NEED_MATRIX_KERNEL) && !pl.lds) return BC_ERR_SHAPE;
  if (pl.lds) {
    const LdsLaunch k = pick_lds_kernel(shape, cache, pl, follows_order(shape, cache, pl));
    snprintf(text, text_bytes, "%s grid=(%u,%u,%u) threads=%d lds=%d chunks=%d%s", k.name, k.grid.x,
             k.grid.y, k.grid.z, k.threads, k.lds_bytes, pl.max_chunks,
             pl.max_chunks > 1 ? " + bc::decode_merge_kernel" : "");
  } else {
    snprintf(text, text_bytes, "bc::decode_valu_kernel<%s, %d, %d, 8> grid=(%d,%d,%d) threads=256 chunks=%d%s",
             shape->kv_dtype == BC_BF16 ? "bc::bf16_t" : "float", shape->d, pl.Gp, pl.max_chunks,
             shape->Hkv, shape->B, pl.max_chunks, pl.max_chunks > 1 ? " + bc::decode_merge_kernel" : "");
  }
  return BC_OK;
}

extern "C" int32_t bc_decode_attn(const bc_shape* shape, const bc_cache* cache, const void* q,
                                  float* out, const uint8_t* active, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  DecodePlan pl;
  const int32_t st = check_attention_args(shape, cache, q, out, workspace, workspace_bytes, &pl);
  if (st != BC_OK) return st;
  return launch_attention(shape, cache, pl, q, out, active, workspace, nullptr, nullptr, nullptr,
                          nullptr, as_stream(stream));
}

// bc_decode_step behind its argument checks (shared with the allocation-free form)
static int32_t decode_step_checked(const bc_shape* shape, const bc_cache* cache, const DecodePlan& pl,
                                   const void* k, const void* v, const void* q, float* out,
                                   const void* beacon_k, const void* beacon_v, const uint8_t* active,
                                   void* workspace, void* stream) {
  if (!k || !v || !aligned16(k) || !aligned16(v)) return BC_ERR_ARG;
  if ((beacon_k == nullptr) != (beacon_v == nullptr)) return BC_ERR_ARG;
  if (beacon_k && (!aligned16(beacon_k) || !aligned16(beacon_v))) return BC_ERR_ARG;
  // one launch, whichever kernel serves the shape: append, attention and eviction fused
  return launch_attention(shape, cache, pl, q, out, active, workspace, k, v, beacon_k, beacon_v,
                          as_stream(stream));
}

extern "C" int32_t bc_decode_step(const bc_shape* shape, const bc_cache* cache, const void* k,
                                  const void* v, const void* q, float* out, const void* beacon_k,
                                  const void* beacon_v, const uint8_t* active, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  DecodePlan pl;
  const int32_t st = check_attention_args(shape, cache, q, out, workspace, workspace_bytes, &pl);
  if (st != BC_OK) return st;
  return decode_step_checked(shape, cache, pl, k, v, q, out, beacon_k, beacon_v, active, workspace, stream);
}

// ---------------------------------------------------------------------------
// bc_decode_step for callers that cannot allocate: the workspace is a fixed array in device memory
// ---------------------------------------------------------------------------
namespace bc {
constexpr size_t kScratchBytes = BC_NOALLOC_SCRATCH_BYTES;
// One copy per GPU the library runs on, at an address of its own, held until the process ends.
// (In host code the array's name is only a handle: its device address comes from
// hipGetSymbolAddress, once per device, below.)
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

static int32_t scratch_of_current_device(unsigned char** ptr) {
  static unsigned char* address[64];
  static std::atomic<bool> known[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BC_ERR_HIP;
  if (!known[dev].load(std::memory_order_acquire)) {
    void* a = nullptr;
    if (hipGetSymbolAddress(&a, HIP_SYMBOL(scratch)) != hipSuccess || a == nullptr) return BC_ERR_HIP;
    address[dev] = static_cast<unsigned char*>(a);      // (two threads racing here store the same value)
    known[dev].store(true, std::memory_order_release);
  }
  *ptr = address[dev];
  return BC_OK;
}
}  // namespace bc

extern "C" int32_t bc_decode_step_noalloc(const bc_shape* shape, const bc_cache* cache, const void* k,
                                          const void* v, const void* q, float* out, const void* beacon_k,
                                          const void* beacon_v, const uint8_t* active, void* stream) {
  // the checks of bc_decode_step (the workspace is checked below, against the scratch array)
  DecodePlan pl;
  int32_t st = check_attention_args(shape, cache, q, out, reinterpret_cast<void*>(uintptr_t(256)), SIZE_MAX, &pl);
  if (st != BC_OK) return st;
  if (!k || !v || !aligned16(k) || !aligned16(v)) return BC_ERR_ARG;
  if ((beacon_k == nullptr) != (beacon_v == nullptr)) return BC_ERR_ARG;
  if (beacon_k && (!aligned16(beacon_k) || !aligned16(beacon_v))) return BC_ERR_ARG;
  // what this call's plan touches: the per-sequence counters, and the partial results only when
  // sequences are split into chunks
  const size_t need = pl.tickets_bytes + (pl.max_chunks > 1 ? pl.total() - pl.tickets_bytes : 0);
  if (need > kScratchBytes) return BC_ERR_WORKSPACE;
  unsigned char* ws = nullptr;
  st = scratch_of_current_device(&ws);
  if (st != BC_OK) return st;
  // Every call on this GPU shares the array and finds what the last one left: the counters must
  // start at zero (a fill kernel, not a memset node: callers may be capturing a graph).
  const int64_t n = (int64_t)(pl.tickets_bytes / 4);
  const int64_t blocks = (n + 255) / 256;
  fill_zero_kernel<<<(int)(blocks < 1024 ? blocks : 1024), 256, 0, as_stream(stream)>>>(
      reinterpret_cast<uint32_t*>(ws), n);
  st = launch_status();
  if (st != BC_OK) return st;
  return decode_step_checked(shape, cache, pl, k, v, q, out, beacon_k, beacon_v, active, ws, stream);
}

extern "C" int32_t bc_beacon_step(const bc_shape* shape, const bc_cache* cache, const void* k,
                                  const void* v, const void* q, float* out, const uint8_t* active,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  DecodePlan pl;
  int32_t st = check_attention_args(shape, cache, q, out, workspace, workspace_bytes, &pl);
  if (st != BC_OK) return st;
  if (!k || !v || !aligned16(k) || !aligned16(v)) return BC_ERR_ARG;
  // one launch: beacon row at the tail, its attention, compaction
  return launch_attention(shape, cache, pl, q, out, active, workspace, k, v, k, v,
                          as_stream(stream), nullptr, nullptr, true);
}

extern "C" int32_t bc_decode_step_budget(const bc_shape* shape, const bc_cache* cache, const void* k,
                                         const void* v, const void* q, float* out,
                                         const void* beacon_k, const void* beacon_v,
                                         const int32_t* budget, uint8_t* live, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  DecodePlan pl;
  int32_t st = check_attention_args(shape, cache, q, out, workspace, workspace_bytes, &pl);
  if (st != BC_OK) return st;
  if (!k || !v || !aligned16(k) || !aligned16(v) || !budget || !live) return BC_ERR_ARG;
  if ((beacon_k == nullptr) != (beacon_v == nullptr)) return BC_ERR_ARG;
  if (beacon_k && (!aligned16(beacon_k) || !aligned16(beacon_v))) return BC_ERR_ARG;
  // The cap is tested on the state the attention saw (before the eviction); the holder of the
  // sequence's last ticket clears the mask after the eviction has used it.
  return launch_attention(shape, cache, pl, q, out, live, workspace, k, v, beacon_k, beacon_v,
                          as_stream(stream), budget, live);
}
