// Device-side building blocks of libpqcache (gfx950, wave64).
//
// Everything here is a __device__ template; the kernels that use them live in
// pqc_kernels.h.  Citations are to the paper's sections (PQ search: Section 2.2 and
// Section 3.1 step 4; top-k: Section 3.1 steps 4-5 and Section 3.2; selective
// attention: Section 2.1 and Section 3.1 step 6).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace pqc {

constexpr int kNB = 2048;        // score bins of the one-pass threshold search
constexpr int kHistCopies = 4;   // histogram replica slots per unit; Shape::histCopies of them are in use
constexpr int kD = 128;          // head dimension
constexpr int kLutRow = 256;     // LDS stride of one partition's table (max centroids)
constexpr int kCandRec = 1024;   // boundary-bin candidate records per unit (ranked inside LDS by the finalize kernel)
constexpr float kNegBig = -1.0e30f;

struct bf16_t {
  uint16_t bits;
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Geometry of one decode step, passed by value to every kernel.
struct Shape {
  int B, Hq, Hkv, G, N, M, C, Dm, K, I, L, Ktot;
  int cap;          // tokens the K/V caches and the code tensor hold per unit (>= N): their stride between units
  int tokA, nblkA;  // histogram kernel: tokens per workgroup, workgroups per unit
  int tokC, nblkC;  // select kernel: tokens per workgroup, workgroups per unit
  int rowsP, nblkP; // list-attention kernel: rows per workgroup, workgroups per unit
  int npart;        // partial slots per unit
  int slices;       // finalize kernel: workgroups per query head (1, 2 or 4), each producing kD/slices output dimensions
  int binStride;    // stored bins per unit (nblkC * tokC)
  int stageStride;  // 8-byte words between the staging slots of consecutive select workgroups: tokC plus a pad, so that
                    // the slots do not all start on the same memory channels
  int histCopies;   // histogram replicas in use (1, 2 or 4): spreads the flush atomics of units with many workgroups
  int sampleN;      // tokens sampled per unit to place the fine bins (<= 1024)
  int rankHi, rankLo;  // sample ranks (from the top) that bracket the K-th largest score
  float scale_log2e;
};

// What a select workgroup leaves behind for every boundary-bin candidate, enough for the finalize kernel to rank it
// and, if admitted, to add it to the attention output without touching the K/V cache again.  Per unit, as arrays
// over the candidates in order of arrival (at most kCandRec), so that what a finalize workgroup reads of them is dense:
//   composite  [kCandRec]      uint64   (score key, ~token): larger ranks first
//   logit      [G][kCandRec]   float    q_h . k for the group's heads (raw, unscaled)
//   v          [kCandRec][kD]  T        the V row
struct CandView {
  unsigned long long* composite;
  float* logit;
  unsigned char* v;
};
__host__ __device__ constexpr size_t cand_unit_bytes(int G, int elem_bytes) {
  return ((size_t)kCandRec * 8 + (size_t)G * kCandRec * 4 + (size_t)kCandRec * kD * elem_bytes + 255) / 256 * 256;
}
__device__ __forceinline__ CandView cand_view(unsigned char* unit_base, int G) {
  CandView c;
  c.composite = reinterpret_cast<unsigned long long*>(unit_base);
  c.logit = reinterpret_cast<float*>(unit_base + (size_t)kCandRec * 8);
  c.v = unit_base + (size_t)kCandRec * 8 + (size_t)G * kCandRec * 4;
  return c;
}

struct BinParams;
// Device pointers carved out of the caller's workspace.
struct Workspace {
  BinParams* ctl;              // [units]                       score -> bin map of the unit
  float* lut;                  // [units][M][C]
  float2* range;               // [units]                       (min, max) score, stand-alone top-k only
  unsigned* hist;              // [2][units][histCopies][kNB]   zero between uses (room for kHistCopies replicas)
  unsigned* cand_count;        // [2][units]   records handed out so far (directly behind hist, zeroed with it)
  unsigned short* bins;        // [units][binStride]  per token: bin + 1, or kBinWindow inside the two windows
  unsigned char* cand_rec;     // [units] blocks of rec_stride bytes: the candidates' composites, logits and V rows (CandView)
  unsigned long long* stage;   // [units][nblkC][stageStride]: selected ids (front, int32) / candidate composites (ending at word tokC)
  int2* stage_cnt;             // [units][nblkC]     (selected, candidates)
  float* partials;             // [units][npart][G][kD+2]
  int rec_stride;
#ifdef PQC_TRACE
  unsigned long long* trace;   // [3 kernels][kTraceWgs][kTraceSlots] time stamps (debug builds only)
#endif
};

// Phase time stamps for debug builds (-DPQC_TRACE); compiled out otherwise.
#ifdef PQC_TRACE
constexpr int kTraceWgs = 4096, kTraceSlots = 16;
#define PQC_MARK(ws, kid, slot)                                                                              \
  do {                                                                                                       \
    if (threadIdx.x == 0) {                                                                                  \
      const size_t wg_ = (size_t)blockIdx.y * gridDim.x + blockIdx.x;                                        \
      if (wg_ < (size_t)kTraceWgs) (ws).trace[((size_t)(kid)*kTraceWgs + wg_) * kTraceSlots + (slot)] = wall_clock64(); \
    }                                                                                                        \
  } while (0)
#define PQC_NOTE(ws, kid, slot, val)                                                                         \
  do {                                                                                                       \
    if (threadIdx.x == 0) {                                                                                  \
      const size_t wg_ = (size_t)blockIdx.y * gridDim.x + blockIdx.x;                                        \
      if (wg_ < (size_t)kTraceWgs) (ws).trace[((size_t)(kid)*kTraceWgs + wg_) * kTraceSlots + (slot)] = (unsigned long long)(val); \
    }                                                                                                        \
  } while (0)
#else
#define PQC_MARK(ws, kid, slot) \
  do {                          \
  } while (0)
#define PQC_NOTE(ws, kid, slot, val) \
  do {                               \
  } while (0)
#endif

// Marks the end of a group of independent loads: the instruction scheduler may not move
// anything across this point, so the loads above are all issued before their first use
// (left alone it tends to interleave load and use to save registers, which turns one
// memory round trip into many).
#define PQC_LOADS_ISSUED() __builtin_amdgcn_sched_barrier(0)

// ---------------------------------------------------------------- small helpers
__device__ __forceinline__ unsigned score_key(float f) {
  // order-preserving map float -> unsigned (larger score, larger key); -0 == +0
  f += 0.0f;
  unsigned u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

__device__ __forceinline__ float key_score(unsigned k) {  // inverse of score_key
  return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xffffffffu));
}

__device__ __forceinline__ unsigned long long make_composite(float score, int token) {
  // larger composite = ranks first: higher score, then lower token index
  return ((unsigned long long)score_key(score) << 32) | (unsigned long long)(0xffffffffu - (unsigned)token);
}

__device__ __forceinline__ int composite_token(unsigned long long c) {
  return (int)(0xffffffffu - (unsigned)(c & 0xffffffffull));
}

// Monotone map score -> bin.  Bin 0 takes every score below c0, kFineBins fine bins
// cover [c0, c1], kHighBins coarse bins lie above c1.  The piece is chosen by exact
// comparisons and each piece is clamped to its own bin range, so the map is
// non-decreasing in s whatever the parameters are (inside a piece: subtraction,
// multiplication by a non-negative constant and truncation all preserve order).  Only
// the number of boundary-bin candidates depends on how well [c0, c1] brackets the K-th
// largest score; the selection itself never does.  (Should the K-th largest score lie
// below c0, every token of bin 0 becomes a candidate: slow, still exact.)
constexpr int kHighBins = 256;
constexpr unsigned kBinWindow = 0xffffu;  // stored bin of a window token: above every threshold
constexpr int kFineBins = kNB - 1 - kHighBins;
struct BinParams {
  float lo, c0, c1, inv_c, inv_hi, hi, pad0, pad1;
};
// The layout travels as scalars held in registers (selecting among the fields of a struct
// in memory makes the compiler index it like an array, which lands it in scratch or LDS).
// (one subtraction, one multiplication and one conversion per score: the piece is selected first)
__device__ __forceinline__ int score_bin(float s, float c0, float c1, float inv_c, float inv_hi) {
  const bool up = s > c1;
  const float x = (s - (up ? c1 : c0)) * (up ? inv_hi : inv_c);
  const int b = min((int)x, up ? kHighBins - 1 : kFineBins - 1) + (up ? 1 + kFineBins : 1);  // the conversion truncates
  return s < c0 ? 0 : b;
}
// Bin layout from bounds lo <= score <= hi and a window [q_lo, q_hi] expected to hold
// the K-th largest score.
__device__ __forceinline__ BinParams make_bins(float lo, float hi, float q_lo, float q_hi) {
  BinParams bp;
  bp.lo = lo;
  bp.hi = hi;
  bp.c0 = fmaxf(lo, q_lo);
  bp.c1 = fminf(hi, q_hi);
  if (!(bp.c1 > bp.c0)) {  // degenerate window: one fine piece over everything
    bp.c0 = lo;
    bp.c1 = hi;
  }
  const float wc = bp.c1 - bp.c0, wh = hi - bp.c1;
  bp.inv_c = (wc > 1e-30f && wc < 3e38f) ? (float)kFineBins / wc : 0.0f;
  bp.inv_hi = (wh > 1e-30f && wh < 3e38f) ? (float)kHighBins / wh : 0.0f;
  bp.pad0 = 0.0f;
  bp.pad1 = 0.0f;
  return bp;
}

// ------------------------------------------------------------ cross-lane helpers
// DPP moves: a lane whose source is outside its row (or masked out) keeps `identity`.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_i(int identity, int x) {
  return __builtin_amdgcn_update_dpp(identity, x, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_f(float identity, float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(x), CTRL, ROW_MASK, 0xf, false));
}
// row_shr:1,2,4,8 then row_bcast:15 (rows 1,3) and row_bcast:31 (rows 2,3)
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_i<0x111>(0, v);
  v += dpp_i<0x112>(0, v);
  v += dpp_i<0x114>(0, v);
  v += dpp_i<0x118>(0, v);
  v += dpp_i<0x142, 0xa>(0, v);
  v += dpp_i<0x143, 0xc>(0, v);
  return v;
}
__device__ __forceinline__ int wave_last(int v) { return __builtin_amdgcn_readlane(v, 63); }
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<0x111>(0.0f, v);
  v += dpp_f<0x112>(0.0f, v);
  v += dpp_f<0x114>(0.0f, v);
  v += dpp_f<0x118>(0.0f, v);
  v += dpp_f<0x142, 0xa>(0.0f, v);
  v += dpp_f<0x143, 0xc>(0.0f, v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<0x111>(-INFINITY, v));
  v = fmaxf(v, dpp_f<0x112>(-INFINITY, v));
  v = fmaxf(v, dpp_f<0x114>(-INFINITY, v));
  v = fmaxf(v, dpp_f<0x118>(-INFINITY, v));
  v = fmaxf(v, dpp_f<0x142, 0xa>(-INFINITY, v));
  v = fmaxf(v, dpp_f<0x143, 0xc>(-INFINITY, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_min(float v) { return -wave_max(-v); }

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float group16_sum(float x) {
  x += dpp_f<0xB1>(0.0f, x);   // quad_perm [1,0,3,2]: neighbour in the pair
  x += dpp_f<0x4E>(0.0f, x);   // quad_perm [2,3,0,1]: other pair of the quad
  x += dpp_f<0x141>(0.0f, x);  // row_half_mirror: other quad of the half row
  x += dpp_f<0x140>(0.0f, x);  // row_mirror: other half of the row
  return x;
}

// Exclusive prefix sum over the threads of a workgroup (NT threads, multiple of 64).
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int v, int* total, int* sm /* [2*(NT/64)+1] */) {
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int inc = wave_inclusive_scan(v);
  if (lane == 63) sm[w] = inc;
  __syncthreads();
  if (w == 0) {
    const int s = lane < NW ? sm[lane] : 0;
    const int si = wave_inclusive_scan(s);
    if (lane < NW) sm[NW + lane] = si - s;
    if (lane == NW - 1) sm[2 * NW] = si;
  }
  __syncthreads();
  const int res = inc - v + sm[NW + w];
  *total = sm[2 * NW];
  __syncthreads();
  return res;
}

// --------------------------------------------------------------- look-up table
// Section 2.2 (search) / Section 3.1 step 4: table[j][c] = qs[j*Dm..] . cent[j][c][..]
// with qs the sum of the group's query heads.  Fixed fp32 order: head order for
// the sum, one fused multiply-add chain per entry.  Also derives the score -> bin map
// from bounds on every possible score (lo = sum_j min_c table[j][c], hi likewise with
// max, added in the same order as a score, so that lo <= score <= hi holds in fp32)
// and from the mean and spread the scores would have under uniform code usage.
template <typename T>
__device__ __forceinline__ float load_as_float(const T* p, int i);
template <>
__device__ __forceinline__ float load_as_float<float>(const float* p, int i) {
  return p[i];
}
template <>
__device__ __forceinline__ float load_as_float<bf16_t>(const bf16_t* p, int i) {
  return __uint_as_float((unsigned)p[i].bits << 16);
}

// Centroids travel global -> registers (coalesced, all loads in flight at once) -> a
// padded LDS tile -> one thread per table entry runs the chain.  With 1024 threads the
// tile holds the whole table (C*(kD+M) floats, up to 136 KB of the CU's 160 KB) and there
// is a single pass; with fewer threads the table goes through a tile of kLutTileFloats
// floats piece by piece.
constexpr int kLutTileFloats = 8192;
// Row stride of the whole-table tile.  Long rows (one or two partitions: few entries, few busy
// waves) are padded by four floats and read 128 bits at a time; short rows keep every thread busy
// and measured faster with an odd stride and 32-bit accesses.
__host__ __device__ constexpr int lut_row_stride(int M) { return M <= 2 ? kD / M + 4 : kD / M + 1; }
__host__ __device__ constexpr int lut_tile_floats(int nt, int M, int C) {
  return nt >= 1024 ? M * C * lut_row_stride(M) : kLutTileFloats + kLutTileFloats / (kD / M);
}
// VWP (whole-table mode): 16-byte pieces of the table per thread; VWP * NT * 4 floats must cover M*C*Dm.
template <typename T, int NT, int M, class MarkFn, class IssueFn, int VWP = (256 * kD) / (4 * NT)>
__device__ __forceinline__ float2 build_lut(const T* __restrict__ q /* [G][kD] of this unit */,
                                               const float* __restrict__ cent /* [M][C][Dm] */, int G, int C,
                                               float* lut, float* qs, float* red /* [4*8] */,
                                               float* tile /* [lut_tile_floats(NT, M, C)] */, MarkFn mark,
                                               IssueFn issue_more /* the caller's own loads, queued behind the table's */) {
  constexpr int Dm = kD / M, RS = lut_row_stride(M);
  constexpr bool kWhole = NT >= 1024;
  constexpr int VW = kWhole ? VWP : 1;                    // float4 per thread
  constexpr int VPG = kLutTileFloats / (4 * NT);      // float4 per thread per tile (piecewise mode)
  constexpr int NG = (256 * kD) / kLutTileFloats;      // tiles at the largest C (piecewise mode)
  const int tid = threadIdx.x;
  const int total = M * C * Dm;                        // floats, a multiple of 4
  const float4* cent4 = reinterpret_cast<const float4*>(cent);
  // (a native vector type: a float4 struct copied from global memory to LDS is turned into one 16-byte copy at
  // the place of the store, which puts every load behind the waits in front of it, one round trip after the other)
  const f32x4_t* centv = reinterpret_cast<const f32x4_t*>(cent);
  f32x4_t vw[VW];
  if constexpr (kWhole) {
#pragma unroll
    for (int x = 0; x < VW; ++x) vw[x] = centv[min(x * NT + tid, total / 4 - 1)];
  }
  {
    // the group's query heads: all loads first (clamped, straight-line), then the sum in head order
    const int dq = tid & (kD - 1);
    float qv[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) qv[h] = load_as_float<T>(q, min(h, G - 1) * kD + dq);
    // Loads return in issue order: whatever the caller streams from HBM goes behind the table's
    // (mostly L2-resident) centroids, so that the table is built while that stream arrives.
    PQC_LOADS_ISSUED();
    if constexpr (!kWhole) issue_more();
    PQC_LOADS_ISSUED();
    float a = qv[0];
#pragma unroll
    for (int h = 1; h < 8; ++h) {
      const float t = __fadd_rn(a, qv[h]);
      a = h < G ? t : a;  // select, not branch: keeps the eight loads above in flight together
    }
    qs[dq] = a;  // every thread (tid and tid + kD hold the same sum): a branch here would split the block, and the
                 // compiler would then move the centroid loads above down to their use, behind this wait
  }
  mark(8);
  if constexpr (kWhole) {
#pragma unroll
    for (int x = 0; x < VW; ++x) {
      // No branch around the store: a thread beyond the table holds the table's last float4 (its load was clamped)
      // and writes it to that float4's place once more.  With a branch here the compiler moves each load down into
      // its branch and waits for it there, one memory round trip after the other.
      const int fl = min((x * NT + tid) * 4, total - 4);  // float index inside the table
      const int row = fl / Dm, col = fl % Dm;             // Dm is a multiple of 4: one row per float4
      float* dst = tile + row * RS + col;
      if constexpr (RS % 4 == 0) {
        *reinterpret_cast<f32x4_t*>(dst) = vw[x];
      } else {
        dst[0] = vw[x][0]; dst[1] = vw[x][1]; dst[2] = vw[x][2]; dst[3] = vw[x][3];
      }
    }
    // the caller's stream from HBM is requested now, behind every wave's centroid loads (a compute unit's loads
    // pass through one address unit): the table is built while that stream arrives
    issue_more();
    PQC_LOADS_ISSUED();
    unsigned* mm = reinterpret_cast<unsigned*>(red);  // [0..8): smallest entry of a partition, [8..16): largest, as score keys
    if (tid < 16) mm[tid] = tid < 8 ? 0xffffffffu : 0u;
    mark(10);
    __syncthreads();  // tile, qs and mm visible
    mark(11);
    for (int e0 = 0; e0 + (tid & ~63) < M * C; e0 += NT) {  // per wave: the wave-wide reductions below need every lane
      const int e = e0 + tid;
      const bool valid = e < M * C;
      const int ec = valid ? e : 0;
      const int j = ec / C, c = ec - j * C;
      const float* qj = qs + j * Dm;
      const float* cr = tile + ec * RS;
      float p = 0.0f;
      if constexpr (RS % 4 == 0) {
        // Few entries, so few busy waves and nothing to hide the LDS latency behind: the operands are read two
        // stages of four 16-byte pieces ahead of the chain (left alone the compiler reads one piece ahead and the
        // chain waits for LDS at every fourth step).
        constexpr int kStages = Dm / 16;
        const f32x4_t* qv4 = reinterpret_cast<const f32x4_t*>(qj);
        const f32x4_t* cv4 = reinterpret_cast<const f32x4_t*>(cr);
        f32x4_t qa[2][4], ca[2][4];
#pragma unroll
        for (int st = 0; st < 2 && st < kStages; ++st)
#pragma unroll
          for (int y = 0; y < 4; ++y) {
            qa[st][y] = qv4[st * 4 + y];
            ca[st][y] = cv4[st * 4 + y];
          }
#pragma unroll
        for (int st = 0; st < kStages; ++st) {
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int y = 0; y < 4; ++y) {
            p = __fmaf_rn(qa[st & 1][y][0], ca[st & 1][y][0], p);
            p = __fmaf_rn(qa[st & 1][y][1], ca[st & 1][y][1], p);
            p = __fmaf_rn(qa[st & 1][y][2], ca[st & 1][y][2], p);
            p = __fmaf_rn(qa[st & 1][y][3], ca[st & 1][y][3], p);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (st + 2 < kStages) {
#pragma unroll
            for (int y = 0; y < 4; ++y) {
              qa[st & 1][y] = qv4[(st + 2) * 4 + y];
              ca[st & 1][y] = cv4[(st + 2) * 4 + y];
            }
          }
        }
      } else {
#pragma unroll
        for (int x = 0; x < Dm / 4; ++x) {  // the query four at a time (one address per wave: a broadcast)
          const float4 qq = reinterpret_cast<const float4*>(qj)[x];
          p = __fmaf_rn(qq.x, cr[4 * x + 0], p);
          p = __fmaf_rn(qq.y, cr[4 * x + 1], p);
          p = __fmaf_rn(qq.z, cr[4 * x + 2], p);
          p = __fmaf_rn(qq.w, cr[4 * x + 3], p);
        }
      }
      if (valid) lut[j * kLutRow + c] = p;
      // the partition's smallest and largest entry (as order-preserving keys): one pair of LDS atomics per wave
      // when the wave's 64 entries lie in one partition, else one pair per entry
      if ((C & 63) == 0) {  // uniform
        const float pmin = wave_min(valid ? p : INFINITY), pmax = wave_max(valid ? p : -INFINITY);
        if ((tid & 63) == 0 && valid) {  // the wave's first entry is valid whenever any is
          atomicMin(&mm[j], score_key(pmin));
          atomicMax(&mm[8 + j], score_key(pmax));
        }
      } else if (valid) {
        atomicMin(&mm[j], score_key(p));
        atomicMax(&mm[8 + j], score_key(p));
      }
    }
    mark(9);
  } else {
    float4 v[VPG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      if (g * kLutTileFloats < total) {  // uniform
#pragma unroll
        for (int x = 0; x < VPG; ++x) {
          const int f = g * (kLutTileFloats / 4) + x * NT + tid;
          v[x] = cent4[min(f, total / 4 - 1)];
        }
        if (g > 0) __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int x = 0; x < VPG; ++x) {
          const int fl = (x * NT + tid) * 4;  // float index inside the tile
          if (g * kLutTileFloats + fl < total) {
            const int row = fl / Dm, col = fl % Dm;
            float* dst = tile + row * (Dm + 1) + col;
            dst[0] = v[x].x; dst[1] = v[x].y; dst[2] = v[x].z; dst[3] = v[x].w;
          }
        }
        __syncthreads();  // tile (and, first time round, qs) visible
        const int rows = min(kLutTileFloats, total - g * kLutTileFloats) / Dm;
        for (int r = tid; r < rows; r += NT) {
          const int e = g * (kLutTileFloats / Dm) + r;
          const int j = e / C, c = e - j * C;
          const float* qj = qs + j * Dm;
          const float* cr = tile + r * (Dm + 1);
          float p = 0.0f;
#pragma unroll
          for (int x = 0; x < Dm; ++x) p = __fmaf_rn(qj[x], cr[x], p);
          lut[j * kLutRow + c] = p;
        }
      }
    }
  }
  __syncthreads();
  mark(13);
  if constexpr (kWhole) {
    // bounds are added in the same order as a score, so lo <= score <= hi holds in fp32
    const unsigned* mm = reinterpret_cast<const unsigned*>(red);
    float lo = key_score(mm[0]), hi = key_score(mm[8]);
    for (int j = 1; j < M; ++j) {
      lo = __fadd_rn(lo, key_score(mm[j]));
      hi = __fadd_rn(hi, key_score(mm[8 + j]));
    }
    return make_float2(lo, hi);
  }
  // per table: min and max (one wave per table)
  const int lane = tid & 63, w = tid >> 6;
  for (int j = w; j < M; j += NT / 64) {
    float mn = INFINITY, mx = -INFINITY;
    for (int c = lane; c < C; c += 64) {
      const float x = lut[j * kLutRow + c];
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if (lane == 0) {
      red[j] = mn;
      red[8 + j] = mx;
    }
  }
  __syncthreads();
  // bounds are added in the same order as a score, so lo <= score <= hi holds in fp32
  float lo = red[0], hi = red[8];
  for (int j = 1; j < M; ++j) {
    lo = __fadd_rn(lo, red[j]);
    hi = __fadd_rn(hi, red[8 + j]);
  }
  return make_float2(lo, hi);
}

// Where the fine bins go: every workgroup of a unit scores the same `n` sampled tokens,
// histograms them over kSampleBins uniform bins of [lo, hi] and takes the bins that hold the
// sample's rank_hi-th and rank_lo-th largest scores as the window.  The ranks bracket
// the K-th largest of all tokens by several standard errors of the sample quantile, so
// the window almost always holds it (and when it does not, only speed is lost).
// Two barriers: the samples are counted, then the first wave alone walks the histogram
// (four bins per lane, a wave-wide prefix sum) and clears it again.
//   hist  LDS [>= kSampleBins], zero on entry, zero again on return      sm  LDS [2]
constexpr int kSampleBins = 256;
template <int NT>
__device__ __forceinline__ BinParams sample_window(float lo, float hi, float my_score, bool have_sample, int rank_hi,
                                                   int rank_lo, unsigned* hist, int* sm) {
  constexpr int NBS = kSampleBins, PER = NBS / 64;
  static_assert(PER == 4, "one 16-byte access per lane");
  const int tid = threadIdx.x;
  const float width = hi - lo;
  const float inv_u = (width > 1e-30f && width < 3e38f) ? (float)NBS / width : 0.0f;
  if (have_sample) atomicAdd(&hist[max(0, min(NBS - 1, __float2int_rz((my_score - lo) * inv_u)))], 1u);
  __syncthreads();
  if (tid < 64) {  // lane l owns bins [NBS - (l+1)*PER, NBS - l*PER): the lanes run from the top bin down
    uint4* mine = reinterpret_cast<uint4*>(hist + NBS - (tid + 1) * PER);
    const uint4 x = *mine;
    *mine = make_uint4(0u, 0u, 0u, 0u);
    const int h[PER] = {(int)x.x, (int)x.y, (int)x.z, (int)x.w};
    const int sum = h[0] + h[1] + h[2] + h[3];
    int cum = wave_inclusive_scan(sum) - sum;  // samples in the bins above this lane's
    int r0 = -1, r1 = -1;
#pragma unroll
    for (int e = PER - 1; e >= 0; --e) {  // this lane's bins, from its top one down
      const int b = NBS - (tid + 1) * PER + e;
      if (rank_hi >= 1 && cum < rank_hi && cum + h[e] >= rank_hi) r0 = b;
      if (rank_lo >= 1 && cum < rank_lo && cum + h[e] >= rank_lo) r1 = b;
      cum += h[e];
    }
    // at most one lane finds each of the two bins: a wave-wide maximum, read from the last lane
    r0 = max(r0, dpp_i<0x111>(-1, r0)); r1 = max(r1, dpp_i<0x111>(-1, r1));
    r0 = max(r0, dpp_i<0x112>(-1, r0)); r1 = max(r1, dpp_i<0x112>(-1, r1));
    r0 = max(r0, dpp_i<0x114>(-1, r0)); r1 = max(r1, dpp_i<0x114>(-1, r1));
    r0 = max(r0, dpp_i<0x118>(-1, r0)); r1 = max(r1, dpp_i<0x118>(-1, r1));
    r0 = max(r0, dpp_i<0x142, 0xa>(-1, r0)); r1 = max(r1, dpp_i<0x142, 0xa>(-1, r1));
    r0 = max(r0, dpp_i<0x143, 0xc>(-1, r0)); r1 = max(r1, dpp_i<0x143, 0xc>(-1, r1));
    if (tid == 63) {
      sm[0] = r0;
      sm[1] = r1;
    }
  }
  __syncthreads();
  const int b_hi = sm[0], b_lo = sm[1];
  const float wu = width * (1.0f / (float)NBS);
  const float q_hi = b_hi >= 0 ? lo + (float)(b_hi + 1) * wu : hi;
  const float q_lo = b_lo >= 0 ? lo + (float)b_lo * wu : lo;
  return make_bins(lo, hi, q_lo, q_hi);
}

// ------------------------------------------------------------------- code scan
// Section 3.1 step 4: a token's score is the sum over partitions of the table entry
// its code names, added left to right.
template <int M>
struct CodeWord;
template <>
struct CodeWord<1> {
  using type = uint8_t;
};
template <>
struct CodeWord<2> {
  using type = uint16_t;
};
template <>
struct CodeWord<4> {
  using type = uint32_t;
};
template <>
struct CodeWord<8> {
  using type = uint64_t;
};

template <int M>
__device__ __forceinline__ float score_from_word(typename CodeWord<M>::type w, const float* lut) {
  float s = lut[(unsigned)(w & 0xff)];
#pragma unroll
  for (int j = 1; j < M; ++j) s = __fadd_rn(s, lut[j * kLutRow + (unsigned)((w >> (8 * j)) & 0xff)]);
  return s;
}

// 16 bytes of codes = P = 16/M consecutive tokens; word i of the chunk.
template <int M>
__device__ __forceinline__ typename CodeWord<M>::type chunk_word(const uint4& raw, int i) {
  const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
  if constexpr (M == 8) {
    return ((unsigned long long)w[2 * i + 1] << 32) | w[2 * i];
  } else if constexpr (M == 4) {
    return w[i];
  } else if constexpr (M == 2) {
    return (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
  } else {
    return (uint8_t)(w[i >> 2] >> (8 * (i & 3)));
  }
}

// ------------------------------------------------------------ threshold search
// Section 3.2 (k-th largest score).  The unit's histogram over kNB monotone score
// bins fixes the bin b* that holds the K-th largest score: bins above it are taken
// whole, bins below dropped, and only b*'s members ("candidates") need ranking.
struct Threshold {
  int bstar;    // kNB when K == 0
  int n_above;  // tokens in bins above bstar
  int need;     // candidates to admit = K - n_above
  int n_cand;   // tokens in bin bstar
};

// Two steps so that a kernel can issue the histogram loads together with its other
// loads: load() only reads (ghist: the unit's kHistCopies replicas), resolve() sums the
// replicas and searches.  Thread tid owns bins [kNB - (tid+1)*PER, kNB - tid*PER).
template <int NT>
struct ThresholdSearch {
  static constexpr int PER = kNB / NT;
  static_assert(PER % 4 == 0, "bins per thread must allow 16-byte loads");
  uint4 x[kHistCopies][PER / 4];
  __device__ __forceinline__ void load(const unsigned* __restrict__ ghist, int copies) {
#pragma unroll
    for (int c = 0; c < kHistCopies; ++c) {
      const uint4* src = reinterpret_cast<const uint4*>(ghist + c * kNB + kNB - (threadIdx.x + 1) * PER);
#pragma unroll
      for (int v = 0; v < PER / 4; ++v) x[c][v] = c < copies ? src[v] : make_uint4(0u, 0u, 0u, 0u);  // uniform
    }
  }
  __device__ __forceinline__ Threshold resolve(int K, int* sm /* [2*(NT/64)+1+4] */) const {
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    unsigned h[PER];  // descending bins: h[e] is bin kNB-1-(tid*PER+e)
#pragma unroll
    for (int e = 0; e < PER; ++e) h[e] = 0u;
#pragma unroll
    for (int c = 0; c < kHistCopies; ++c)
#pragma unroll
      for (int v = 0; v < PER / 4; ++v) {
        h[PER - 1 - (4 * v + 0)] += x[c][v].x;
        h[PER - 1 - (4 * v + 1)] += x[c][v].y;
        h[PER - 1 - (4 * v + 2)] += x[c][v].z;
        h[PER - 1 - (4 * v + 3)] += x[c][v].w;
      }
    int sum = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) sum += (int)h[e];
    int total;
    int cum = block_exclusive_scan<NT>(sum, &total, sm);
    int* res = sm + 2 * NW + 1;
    if (tid == 0) {
      res[0] = kNB;
      res[1] = 0;
      res[2] = 0;
      res[3] = 0;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (K > 0 && cum < K && cum + (int)h[e] >= K) {
        res[0] = kNB - 1 - (tid * PER + e);
        res[1] = cum;
        res[2] = K - cum;
        res[3] = (int)h[e];
      }
      cum += (int)h[e];
    }
    __syncthreads();
    Threshold t{res[0], res[1], res[2], res[3]};
    __syncthreads();
    return t;
  }
};

// ------------------------------------------------- threshold from code-pair counts
// With M = 2 and C <= 64 a token's score takes one of C*C values, one per pair of codes.
// Given how many tokens carry each pair (a statistic of the codes alone, kept with them),
// the K-th largest score follows from the table without a pass over the tokens: weight
// the C*C pair scores by their counts, find the uniform score bin that holds the K-th
// largest, then resolve the few pairs inside that bin exactly.  The result is the score
// key of the K-th largest middle token: larger keys are selected, equal keys are
// candidates (ranked by token index later).  Scores use the same fp32 order as everywhere.
constexpr int kPairSlots = 4096;  // C*C <= kPairSlots
constexpr int kPairC = 64;        // largest C
constexpr int kPairList = 256;    // pairs resolved by direct ranking; more fall back to a radix search
struct PairLds {
  unsigned cnt[kPairSlots];       // tokens per pair (c0 + C*c1), window tokens taken out
  float lut[2 * kPairC];          // table[j][c] at j*kPairC + c
  float qs[kD];
  unsigned hist[kNB];
  unsigned long long lst[kPairList];  // (key << 32) | count of the pairs in the threshold bin
  int res[8];
};
struct PairThreshold {
  unsigned key;  // score key of the K-th largest middle token
  bool none;     // K == 0: nothing is retrieved
};

template <typename T, int NT, class MarkFn>
__device__ __forceinline__ PairThreshold pair_threshold(const Shape& s, const T* __restrict__ q /* [G][kD] of the unit */,
                                                        const float* __restrict__ cent /* [2][C][64] of the unit */,
                                                        const unsigned* __restrict__ pair_counts /* [C*C] of the unit */,
                                                        const uint8_t* __restrict__ codes_u /* [N][2] of the unit */,
                                                        PairLds& L, int* scan_sm /* [2*(NT/64)+1] */, MarkFn mark,
                                                        int uncounted /* a window token the counts do not hold yet, or -1 */) {
  static_assert(NT == 256, "written for 256 threads");
  constexpr int Dm = kD / 2, PPT = kPairSlots / NT, BPT = kNB / NT;
  const int tid = threadIdx.x, C = s.C, np = C * C;
  // ---- loads: one table entry's centroid per thread (2C threads), query, counts, window codes
  const int e = min(tid, 2 * C - 1);
  const float4* crow = reinterpret_cast<const float4*>(cent + (size_t)e * Dm);
  float4 cr[Dm / 4];
#pragma unroll
  for (int x = 0; x < Dm / 4; ++x) cr[x] = crow[x];
  float qv[8];
#pragma unroll
  for (int h = 0; h < 8; ++h) qv[h] = load_as_float<T>(q, min(h, s.G - 1) * kD + (tid & (kD - 1)));
  unsigned pc[PPT];  // pair x*NT + tid
#pragma unroll
  for (int x = 0; x < PPT; ++x) pc[x] = pair_counts[min(x * NT + tid, np - 1)];
  const int nwin = s.I + s.L;
  unsigned short wcode = 0;  // first window token of this thread (the usual case: I + L <= NT)
  {
    const int wt = min(tid, max(nwin - 1, 0));
    const int t = wt < s.I ? wt : s.N - s.L + (wt - s.I);
    wcode = *reinterpret_cast<const unsigned short*>(codes_u + (size_t)min(max(t, 0), s.N - 1) * 2);
  }
  PQC_LOADS_ISSUED();
  {
    float a = qv[0];
#pragma unroll
    for (int h = 1; h < 8; ++h) {
      const float t = __fadd_rn(a, qv[h]);
      a = h < s.G ? t : a;
    }
    if (tid < kD) L.qs[tid] = a;
  }
#pragma unroll
  for (int x = 0; x < PPT; ++x)
    if (x * NT + tid < np) L.cnt[x * NT + tid] = pc[x];
#pragma unroll
  for (int x = 0; x < BPT; ++x) L.hist[x * NT + tid] = 0u;
  if (tid < 8) L.res[tid] = (tid == 4 || tid == 6) ? -1 : 0;  // slots 4..7: (min, max) keys of the two partitions
  __syncthreads();
  mark(9);
  // ---- table entries (fixed-order chain) and the window tokens taken out of the counts
  if (tid < 2 * C) {
    const int j = tid / C, c = tid - j * C;
    const float* qj = L.qs + j * Dm;
    float p = 0.0f;
#pragma unroll
    for (int x = 0; x < Dm / 4; ++x) {
      p = __fmaf_rn(qj[4 * x + 0], cr[x].x, p);
      p = __fmaf_rn(qj[4 * x + 1], cr[x].y, p);
      p = __fmaf_rn(qj[4 * x + 2], cr[x].z, p);
      p = __fmaf_rn(qj[4 * x + 3], cr[x].w, p);
    }
    L.lut[j * kPairC + c] = p;
    const unsigned pk = score_key(p);  // per-partition minimum and maximum, through order-preserving keys
    atomicMin(reinterpret_cast<unsigned*>(&L.res[4 + 2 * j]), pk);
    atomicMax(reinterpret_cast<unsigned*>(&L.res[5 + 2 * j]), pk);
  }
  for (int wt = tid; wt < nwin; wt += NT) {
    unsigned short cw = wcode;
    const int t = wt < s.I ? wt : s.N - s.L + (wt - s.I);
    if (wt >= NT) cw = *reinterpret_cast<const unsigned short*>(codes_u + (size_t)t * 2);
    const int w0 = cw & 0xff, w1 = cw >> 8;  // a code outside [0, C) was never counted
    if (w0 < C && w1 < C && t != uncounted) atomicSub(&L.cnt[w0 + C * w1], 1u);
  }
  __syncthreads();
  mark(10);
  // ---- bounds (added in the same order as a score), weighted histogram over uniform bins
  const float mn0 = key_score((unsigned)L.res[4]), mx0 = key_score((unsigned)L.res[5]);
  const float mn1 = key_score((unsigned)L.res[6]), mx1 = key_score((unsigned)L.res[7]);
  const float lo = __fadd_rn(mn0, mn1), hi = __fadd_rn(mx0, mx1), width = hi - lo;
  const float inv = (width > 1e-30f && width < 3e38f) ? (float)kNB / width : 0.0f;
  unsigned pkey[PPT];
  int pbin[PPT];
#pragma unroll
  for (int x = 0; x < PPT; ++x) {
    const int pr = x * NT + tid;
    int c1, c0;
    if (C == kPairC) {  // uniform; spares an integer division per pair
      c1 = pr >> 6;
      c0 = pr & (kPairC - 1);
    } else {
      c1 = min(pr, np - 1) / C;
      c0 = min(pr, np - 1) - c1 * C;
    }
    const float sc = __fadd_rn(L.lut[c0], L.lut[kPairC + c1]);
    pkey[x] = score_key(sc);
    pbin[x] = max(0, min(kNB - 1, __float2int_rz((sc - lo) * inv)));
    pc[x] = pr < np ? L.cnt[pr] : 0u;
    if (pc[x]) atomicAdd(&L.hist[pbin[x]], pc[x]);
  }
  __syncthreads();
  mark(11);
  // ---- the bin that holds the K-th largest: thread tid owns bins kNB-1-(tid*BPT+e), descending
  unsigned h[BPT];
  int sum = 0;
#pragma unroll
  for (int x = 0; x < BPT; ++x) {
    h[x] = L.hist[kNB - 1 - (tid * BPT + x)];
    sum += (int)h[x];
  }
  int total;
  int cum = block_exclusive_scan<NT>(sum, &total, scan_sm);
  if (tid == 0) {
    L.res[0] = -1;  // threshold bin
    L.res[1] = 0;   // tokens in bins above it
  }
  __syncthreads();
#pragma unroll
  for (int x = 0; x < BPT; ++x) {
    if (s.K > 0 && cum < s.K && cum + (int)h[x] >= s.K) {
      L.res[0] = kNB - 1 - (tid * BPT + x);
      L.res[1] = cum;
    }
    cum += (int)h[x];
  }
  __syncthreads();
  const int bstar = L.res[0];
  const int want = s.K - L.res[1];  // rank of the K-th largest among the tokens of bin bstar (1-based)
  PairThreshold out;
  out.none = bstar < 0;
  out.key = 0xffffffffu;
  if (bstar < 0) return out;  // uniform
  mark(12);
  // ---- the pairs of that bin
#pragma unroll
  for (int x = 0; x < PPT; ++x)
    if (pc[x] && pbin[x] == bstar) {
      const int slot = atomicAdd(&L.res[2], 1);
      if (slot < kPairList) L.lst[slot] = ((unsigned long long)pkey[x] << 32) | pc[x];
    }
  __syncthreads();
  const int n_in = L.res[2];
  if (n_in <= kPairList) {
    if (tid < n_in) {
      const unsigned long long mine = L.lst[tid];
      const unsigned mk = (unsigned)(mine >> 32);
      long long above = 0, same = 0;
      for (int j0 = 0; j0 < n_in; j0 += 8) {  // eight independent LDS reads per round
        unsigned long long o[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) o[x] = L.lst[min(j0 + x, n_in - 1)];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const unsigned ok = (unsigned)(o[x] >> 32), oc = j0 + x < n_in ? (unsigned)o[x] : 0u;
          above += ok > mk ? oc : 0u;
          same += ok == mk ? oc : 0u;
        }
      }
      if (above < want && want <= above + same) L.res[3] = (int)mk;
    }
    __syncthreads();
    out.key = (unsigned)L.res[3];
  } else {
    // many pairs share the bin (nearly equal scores): 8-bit radix search over their keys
    unsigned prefix = 0u;
    long long w = want;
    for (int shift = 24; shift >= 0; shift -= 8) {
      L.hist[tid] = 0u;  // 256 digits
      __syncthreads();
#pragma unroll
      for (int x = 0; x < PPT; ++x)
        if (pc[x] && pbin[x] == bstar && (shift == 24 || (pkey[x] >> (shift + 8)) == (prefix >> (shift + 8))))
          atomicAdd(&L.hist[(pkey[x] >> shift) & 255u], pc[x]);
      __syncthreads();
      if (tid == 0) {
        long long c2 = 0;
        int dg = 255;
        for (; dg > 0; --dg) {
          if (c2 + (long long)L.hist[dg] >= w) break;
          c2 += L.hist[dg];
        }
        L.res[4] = dg;
        L.res[5] = (int)(w - c2);
      }
      __syncthreads();
      prefix |= (unsigned)L.res[4] << shift;
      w = L.res[5];
      __syncthreads();
    }
    out.key = prefix;
  }
  return out;
}

// ------------------------------------------------------- attention, vector ALU
// Section 2.1 restricted to listed tokens (Section 3.1 step 6).  Lane layout inside
// a wave: sub = lane & 15 owns 8 of the 128 dimensions of a row, slot = lane >> 4
// picks one of 4 rows handled at once; a 16-lane group reads one contiguous row.
// Logits are kept in the log2 domain (q is pre-multiplied by scale*log2(e)).
// Used for fp32 caches, for candidate logits and for the rare slow finalize path.
template <typename T>
struct RowRaw;
template <>
struct RowRaw<bf16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const bf16_t* base, int t, int sub) {
    a = *reinterpret_cast<const uint4*>(base + (size_t)t * kD + sub * 8);
  }
  __device__ __forceinline__ void load_row(const void* row, int sub) {
    a = *reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(row) + sub * 16);
  }
  __device__ __forceinline__ void zero() { a = make_uint4(0, 0, 0, 0); }
  __device__ __forceinline__ void unpack(float (&f)[8]) const {
    f[0] = __uint_as_float(a.x << 16);
    f[1] = __uint_as_float(a.x & 0xffff0000u);
    f[2] = __uint_as_float(a.y << 16);
    f[3] = __uint_as_float(a.y & 0xffff0000u);
    f[4] = __uint_as_float(a.z << 16);
    f[5] = __uint_as_float(a.z & 0xffff0000u);
    f[6] = __uint_as_float(a.w << 16);
    f[7] = __uint_as_float(a.w & 0xffff0000u);
  }
  __device__ __forceinline__ void store(unsigned char* dst, int sub) const { *reinterpret_cast<uint4*>(dst + sub * 16) = a; }
};
template <>
struct RowRaw<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* base, int t, int sub) {
    a = *reinterpret_cast<const float4*>(base + (size_t)t * kD + sub * 4);
    b = *reinterpret_cast<const float4*>(base + (size_t)t * kD + 64 + sub * 4);
  }
  __device__ __forceinline__ void load_row(const void* row, int sub) {
    a = *reinterpret_cast<const float4*>(static_cast<const unsigned char*>(row) + sub * 16);
    b = *reinterpret_cast<const float4*>(static_cast<const unsigned char*>(row) + 256 + sub * 16);
  }
  __device__ __forceinline__ void zero() {
    a = make_float4(0, 0, 0, 0);
    b = a;
  }
  __device__ __forceinline__ void unpack(float (&f)[8]) const {
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
  __device__ __forceinline__ void store(unsigned char* dst, int sub) const {
    *reinterpret_cast<float4*>(dst + sub * 16) = a;
    *reinterpret_cast<float4*>(dst + 256 + sub * 16) = b;
  }
};

// Dimension held in register e of lane-group member `sub`.
template <typename T>
__device__ __forceinline__ int owned_dim(int sub, int e);
template <>
__device__ __forceinline__ int owned_dim<bf16_t>(int sub, int e) {
  return sub * 8 + e;
}
template <>
__device__ __forceinline__ int owned_dim<float>(int sub, int e) {
  return e < 4 ? sub * 4 + e : 64 + sub * 4 + (e - 4);
}

template <int G>
struct AttnState {
  float m[G], l[G], acc[G][8];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m[h] = kNegBig;
      l[h] = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;
    }
  }
};

template <typename T, int G>
__device__ __forceinline__ void load_query(const T* __restrict__ q /* [G][kD] */, float factor, float (&qr)[G][8]) {
  const int sub = threadIdx.x & 15;
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) qr[h][e] = load_as_float<T>(q, h * kD + owned_dim<T>(sub, e)) * factor;
}

// Attend the rows list(p), p in [first, count) stepping by `stride`, where every
// wave-iteration covers 4*R consecutive list positions.  list(p) must be valid
// for p < count; tokens are clamped into [0, N).
template <typename T, int G, int R, class ListFn>
__device__ __forceinline__ void attend_rows(const T* __restrict__ kbase, const T* __restrict__ vbase, int N,
                                            ListFn list, int count, int first, int stride,
                                            const float (&qr)[G][8], AttnState<G>& st) {
  const int lane = threadIdx.x & 63;
  const int sub = lane & 15, slot = lane >> 4;
  for (int base = first; base < count; base += stride) {
    RowRaw<T> kr[R], vr[R];
    bool ok[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int p = base + r * 4 + slot;
      ok[r] = p < count;
      if (ok[r]) {
        int t = list(p);
        t = max(0, min(N - 1, t));
        kr[r].load(kbase, t, sub);
        vr[r].load(vbase, t, sub);
      } else {
        kr[r].zero();
        vr[r].zero();
      }
    }
    PQC_LOADS_ISSUED();
    float s[R][G];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float kf[8];
      kr[r].unpack(kf);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float d = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d = fmaf(qr[h][e], kf[e], d);
        s[r][h] = group16_sum(d);
      }
    }
    float pw[R][G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mb = st.m[h];
#pragma unroll
      for (int r = 0; r < R; ++r) mb = ok[r] ? fmaxf(mb, s[r][h]) : mb;
      const float corr = __builtin_amdgcn_exp2f(st.m[h] - mb);
      float lsum = 0.0f;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        pw[r][h] = ok[r] ? __builtin_amdgcn_exp2f(s[r][h] - mb) : 0.0f;
        lsum += pw[r][h];
      }
      st.l[h] = st.l[h] * corr + lsum;
      st.m[h] = mb;
#pragma unroll
      for (int e = 0; e < 8; ++e) st.acc[h][e] *= corr;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float vf[8];
      vr[r].unpack(vf);
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[h][e] = fmaf(pw[r][h], vf[e], st.acc[h][e]);
    }
  }
}

// Merge the 4 row slots of a wave (all lanes end with the merged state).
template <int G>
__device__ __forceinline__ void merge_slots(AttnState<G>& st) {
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float mo = __shfl_xor(st.m[h], o), lo = __shfl_xor(st.l[h], o);
      const float mn = fmaxf(st.m[h], mo);
      const float a = __builtin_amdgcn_exp2f(st.m[h] - mn), b = __builtin_amdgcn_exp2f(mo - mn);
      st.l[h] = st.l[h] * a + lo * b;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float ao = __shfl_xor(st.acc[h][e], o);
        st.acc[h][e] = st.acc[h][e] * a + ao * b;
      }
      st.m[h] = mn;
    }
  }
}

// Per-wave softmax state in LDS: red[w][h] = { m, l, acc[kD] }.
template <typename T, int G>
__device__ __forceinline__ void stash_wave_state(AttnState<G>& st, float* red) {
  merge_slots<G>(st);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane < 16) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float* dst = red + ((size_t)w * G + h) * (kD + 2);
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[2 + owned_dim<T>(lane, e)] = st.acc[h][e];
      if (lane == 0) {
        dst[0] = st.m[h];
        dst[1] = st.l[h];
      }
    }
  }
}

template <int G, int NW>
__device__ __forceinline__ void combine_waves(const float* red, int h, int d, float& m, float& l, float& acc) {
  m = kNegBig;
#pragma unroll
  for (int w = 0; w < NW; ++w) m = fmaxf(m, red[((size_t)w * G + h) * (kD + 2)]);
  l = 0.0f;
  acc = 0.0f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const float* src = red + ((size_t)w * G + h) * (kD + 2);
    const float f = __builtin_amdgcn_exp2f(src[0] - m);
    l = fmaf(src[1], f, l);
    acc = fmaf(src[2 + d], f, acc);
  }
}

// Build switch for the record of why the matrix cores are used: with -DPQC_VECTOR_ATTENTION bf16 caches take the
// vector-ALU attention above, like fp32 caches (a compile-time choice, there is no run-time dispatch between the two).
#ifdef PQC_VECTOR_ATTENTION
constexpr bool kMatrixCoreAttention = false;
#else
constexpr bool kMatrixCoreAttention = true;
#endif

// ------------------------------------------------------ attention, matrix cores
// bf16 caches.  Per wave and per tile of 16 listed rows:
//   S[token][head] = K_tile[16 x 128] . Q^T[128 x 16]     4 x v_mfma_f32_16x16x32_bf16
//   O[head][dim]  += P[head][token]  . V_tile[16 x 128]   8 x 2 x v_mfma_f32_16x16x16_bf16
// Operand layouts (lane l, quad = l / 16, col = l % 16):
//   16x16x32: A[m=col][k=8*quad+e], B[k=8*quad+e][n=col], D[m=4*quad+i][n=col]
//   16x16x16: A[m=col][k=4*quad+e], B[k=4*quad+e][n=col], D[m=4*quad+i][n=col]
// so the QK output (tokens 4*quad+i of head col) is, lane for lane, the A operand of
// the PV product.  Heads G..15 are zero padding.  K rows feed the matrix core straight
// from global memory (lane: row col, 16 bytes at dims 32*kk + 8*quad); V rows are
// transposed through a wave-private LDS tile (row stride 264 bytes: the four quads of
// a transposed read land in different banks).  P is split into two bf16 terms
// (p = hi + lo, error 2^-17) because one bf16 term alone would cost 2^-9 of the result.
//
// Softmax: a wave first computes the logits of a stage of up to kMfmaTiles tiles,
// takes its maximum per head, rescales O once if the maximum grew, then accumulates.
constexpr int kMfmaTiles = 2;          // tiles (of 16 rows) per stage and wave
constexpr int kVTileStride = 264;      // bytes per V row in the LDS transpose tile
constexpr int kVTileBytes = 16 * kVTileStride;

struct MfmaState {
  f32x4_t o[8];  // O[head 4*quad+i][dim 16*j + col]
  float m, l;    // head col, over this lane's tokens (log2 domain); merged across quads at the end
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    m = kNegBig;
    l = 0.0f;
  }
};

// Q^T fragments (B operand of the QK product) for this lane; heads >= G are zero.
__device__ __forceinline__ void load_q_frags(const bf16_t* __restrict__ q /* [G][kD] */, int G, bf16x8_t (&qf)[4]) {
  const int lane = threadIdx.x & 63, col = lane & 15, quad = lane >> 4;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (col < G) raw = *reinterpret_cast<const uint4*>(q + (size_t)col * kD + 32 * kk + 8 * quad);
    __builtin_memcpy(&qf[kk], &raw, 16);
  }
}

__device__ __forceinline__ unsigned bf16_round_bits(float f) {  // round to nearest even, finite inputs
  const unsigned u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// One stage = kMfmaTiles tiles.  Two stages are kept in registers: while one is being
// consumed the loads of the next are in flight, so a wave never sits without outstanding
// memory requests until its rows run out.  Loads are unconditional (positions past the
// end of the list re-read its last row, which the caches hold); masking happens on the
// logits.
struct MfmaStage {
  uint4 kr[kMfmaTiles][4], vr[kMfmaTiles][4];
};

template <class ListFn>
__device__ __forceinline__ void mfma_issue(const bf16_t* __restrict__ kbase, const bf16_t* __restrict__ vbase, int N,
                                           ListFn list, int count, int base, MfmaStage& g) {
  const int lane = threadIdx.x & 63, col = lane & 15, quad = lane >> 4;
#pragma unroll
  for (int tl = 0; tl < kMfmaTiles; ++tl) {
    int t = list(min(base + tl * 16 + col, count - 1));
    t = max(0, min(N - 1, t));
    const uint4* kp = reinterpret_cast<const uint4*>(kbase + (size_t)t * kD + 8 * quad);
    const uint4* vp = reinterpret_cast<const uint4*>(vbase + (size_t)t * kD + 8 * quad);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      g.kr[tl][kk] = kp[4 * kk];  // dims 32*kk + 8*quad .. +7
      g.vr[tl][kk] = vp[4 * kk];
    }
  }
}

__device__ __forceinline__ void mfma_consume(const MfmaStage& g, int count, int base, float scale_log2e,
                                             const bf16x8_t (&qf)[4], unsigned char* vt, MfmaState& st) {
  const int lane = threadIdx.x & 63, col = lane & 15, quad = lane >> 4;
  // logits of the stage
  f32x4_t s[kMfmaTiles];
  float mx = kNegBig;
#pragma unroll
  for (int tl = 0; tl < kMfmaTiles; ++tl) {
    s[tl] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (base + tl * 16 < count) {  // wave-uniform
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8_t a;
        __builtin_memcpy(&a, &g.kr[tl][kk], 16);
        s[tl] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[kk], s[tl], 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = base + tl * 16 + 4 * quad + i < count;
        s[tl][i] = ok ? s[tl][i] * scale_log2e : kNegBig;
        mx = fmaxf(mx, s[tl][i]);
      }
    }
  }
  // the stage's maximum per head (over the four quads: row_ror 16 and 32 of the wave), and the
  // one-off rescale of O
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float mnew = fmaxf(st.m, mx);
  const float corr = __builtin_amdgcn_exp2f(st.m - mnew);
  st.l *= corr;
  st.m = mnew;
  if (__any(corr != 1.0f)) {
    float cr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) cr[i] = __shfl(corr, 4 * quad + i);  // corr of head 4*quad+i lives in lane col == that head
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) st.o[j][i] *= cr[i];
  }
  // accumulate
#pragma unroll
  for (int tl = 0; tl < kMfmaTiles; ++tl) {
    if (base + tl * 16 < count) {
      // V tile -> LDS, row `col`, bytes 64*kk + 16*quad (two 8-byte stores: rows are 8-byte aligned)
      unsigned char* vrow = vt + col * kVTileStride + 16 * quad;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        *reinterpret_cast<uint2*>(vrow + 64 * kk) = make_uint2(g.vr[tl][kk].x, g.vr[tl][kk].y);
        *reinterpret_cast<uint2*>(vrow + 64 * kk + 8) = make_uint2(g.vr[tl][kk].z, g.vr[tl][kk].w);
      }
      // P = exp2(S - m), as hi + lo bf16 terms (masked rows hold kNegBig: P = 0)
      unsigned hi[4], lo[4];
      float psum = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(s[tl][i] - mnew);
        psum += p;
        hi[i] = bf16_round_bits(p);
        lo[i] = bf16_round_bits(p - __uint_as_float(hi[i] << 16));
      }
      st.l += psum;
      s16x4_t pa_hi, pa_lo;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pa_hi[i] = (short)hi[i];
        pa_lo[i] = (short)lo[i];
      }
      // the wave's LDS stores must land before its lanes read each other's rows
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const unsigned short* vt16 = reinterpret_cast<const unsigned short*>(vt);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        s16x4_t vb;  // B[k = token 4*quad+e][n = dim 16*j + col]
#pragma unroll
        for (int e = 0; e < 4; ++e) vb[e] = (short)vt16[(4 * quad + e) * (kVTileStride / 2) + 16 * j + col];
        st.o[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa_hi, vb, st.o[j], 0, 0, 0);
        st.o[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa_lo, vb, st.o[j], 0, 0, 0);
      }
      // tile fully read before the next tile overwrites it
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }
}

// Rows list(first), list(first+1), ... in stages of 16*kMfmaTiles positions, `stride` apart.
template <class ListFn>
__device__ __forceinline__ void mfma_attend(const bf16_t* __restrict__ kbase, const bf16_t* __restrict__ vbase, int N,
                                            ListFn list, int count, int first, int stride, float scale_log2e,
                                            const bf16x8_t (&qf)[4], unsigned char* vt /* wave-private LDS [kVTileBytes] */,
                                            MfmaState& st) {
  if (first >= count) return;  // wave-uniform
  MfmaStage ga, gb;
  int base = first;
  mfma_issue(kbase, vbase, N, list, count, base, ga);
  for (;;) {
    mfma_issue(kbase, vbase, N, list, count, base + stride, gb);
    PQC_LOADS_ISSUED();
    mfma_consume(ga, count, base, scale_log2e, qf, vt, st);
    base += stride;
    if (base >= count) break;
    mfma_issue(kbase, vbase, N, list, count, base + stride, ga);
    PQC_LOADS_ISSUED();
    mfma_consume(gb, count, base, scale_log2e, qf, vt, st);
    base += stride;
    if (base >= count) break;
  }
}

// Per-wave state -> red[w][h] = { m, l, acc[kD] } (same slots as the vector path).
template <int G>
__device__ __forceinline__ void mfma_stash_wave_state(MfmaState& st, float* red) {
  const int lane = threadIdx.x & 63, col = lane & 15, quad = lane >> 4, w = threadIdx.x >> 6;
  // the four quads of head `col` hold partial sums under one shared maximum
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (quad == 0 && col < G) {
    float* dst = red + ((size_t)w * G + col) * (kD + 2);
    dst[0] = st.m;
    dst[1] = l;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int h = 4 * quad + i;
    if (h < G) {
      float* dst = red + ((size_t)w * G + h) * (kD + 2) + 2;
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[16 * j + col] = st.o[j][i];
    }
  }
}

}  // namespace pqc
