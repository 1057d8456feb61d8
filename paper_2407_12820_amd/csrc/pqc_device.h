// Device-side building blocks of libpqcache (gfx950, wave64).
//
// Everything here is a __device__ template; the kernels that use them live in
// pqc_kernels.h and are instantiated by the launch files.  Citations are to the
// paper's sections (PQ search: Section 2.2 and Section 3.1 step 4; top-k: Section
// 3.1 steps 4-5 and Section 3.2; selective attention: Section 2.1 and Section 3.1
// step 6).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pqc {

constexpr int kNB = 2048;        // score bins of the one-pass threshold search
constexpr int kD = 128;          // head dimension
constexpr int kLutRow = 256;     // LDS stride of one partition's table (max centroids)
constexpr int kCandLds = 1024;   // boundary-bin candidates resolved inside LDS
constexpr float kNegBig = -1.0e30f;

struct bf16_t {
  uint16_t bits;
};

// Geometry of one decode step, passed by value to every kernel.
struct Shape {
  int B, Hq, Hkv, G, N, M, C, Dm, K, I, L, Ktot;
  int tokA, nblkA;  // histogram kernel: tokens per workgroup, workgroups per unit
  int tokC, nblkC;  // select kernel: tokens per workgroup, workgroups per unit
  int rowsP, nblkP; // list-attention kernel: rows per workgroup, workgroups per unit
  int npart;        // partial slots per unit
  float scale_log2e;
};

// Device pointers carved out of the caller's workspace.
struct BinParams;
struct Workspace {
  BinParams* ctl;              // [units]            score -> bin map of the unit
  float* lut;                  // [units][M][C]
  unsigned* hist;              // [units][kNB]       zero between calls
  unsigned long long* stage;   // [units][nblkC][tokC] selected ids (front, int32) / candidates (back, u64)
  int2* stage_cnt;             // [units][nblkC]     (selected, candidates)
  float* partials;             // [units][npart][G][kD+2]
#ifdef PQC_TRACE
  unsigned long long* trace;   // [3 kernels][kTraceWgs][kTraceSlots] cycle stamps (debug builds only)
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
#else
#define PQC_MARK(ws, kid, slot) \
  do {                          \
  } while (0)
#endif

// ---------------------------------------------------------------- small helpers
__device__ __forceinline__ unsigned score_key(float f) {
  // order-preserving map float -> unsigned (larger score, larger key); -0 == +0
  f += 0.0f;
  unsigned u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

__device__ __forceinline__ unsigned long long make_composite(float score, int token) {
  // larger composite = ranks first: higher score, then lower token index
  return ((unsigned long long)score_key(score) << 32) | (unsigned long long)(0xffffffffu - (unsigned)token);
}

__device__ __forceinline__ int composite_token(unsigned long long c) {
  return (int)(0xffffffffu - (unsigned)(c & 0xffffffffull));
}

// Monotone map score -> bin.  Three linear pieces: kTailBins coarse bins below c0,
// kNB - 2*kTailBins fine bins over [c0, c1], kTailBins coarse bins above c1.  The
// piece is chosen by exact comparisons and each piece is clamped to its own bin
// range, so the map is non-decreasing in s whatever the parameters are (inside a
// piece: subtraction, multiplication by a non-negative constant and truncation all
// preserve order).  Only the number of boundary-bin candidates depends on how well
// [c0, c1] brackets the K-th largest score; the selection itself never does.
constexpr int kTailBins = 64;
constexpr int kFineBins = kNB - 2 * kTailBins;
struct BinParams {
  float lo, c0, c1, inv_lo, inv_c, inv_hi, pad0, pad1;
};
__device__ __forceinline__ int score_bin(float s, const BinParams& bp) {
  if (s < bp.c0) return max(0, min(kTailBins - 1, __float2int_rz((s - bp.lo) * bp.inv_lo)));
  if (s <= bp.c1) return kTailBins + max(0, min(kFineBins - 1, __float2int_rz((s - bp.c0) * bp.inv_c)));
  return kTailBins + kFineBins + max(0, min(kTailBins - 1, __float2int_rz((s - bp.c1) * bp.inv_hi)));
}
// Bin layout from bounds lo <= score <= hi and a location/spread estimate of the scores:
// the fine piece covers [mean - 3 sd, mean + 5 sd] (the K-th largest score of a
// selection of a few percent to a half of the tokens lies there for bell-shaped scores).
__device__ __forceinline__ BinParams make_bins(float lo, float hi, float mean, float sd) {
  BinParams bp;
  bp.lo = lo;
  bp.c0 = fmaxf(lo, mean - 3.0f * sd);
  bp.c1 = fminf(hi, mean + 5.0f * sd);
  if (!(bp.c1 > bp.c0)) {  // degenerate spread: one fine piece over everything
    bp.c0 = lo;
    bp.c1 = hi;
  }
  const float wl = bp.c0 - lo, wc = bp.c1 - bp.c0, wh = hi - bp.c1;
  bp.inv_lo = (wl > 1e-30f && wl < 3e38f) ? (float)kTailBins / wl : 0.0f;
  bp.inv_c = (wc > 1e-30f && wc < 3e38f) ? (float)kFineBins / wc : 0.0f;
  bp.inv_hi = (wh > 1e-30f && wh < 3e38f) ? (float)kTailBins / wh : 0.0f;
  bp.pad0 = bp.pad1 = 0.0f;
  return bp;
}

// Exclusive prefix sum over the threads of a workgroup (NT threads, multiple of 64).
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int v, int* total, int* sm /* [2*(NT/64)+1] */) {
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int n = __shfl_up(inc, o);
    if (lane >= o) inc += n;
  }
  if (lane == 63) sm[w] = inc;
  __syncthreads();
  if (w == 0) {
    int s = lane < NW ? sm[lane] : 0;
    int si = s;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int n = __shfl_up(si, o);
      if (lane >= o) si += n;
    }
    if (lane < NW) sm[NW + lane] = si - s;
    if (lane == NW - 1) sm[2 * NW] = si;
  }
  __syncthreads();
  int res = inc - v + sm[NW + w];
  *total = sm[2 * NW];
  __syncthreads();
  return res;
}

// --------------------------------------------------------------- look-up table
// Section 2.2 (search) / Section 3.1 step 4: table[j][c] = qs[j*Dm..] . cent[j][c][..]
// with qs the sum of the group's query heads.  Fixed fp32 order: head order for
// the sum, one fused multiply-add chain per entry.  Also derives bounds on every
// possible score: lo = sum_j min_c table[j][c], hi likewise with max, added in the
// same order as a score, so that lo <= score <= hi holds in fp32.
//   lut   LDS [M][kLutRow]      qs  LDS [kD]      red LDS [2*8]
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
// padded LDS tile of kLutTileFloats floats -> one thread per table entry runs the chain.
constexpr int kLutTileFloats = 8192;
template <typename T, int NT, int M>
__device__ __forceinline__ BinParams build_lut(const T* __restrict__ q /* [G][kD] of this unit */,
                                               const float* __restrict__ cent /* [M][C][Dm] */, int G, int C,
                                               float* lut, float* qs, float* red /* [4*8] */,
                                               float* tile /* [kLutTileFloats + kLutTileFloats/Dm] */) {
  constexpr int Dm = kD / M;
  constexpr int VPG = kLutTileFloats / (4 * NT);      // float4 per thread per tile
  constexpr int NG = (256 * kD) / kLutTileFloats;      // tiles at the largest C
  constexpr bool kPrefetchAll = (VPG * NG <= 8);       // keep every tile's loads in flight
  const int tid = threadIdx.x;
  const int total = M * C * Dm;                        // floats, a multiple of 4
  const float4* cent4 = reinterpret_cast<const float4*>(cent);
  float4 v[kPrefetchAll ? NG : 1][VPG];
  if constexpr (kPrefetchAll) {
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int x = 0; x < VPG; ++x) {
        const int f = g * (kLutTileFloats / 4) + x * NT + tid;
        if (4 * f < total) v[g][x] = cent4[f];
      }
  }
  if (tid < kD) {
    float a = load_as_float<T>(q, tid);
    for (int h = 1; h < G; ++h) a = __fadd_rn(a, load_as_float<T>(q, h * kD + tid));
    qs[tid] = a;
  }
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    if (g * kLutTileFloats < total) {  // uniform
      if constexpr (!kPrefetchAll) {
#pragma unroll
        for (int x = 0; x < VPG; ++x) {
          const int f = g * (kLutTileFloats / 4) + x * NT + tid;
          if (4 * f < total) v[0][x] = cent4[f];
        }
      }
      if (g > 0) __syncthreads();  // previous tile fully consumed
#pragma unroll
      for (int x = 0; x < VPG; ++x) {
        const int fl = (x * NT + tid) * 4;  // float index inside the tile
        if (g * kLutTileFloats + fl < total) {
          const float4 cv = v[kPrefetchAll ? g : 0][x];
          const int row = fl / Dm, col = fl % Dm;  // Dm is a multiple of 4: one row per float4
          float* dst = tile + row * (Dm + 1) + col;
          dst[0] = cv.x; dst[1] = cv.y; dst[2] = cv.z; dst[3] = cv.w;
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
  __syncthreads();
  // per table: min, max, sum, sum of squares (one wave per table, fixed reduction tree)
  const int lane = tid & 63, w = tid >> 6;
  for (int j = w; j < M; j += NT / 64) {
    float mn = INFINITY, mx = -INFINITY, sm = 0.0f, sq = 0.0f;
    for (int c = lane; c < C; c += 64) {
      const float v = lut[j * kLutRow + c];
      mn = fminf(mn, v);
      mx = fmaxf(mx, v);
      sm += v;
      sq = fmaf(v, v, sq);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      mn = fminf(mn, __shfl_xor(mn, o));
      mx = fmaxf(mx, __shfl_xor(mx, o));
      sm += __shfl_xor(sm, o);
      sq += __shfl_xor(sq, o);
    }
    if (lane == 0) {
      red[j] = mn;
      red[8 + j] = mx;
      red[16 + j] = sm;
      red[24 + j] = sq;
    }
  }
  __syncthreads();
  // bounds are added in the same order as a score, so lo <= score <= hi holds in fp32
  float lo = red[0], hi = red[8];
  const float invC = 1.0f / (float)C;
  float mean = red[16] * invC, var = fmaxf(0.0f, red[24] * invC - (red[16] * invC) * (red[16] * invC));
  for (int j = 1; j < M; ++j) {
    lo = __fadd_rn(lo, red[j]);
    hi = __fadd_rn(hi, red[8 + j]);
    const float mj = red[16 + j] * invC;
    mean += mj;
    var += fmaxf(0.0f, red[24 + j] * invC - mj * mj);
  }
  return make_bins(lo, hi, mean, sqrtf(var));
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

template <int NT>
__device__ __forceinline__ Threshold find_threshold(const unsigned* __restrict__ ghist, int K, int* sm /* [2*(NT/64)+1+4] */) {
  constexpr int PER = kNB / NT;
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x;
  unsigned h[PER];
  int sum = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    h[e] = ghist[kNB - 1 - (tid * PER + e)];
    sum += (int)h[e];
  }
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

// ------------------------------------------------------------------- attention
// Section 2.1 restricted to listed tokens (Section 3.1 step 6).  Lane layout inside
// a wave: sub = lane & 15 owns 8 of the 128 dimensions of a row, slot = lane >> 4
// picks one of 4 rows handled at once; a 16-lane group reads one contiguous row.
// Logits are kept in the log2 domain (q is pre-multiplied by scale*log2(e)).
template <typename T>
struct RowRaw;
template <>
struct RowRaw<bf16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const bf16_t* base, int t, int sub) {
    a = *reinterpret_cast<const uint4*>(base + (size_t)t * kD + sub * 8);
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
};
template <>
struct RowRaw<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* base, int t, int sub) {
    a = *reinterpret_cast<const float4*>(base + (size_t)t * kD + sub * 4);
    b = *reinterpret_cast<const float4*>(base + (size_t)t * kD + 64 + sub * 4);
  }
  __device__ __forceinline__ void zero() {
    a = make_float4(0, 0, 0, 0);
    b = a;
  }
  __device__ __forceinline__ void unpack(float (&f)[8]) const {
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
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
__device__ __forceinline__ void load_query(const T* __restrict__ q /* [G][kD] */, float scale_log2e, float (&qr)[G][8]) {
  const int sub = threadIdx.x & 15;
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) qr[h][e] = load_as_float<T>(q, h * kD + owned_dim<T>(sub, e)) * scale_log2e;
}

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float group16_sum(float x) {
  x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]: neighbour in the pair
  x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]: other pair of the quad
  x += dpp_move<0x141>(x);  // row_half_mirror: other quad of the half row
  x += dpp_move<0x140>(x);  // row_mirror: other half of the row
  return x;
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

// Combine the waves of a workgroup through LDS and return, for output element
// (h, d) = (o / kD, o % kD), o = threadIdx.x + i*NT, the merged (m, l, acc).
//   red  LDS [NW][G][kD+2]
template <typename T, int G, int NW>
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

}  // namespace pqc
