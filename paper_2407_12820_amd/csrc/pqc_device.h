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
struct Workspace {
  float2* ctl;                 // [units]            (lo, bins per unit of score)
  float* lut;                  // [units][M][C]
  unsigned* hist;              // [units][kNB]       zero between calls
  unsigned long long* stage;   // [units][nblkC][tokC] selected ids (front, int32) / candidates (back, u64)
  int2* stage_cnt;             // [units][nblkC]     (selected, candidates)
  float* partials;             // [units][npart][G][kD+2]
};

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

__device__ __forceinline__ int score_bin(float s, float lo, float inv_w) {
  // monotone non-decreasing in s: subtraction, multiplication by a non-negative
  // constant and truncation all preserve order
  int b = __float2int_rz((s - lo) * inv_w);
  return max(0, min(kNB - 1, b));
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

template <typename T, int NT>
__device__ __forceinline__ void build_lut(const T* __restrict__ q /* [G][kD] of this unit */,
                                          const float* __restrict__ cent /* [M][C][Dm] */, int G, int M,
                                          int C, int Dm, float* lut, float* qs, float* red, float* lo_out,
                                          float* inv_w_out) {
  const int tid = threadIdx.x;
  if (tid < kD) {
    float a = load_as_float<T>(q, tid);
    for (int h = 1; h < G; ++h) a = __fadd_rn(a, load_as_float<T>(q, h * kD + tid));
    qs[tid] = a;
  }
  __syncthreads();
  for (int e = tid; e < M * C; e += NT) {
    const int j = e / C, c = e - j * C;
    const float4* row = reinterpret_cast<const float4*>(cent + (size_t)e * Dm);
    const float* qj = qs + j * Dm;
    float p = 0.0f;
    for (int x = 0; x < Dm / 4; ++x) {
      float4 cv = row[x];
      p = __fmaf_rn(qj[4 * x + 0], cv.x, p);
      p = __fmaf_rn(qj[4 * x + 1], cv.y, p);
      p = __fmaf_rn(qj[4 * x + 2], cv.z, p);
      p = __fmaf_rn(qj[4 * x + 3], cv.w, p);
    }
    lut[j * kLutRow + c] = p;
  }
  __syncthreads();
  const int lane = tid & 63, w = tid >> 6;
  for (int j = w; j < M; j += NT / 64) {
    float mn = INFINITY, mx = -INFINITY;
    for (int c = lane; c < C; c += 64) {
      float v = lut[j * kLutRow + c];
      mn = fminf(mn, v);
      mx = fmaxf(mx, v);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      mn = fminf(mn, __shfl_xor(mn, o));
      mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    if (lane == 0) {
      red[j] = mn;
      red[8 + j] = mx;
    }
  }
  __syncthreads();
  float lo = red[0], hi = red[8];
  for (int j = 1; j < M; ++j) {
    lo = __fadd_rn(lo, red[j]);
    hi = __fadd_rn(hi, red[8 + j]);
  }
  const float width = hi - lo;
  *lo_out = lo;
  *inv_w_out = (width > 1e-30f) ? (float)kNB / width : 0.0f;
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

// Where a kernel takes its scores from: PQ codes through the LDS table (the decode
// path) or a score array in global memory (the stand-alone top-k stage).
template <int M_>
struct CodeSource {
  static constexpr int M = M_;
  static constexpr bool kFromCodes = true;
  const typename CodeWord<M_>::type* codes;  // this unit's [N] code words
  const float* lut;                          // LDS
  __device__ __forceinline__ float score(int t) const { return score_from_word<M_>(codes[t], lut); }
};
struct ScoreSource {
  static constexpr int M = 0;
  static constexpr bool kFromCodes = false;
  const float* scores;  // this unit's [N] scores
  __device__ __forceinline__ float score(int t) const { return scores[t]; }
};

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

__device__ __forceinline__ float group16_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  x += __shfl_xor(x, 4);
  x += __shfl_xor(x, 8);
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
