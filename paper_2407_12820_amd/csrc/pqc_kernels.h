// Kernels of libpqcache (gfx950).  Grid layout: blockIdx.y = unit (sequence b, KV
// head g); blockIdx.x = workgroup inside the unit (query head for finalize_kernel).
//
// Decode path (pqc_decode), three launches, every dependency at a kernel boundary:
//   hist_kernel      table -> scan codes -> histogram of scores over kNB bins, and every
//                    token's bin number left behind for the next kernel
//   select_kernel    threshold bin from the histogram -> tokens whose stored bin lies
//                    above it (and the two windows) are listed in ascending order
//                    without atomics and attended at once; tokens inside the bin
//                    ("candidates") are recorded with their logits and V row
//   finalize_kernel  one workgroup per query head ranks the candidates and folds the
//                    admitted ones and all partial softmax states into the output;
//                    copy workgroups beside them write the indices and zero the unit's
//                    histogram and record counter again, which nothing reads after the
//                    select kernel: every call leaves them as it found them
//
// Codes are read 16 bytes at a time (P = 16/M tokens).  A unit's codes start at byte
// u*N*M, which need not be 16-byte aligned: chunks are laid over the aligned-down
// address, so chunk 0 may begin with up to P-1 "phantom" tokens of the previous unit
// and the last chunk may end with phantoms; both are masked by the token range check.
#pragma once
#include "pqc_device.h"

namespace pqc {

constexpr int kMaxVecA = 4;   // 16-byte code chunks per thread, histogram kernel

// ------------------------------------------------------------------ sources
// Where a kernel takes its scores from: PQ codes through the LDS table (the decode
// path) or a score array in global memory (the stand-alone top-k stage).
template <int M_>
struct CodeChunks {
  static constexpr int M = M_;
  static constexpr int P = 16 / M_;  // tokens per chunk
  static constexpr bool kFromCodes = true;
  using Raw = uint4;
  const uint8_t* all;       // whole code tensor
  long long total_bytes;    // its size
  long long unit_byte0;     // aligned-down byte offset of this unit's codes
  int lead;                 // phantom tokens before token 0
  const float* lut;         // LDS
  const uint8_t* spare;     // 16 readable bytes of any content
  __device__ __forceinline__ void init(const void* ptr, int u, int N, int units, const float* lut_, const void* spare16) {
    all = static_cast<const uint8_t*>(ptr);
    spare = static_cast<const uint8_t*>(spare16);
    total_bytes = (long long)units * N * M;
    const long long ob = (long long)u * N * M;
    unit_byte0 = ob & ~15ll;
    lead = (int)((ob - unit_byte0) / M);
    lut = lut_;
  }
  // Unconditional 16-byte load (straight-line code keeps many loads in flight, and lets the
  // compiler count them when it waits for earlier ones): a chunk at or beyond the tensor's last
  // full 16 bytes is redirected to that last full chunk (to the spare bytes if the tensor has
  // none), and fix_tail() patches the one chunk that holds the tensor's ragged end afterwards.
  __device__ __forceinline__ Raw load(int chunk) const {
    const long long last_full = (total_bytes & ~15ll) - 16;  // < 0 for tensors under 16 bytes
    long long off = unit_byte0 + 16ll * chunk;
    off = off < last_full ? off : last_full;
    off = off > 0 ? off : 0;
    const uint8_t* p = total_bytes < 16 ? spare : all + off;
    return *reinterpret_cast<const uint4*>(p);
  }
  __device__ __forceinline__ void fix_tail(Raw& r, int chunk) const {
    const long long off = unit_byte0 + 16ll * chunk;
    if (off + 16 > total_bytes && off < total_bytes) {  // at most one chunk in the whole tensor
      unsigned w[4] = {0u, 0u, 0u, 0u};
      for (int b = 0; b < 16; ++b)
        if (off + b < total_bytes) w[b >> 2] |= (unsigned)all[off + b] << (8 * (b & 3));
      r = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
  __device__ __forceinline__ float score(const Raw& r, int i) const { return score_from_word<M>(chunk_word<M>(r, i), lut); }
  // one token: the load (issue early) and the table look-up (after the table is ready)
  using One = typename CodeWord<M>::type;
  __device__ __forceinline__ One load_one(int t, int u, int N) const {
    const uint8_t* p = all + ((long long)u * N + t) * M;
    One w = 0;
#pragma unroll
    for (int j = 0; j < M; ++j) w |= (One)p[j] << (8 * j);
    return w;
  }
  __device__ __forceinline__ float score_one(One w) const { return score_from_word<M>(w, lut); }
  __device__ __forceinline__ float score_of_token(int t, int u, int N) const { return score_one(load_one(t, u, N)); }
};

struct ScoreChunks {
  static constexpr int M = 0;
  static constexpr int P = 4;
  static constexpr bool kFromCodes = false;
  struct Raw {
    float f[4];
  };
  const float* scores;  // this unit's [N] scores
  int n;
  int lead;
  __device__ __forceinline__ void init(const void* ptr, int u, int N, int, const float*, const void*) {
    scores = static_cast<const float*>(ptr) + (size_t)u * N;
    n = N;
    lead = 0;
  }
  __device__ __forceinline__ Raw load(int chunk) const {
    Raw r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      long long t = (long long)chunk * 4 + i;
      t = t < n ? t : n - 1;  // clamped: straight-line loads; tokens >= n are masked by the caller
      r.f[i] = scores[t];
    }
    return r;
  }
  __device__ __forceinline__ void fix_tail(Raw&, int) const {}
  __device__ __forceinline__ float score(const Raw& r, int i) const { return r.f[i]; }
  using One = float;
  __device__ __forceinline__ One load_one(int t, int, int) const { return scores[t]; }
  __device__ __forceinline__ float score_one(One w) const { return w; }
  __device__ __forceinline__ float score_of_token(int t, int, int) const { return scores[t]; }
};

// ------------------------------------------------------------------ utilities
__global__ void reset_kernel(unsigned* a, size_t na) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < na) a[i] = 0u;
}

// Stand-alone table (pqc_lut).
template <typename T, int M>
__global__ __launch_bounds__(256) void lut_kernel(Shape s, const T* __restrict__ q, const float* __restrict__ cent,
                                                  float* __restrict__ table) {
  __shared__ float lut[M * kLutRow];
  __shared__ float qs[kD];
  __shared__ float red[32];
  __shared__ float tile[lut_tile_floats(256, M, 256)];
  const int u = blockIdx.y, b = u / s.Hkv, g = u % s.Hkv;
  build_lut<T, 256, M>(q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * M * s.C * (kD / M), s.G, s.C, lut,
                       qs, red, tile, [](int) {}, []() {});
  for (int e = threadIdx.x; e < M * s.C; e += 256) table[(size_t)u * M * s.C + e] = lut[(e / s.C) * kLutRow + (e % s.C)];
}

// Stand-alone scan (pqc_scan): scores[N], -inf inside the two windows.
template <int M>
__global__ __launch_bounds__(256) void scan_kernel(Shape s, const float* __restrict__ table,
                                                   const uint8_t* __restrict__ codes, float* __restrict__ scores) {
  __shared__ float lut[M * kLutRow];
  const int u = blockIdx.y;
  for (int e = threadIdx.x; e < M * s.C; e += 256) lut[(e / s.C) * kLutRow + (e % s.C)] = table[(size_t)u * M * s.C + e];
  __syncthreads();
  using W = typename CodeWord<M>::type;
  const W* cw = reinterpret_cast<const W*>(codes) + (size_t)u * s.cap;
  const int t0 = blockIdx.x * 2048;
  for (int t = t0 + threadIdx.x; t < min(t0 + 2048, s.N); t += 256) {
    const bool mid = t >= s.I && t < s.N - s.L;
    scores[(size_t)u * s.N + t] = mid ? score_from_word<M>(cw[t], lut) : -INFINITY;
  }
}

// Score range of the middle tokens of a score array (stand-alone top-k only).
__global__ __launch_bounds__(1024) void score_range_kernel(Shape s, const float* __restrict__ scores,
                                                           float2* __restrict__ range) {
  __shared__ float smn[16], smx[16];
  const int u = blockIdx.y;
  float mn = INFINITY, mx = -INFINITY;
  for (int t = s.I + threadIdx.x; t < s.N - s.L; t += 1024) {
    const float v = scores[(size_t)u * s.N + t];
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  mn = wave_min(mn);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) {
    smn[threadIdx.x >> 6] = mn;
    smx[threadIdx.x >> 6] = mx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w) {
      mn = fminf(mn, smn[w]);
      mx = fmaxf(mx, smx[w]);
    }
    range[u] = make_float2(mn, mx);
  }
}

// ------------------------------------------------------------- 1. histogram
// SRC = CodeChunks<M>: builds the unit's table first; score bounds come from the table.
// SRC = ScoreChunks: bounds come from score_range_kernel.  Every workgroup of a unit
// then derives the same bin layout from the same sampled tokens (workgroup 0 publishes
// table and layout for the select kernel) and counts its own tokens.  Workgroups of a
// unit spread their counts over histCopies replicas.
// VW: 16-byte pieces of the centroid tensor per thread (1024 * 4 * VW floats cover the unit's M*C*Dm);
// VA: 16-byte chunks of codes (or scores) per thread (1024 * VA chunks cover the workgroup's tokA tokens).
// Both are template parameters so that no thread issues loads it does not need: the loads of a workgroup's
// sixteen waves go through one address unit, 64 bytes per clock, and redundant ones cost as much as real ones.
template <typename T, class SRC, int VW, int VA>
__global__ __launch_bounds__(1024) void hist_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                    const float* __restrict__ cent, const void* __restrict__ src_ptr) {
  constexpr int NT = 1024, P = SRC::P;
  static_assert(VA >= 1 && VA <= kMaxVecA, "chunks per thread");
  constexpr int LM = SRC::kFromCodes ? SRC::M : 1;
  __shared__ float lut[LM * kLutRow];
  __shared__ __attribute__((aligned(16))) float qs[kD];
  __shared__ float red[32];
  extern __shared__ __attribute__((aligned(16))) float tile[];  // lut_tile_floats(NT, LM, C) floats when the source is codes
  __shared__ unsigned hist[kNB];
  __shared__ int scan_sm[2 * (NT / 64) + 1 + 2];
  const int tid = threadIdx.x, units = s.B * s.Hkv;
  // Workgroups are handed to the 8 XCDs round-robin in launch order (x fastest).  The
  // workgroups of a unit all read that unit's centroids, so eight units at a time are
  // interleaved: the workgroups of one unit then share an XCD and its L2.
  int u = blockIdx.y, bx = blockIdx.x;
  {
    const int nx = gridDim.x, lin = blockIdx.y * nx + blockIdx.x;
    if (lin < (units & ~7) * nx) {
      const int i = lin % (8 * nx);
      u = (lin / (8 * nx)) * 8 + (i & 7);
      bx = i >> 3;
    }
  }
  PQC_MARK(ws, 0, 0);
#ifdef PQC_TRACE
  PQC_NOTE(ws, 0, 15, (__builtin_amdgcn_s_getreg(20 | (3 << 11)) & 15) | (u << 8));  // XCC_ID[3:0], unit
#endif
  SRC src;
  const int src_stride = SRC::kFromCodes ? s.cap : s.N;  // tokens between units: code tensor, or dense score array
  src.init(src_ptr, u, src_stride, units, lut, ws.hist);
  // this workgroup's chunks and this thread's sample: the loads are issued before anything else,
  // except that a table build puts its centroid loads in front of them
  const int chunks = s.tokA / P, chunk0 = bx * chunks;
  typename SRC::Raw raw[VA];
  typename SRC::One sample;
  const bool have_sample = tid < s.sampleN;
  auto issue_loads = [&]() {
#pragma unroll
    for (int v = 0; v < VA; ++v) raw[v] = src.load(chunk0 + min(v * NT + tid, chunks - 1));
    const int sample_i = min(tid, s.sampleN - 1);
    sample = src.load_one(min(s.N - 1, s.I + (int)(((long long)sample_i * max(0, s.N - s.I - s.L)) / s.sampleN)), u, src_stride);
  };
  float2 bounds;
  if constexpr (SRC::kFromCodes) {
    const int b = u / s.Hkv, g = u % s.Hkv;
    for (int i = tid; i < kNB; i += NT) hist[i] = 0u;
    auto mark = [&](int slot) { PQC_MARK(ws, 0, slot); };
    bounds = build_lut<T, NT, LM, decltype(mark), decltype(issue_loads), VW>(
        q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * LM * s.C * (kD / LM), s.G, s.C, lut, qs, red, tile,
        mark, issue_loads);
    if (bx == 0)
      for (int e = tid; e < LM * s.C; e += NT) ws.lut[(size_t)u * LM * s.C + e] = lut[(e / s.C) * kLutRow + (e % s.C)];
  } else {
    issue_loads();
    PQC_LOADS_ISSUED();
    for (int i = tid; i < kNB; i += NT) hist[i] = 0u;
    bounds = ws.range[u];
    __syncthreads();
  }
  PQC_MARK(ws, 0, 1);
#pragma unroll
  for (int v = 0; v < VA; ++v) src.fix_tail(raw[v], chunk0 + min(v * NT + tid, chunks - 1));
  const BinParams bp =
      sample_window<NT>(bounds.x, bounds.y, src.score_one(sample), have_sample, s.rankHi, s.rankLo, hist, scan_sm);
  if (bx == 0 && tid == 0) ws.ctl[u] = bp;
  const float b_c0 = bp.c0, b_c1 = bp.c1, b_ic = bp.inv_c, b_ihi = bp.inv_hi;
  PQC_MARK(ws, 0, 2);
  // most tokens score below the window: they are counted in a register (bin 0), the rest
  // go to their LDS bin (an LDS atomic costs in proportion to the lanes that take part)
  int n_low = 0;
  unsigned short* bins_u = ws.bins + (size_t)u * s.binStride;
#pragma unroll
  for (int v = 0; v < VA; ++v) {
    if (v * NT + tid < chunks) {
      const int t0 = (chunk0 + v * NT + tid) * P - src.lead;
      unsigned st[P];  // what the select kernel will read back: bin + 1, or the window mark
      if (t0 >= s.I && t0 + P <= s.N - s.L) {  // all P tokens are middle tokens (all but the chunks at the two ends)
#pragma unroll
        for (int i = 0; i < P; ++i) {
          const float sc = src.score(raw[v], i);
          const int bin = score_bin(sc, b_c0, b_c1, b_ic, b_ihi);
          if (!(sc < b_c0)) atomicAdd(&hist[bin], 1u);
          n_low += sc < b_c0 ? 1 : 0;
          st[i] = (unsigned)bin + 1u;
        }
      } else {
#pragma unroll
        for (int i = 0; i < P; ++i) {
          const int t = t0 + i;
          const float sc = src.score(raw[v], i);
          const bool mid = t >= s.I && t < s.N - s.L;
          const int bin = score_bin(sc, b_c0, b_c1, b_ic, b_ihi);
          if (mid && !(sc < b_c0)) atomicAdd(&hist[bin], 1u);
          n_low += (mid && sc < b_c0) ? 1 : 0;
          st[i] = mid ? (unsigned)bin + 1u : kBinWindow;
        }
      }
      if (src.lead == 0 && t0 + P <= s.N) {  // the usual case: aligned, all P tokens exist
        if constexpr (P == 1) {
          bins_u[t0] = (unsigned short)st[0];
        } else {
          unsigned pw[P / 2];
#pragma unroll
          for (int i = 0; i < P / 2; ++i) pw[i] = st[2 * i] | (st[2 * i + 1] << 16);
          if constexpr (P == 2) *reinterpret_cast<unsigned*>(bins_u + t0) = pw[0];
          if constexpr (P == 4) *reinterpret_cast<uint2*>(bins_u + t0) = make_uint2(pw[0], pw[1]);
          if constexpr (P >= 8) {
#pragma unroll
            for (int i = 0; i < P / 8; ++i)
              reinterpret_cast<uint4*>(bins_u + t0)[i] = make_uint4(pw[4 * i], pw[4 * i + 1], pw[4 * i + 2], pw[4 * i + 3]);
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < P; ++i)
          if (t0 + i >= 0 && t0 + i < s.N) bins_u[t0 + i] = (unsigned short)st[i];
      }
    }
  }
  n_low = wave_last(wave_inclusive_scan(n_low));
  if ((tid & 63) == 0 && n_low) atomicAdd(&hist[0], (unsigned)n_low);
  __syncthreads();
  PQC_MARK(ws, 0, 3);
  unsigned* gh = ws.hist + ((size_t)u * s.histCopies + (bx % s.histCopies)) * kNB;
  for (int i = tid; i < kNB; i += NT)
    if (hist[i]) atomicAdd(&gh[i], hist[i]);
  PQC_MARK(ws, 0, 4);
}

// ---------------------------------------------------- 2. select (+ attention)
// One workgroup owns tokens [blockIdx.x*tokC, +tokC) of its unit; its 4 waves each own
// a contiguous quarter.  The histogram kernel left every token's bin behind, so a token
// is classified by comparing that number with the threshold bin.  Per wave, lanes hold
// 8 consecutive tokens, counts are prefix-summed across lanes, and the wave appends to
// its own LDS segment: selected tokens (ascending) from the front, boundary-bin
// candidates from the back.  SRC is only used to score the few candidates exactly.
constexpr int kMaxVecC = 4;  // 8-token groups per lane (tokC <= 8192)

// PAIRS (M = 2 only): there is no histogram kernel in front; the threshold comes from the
// code-pair counts (pair_threshold) and tokens are classified by their exact score keys.
template <typename T, int G, class SRC, bool ATTN, bool PAIRS = false>
__global__ __launch_bounds__(256, 2) void select_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                     const T* __restrict__ kc, const T* __restrict__ vc,
                                                     const void* __restrict__ src_ptr,
                                                     const float* __restrict__ cent = nullptr,
                                                     const unsigned* __restrict__ pair_counts = nullptr,
                                                     int uncounted = -1 /* PAIRS: a window token not in the counts yet */) {
  constexpr int NT = 256, NW = 4;
  constexpr bool kMfma = ATTN && sizeof(T) == 2 && kMatrixCoreAttention;
  static_assert(!PAIRS || (SRC::kFromCodes && SRC::M == 2), "pair counts exist for two partitions only");
  extern __shared__ unsigned short list[];  // [tokC] token offsets from the workgroup's first token
  __shared__ std::conditional_t<PAIRS, PairLds, int> pl;
  __shared__ int scan_sm[2 * NW + 1 + 4];
  __shared__ int wcnt[2 * NW];
  __shared__ float red[ATTN ? NW * G * (kD + 2) : 1];
  __shared__ float qlds[ATTN ? G * kD : 1];
  __shared__ __attribute__((aligned(16))) unsigned char vtile[kMfma ? NW * kVTileBytes : 16];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = u / s.Hkv, g = u % s.Hkv;
  PQC_MARK(ws, 1, 0);
  // this wave's stored bins, the query and the histogram: all requested up front
  const int tpw = s.tokC / NW;           // tokens per wave, in groups of 8 per lane
  const int gpw = (tpw + 511) / 512;     // groups per lane: 1, 2 or 4 (the last lanes idle when tpw < 512)
  const int wave_t0 = blockIdx.x * s.tokC + w * tpw;
  // 16 bytes per group of 8 tokens: their stored bins, or (PAIRS) their codes
  const unsigned short* bins_u =
      PAIRS ? reinterpret_cast<const unsigned short*>(static_cast<const uint8_t*>(src_ptr) + (size_t)u * s.cap * 2)
            : ws.bins + (size_t)u * s.binStride;
  const int last_group = PAIRS ? s.cap - 8 : s.binStride - 8;  // PAIRS: the capacity is a multiple of 8
  uint4 raw[kMaxVecC];
#pragma unroll
  for (int v = 0; v < kMaxVecC; ++v)
    raw[v] = *reinterpret_cast<const uint4*>(bins_u + min(wave_t0 + min((v * 64 + lane) * 8, tpw - 8), last_group));
  constexpr int QV = ATTN ? (G * kD + NT - 1) / NT : 1;  // query elements per thread
  float qreg[QV];
  if constexpr (ATTN) {
#pragma unroll
    for (int x = 0; x < QV; ++x)
      qreg[x] = load_as_float<T>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, min(x * NT + tid, G * kD - 1));
  }
  Threshold th{0, 0, 0, 0};
  PairThreshold pth{0u, true};
  if constexpr (PAIRS) {
    PQC_LOADS_ISSUED();
    if constexpr (ATTN) {
#pragma unroll
      for (int x = 0; x < QV; ++x)
        if (x * NT + tid < G * kD) qlds[x * NT + tid] = qreg[x];
    }
    pth = pair_threshold<T, NT>(s, q + ((size_t)b * s.Hq + (size_t)g * G) * kD, cent + (size_t)u * 2 * s.C * (kD / 2),
                                pair_counts + (size_t)u * s.C * s.C, static_cast<const uint8_t*>(src_ptr) + (size_t)u * s.cap * 2,
                                pl, scan_sm, [&](int slot) { PQC_MARK(ws, 1, slot); }, uncounted);  // syncs: qlds ready
  } else {
    ThresholdSearch<NT> ts;
    ts.load(ws.hist + (size_t)u * s.histCopies * kNB, s.histCopies);
    PQC_LOADS_ISSUED();
    if constexpr (ATTN) {
#pragma unroll
      for (int x = 0; x < QV; ++x)
        if (x * NT + tid < G * kD) qlds[x * NT + tid] = qreg[x];
    }
    th = ts.resolve(s.K, scan_sm);  // syncs: qlds ready
  }
  PQC_MARK(ws, 1, 1);

  const int segN = s.tokC / NW;
  unsigned short* seg = list + w * segN;
  const int wg_t0 = blockIdx.x * s.tokC;
  int nsel = 0, ncand = 0;
  const unsigned thr = (unsigned)th.bstar + 1u;  // in stored form
#pragma unroll
  for (int v = 0; v < kMaxVecC; ++v) {
    if (v < gpw) {  // uniform
      const int t0 = wave_t0 + (v * 64 + lane) * 8;
      const unsigned wv[4] = {raw[v].x, raw[v].y, raw[v].z, raw[v].w};
      unsigned selm = 0u, candm = 0u;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const unsigned st = (wv[i >> 1] >> (16 * (i & 1))) & 0xffffu;
        if constexpr (PAIRS) {
          const int t = t0 + i;
          const bool window = t < s.I || t >= s.N - s.L;
          const unsigned key =
              score_key(__fadd_rn(pl.lut[min(st & 0xffu, (unsigned)kPairC - 1)], pl.lut[kPairC + min(st >> 8, (unsigned)kPairC - 1)]));
          selm |= ((window || (!pth.none && key > pth.key)) ? 1u : 0u) << i;
          candm |= ((!window && !pth.none && key == pth.key) ? 1u : 0u) << i;
        } else {
          selm |= (st > thr ? 1u : 0u) << i;
          candm |= (st == thr ? 1u : 0u) << i;
        }
      }
      const int nreal = (v * 64 + lane) * 8 < tpw ? min(8, max(0, s.N - t0)) : 0;  // tokens of this group that exist
      selm &= (1u << nreal) - 1u;
      candm &= (1u << nreal) - 1u;
      const int cnt = __popc(selm) | (__popc(candm) << 16);
      const int inc = wave_inclusive_scan(cnt);
      const int tot = wave_last(inc);
      int ps = nsel + ((inc - cnt) & 0xffff), pc = ncand + ((inc - cnt) >> 16);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (selm & (1u << i)) seg[ps++] = (unsigned short)(t0 + i - wg_t0);
        if (candm & (1u << i)) seg[segN - 1 - (pc++)] = (unsigned short)(t0 + i - wg_t0);
      }
      nsel += tot & 0xffff;
      ncand += tot >> 16;
    }
  }
  PQC_MARK(ws, 1, 8);
  if (lane == 0) {
    wcnt[w] = nsel;
    wcnt[NW + w] = ncand;
  }
  __syncthreads();
  PQC_MARK(ws, 1, 2);
  int csel[NW + 1], ccand[NW + 1];
  csel[0] = 0;
  ccand[0] = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    csel[i + 1] = csel[i] + wcnt[i];
    ccand[i + 1] = ccand[i] + wcnt[NW + i];
  }
  const int tot_sel = csel[NW], tot_cand = ccand[NW];
  // record slots for this workgroup's candidates: requested now, needed only after the
  // attention below, which hides the round trip of the returning atomic
  int rec_base;  // set and read by thread 0 only; no initialiser, or the merge with it would wait for the atomic here
  if (tid == 0 && tot_cand > 0) rec_base = (int)atomicAdd(&ws.cand_count[u], (unsigned)tot_cand);
  // A candidate's exact score comes from its codes and the unit's table (same evaluation order
  // as everywhere), or from the score array of the stand-alone top-k.
  struct CandKey {
    unsigned cb[SRC::kFromCodes ? SRC::M : 1];
    float sc;
  };
  auto cand_token = [&](int c) -> int {
    int i = 0;
#pragma unroll
    for (int x = 1; x < NW; ++x) i += (c >= ccand[x]) ? 1 : 0;
    return wg_t0 + list[i * segN + segN - 1 - (c - ccand[i])];
  };
  auto cand_key_load = [&](int t) -> CandKey {
    CandKey k;
    k.sc = 0.0f;
    if constexpr (SRC::kFromCodes) {
      const uint8_t* cp = static_cast<const uint8_t*>(src_ptr) + ((size_t)u * s.cap + t) * SRC::M;
#pragma unroll
      for (int j = 0; j < SRC::M; ++j) k.cb[j] = cp[j];
    } else {
      k.cb[0] = 0u;
      k.sc = static_cast<const float*>(src_ptr)[(size_t)u * s.N + t];
    }
    return k;
  };
  auto cand_score = [&](const CandKey& k) -> float {
    if constexpr (PAIRS) {
      return __fadd_rn(pl.lut[min(k.cb[0], (unsigned)kPairC - 1)], pl.lut[kPairC + min(k.cb[1], (unsigned)kPairC - 1)]);
    } else if constexpr (SRC::kFromCodes) {
      const float* tb = ws.lut + (size_t)u * SRC::M * s.C;
      float sc = tb[k.cb[0]];
#pragma unroll
      for (int j = 1; j < SRC::M; ++j) sc = __fadd_rn(sc, tb[j * s.C + k.cb[j]]);
      return sc;
    } else {
      return k.sc;
    }
  };
  auto sel_at = [&](int p) -> int {
    int i = 0;
#pragma unroll
    for (int x = 1; x < NW; ++x) i += (p >= csel[x]) ? 1 : 0;
    return wg_t0 + list[i * segN + (p - csel[i])];
  };

  // selected list for the finalize kernel's index output
  unsigned long long* stage = ws.stage + ((size_t)u * s.nblkC + blockIdx.x) * s.stageStride;
  int* stage32 = reinterpret_cast<int*>(stage);
  PQC_MARK(ws, 1, 3);

  const T* kbase = kc + (size_t)u * s.cap * kD;
  const T* vbase = vc + (size_t)u * s.cap * kD;
  // The first candidates (one per 16-lane group): their codes and K/V rows are requested now, so that
  // after the attention only the table look-up, arithmetic and the record write remain.
  const int sub = lane & 15, grp = tid >> 4;
  int c0_t = 0;
  CandKey c0_key;
  RowRaw<T> c0_k, c0_v;
  c0_key.sc = 0.0f;
#pragma unroll
  for (int j = 0; j < (SRC::kFromCodes ? SRC::M : 1); ++j) c0_key.cb[j] = 0u;
  c0_k.zero();
  c0_v.zero();
  if (grp < tot_cand) {
    c0_t = cand_token(grp);
    c0_key = cand_key_load(c0_t);
    if constexpr (ATTN) {
      c0_k.load(kbase, c0_t, sub);
      c0_v.load(vbase, c0_t, sub);
    }
  }
  // Rows this workgroup attends: its own tokens above the threshold bin, and, instead of the
  // window tokens it happens to hold (the list's first nI and last nL entries), every
  // nblkC-th token of the two windows, so that the window rows are spread over the unit's
  // workgroups.
  const int tok_lo = (int)blockIdx.x * s.tokC, tok_hi = min(s.N, ((int)blockIdx.x + 1) * s.tokC);
  const int nI = max(0, min(s.I, tok_hi) - tok_lo), nL = max(0, tok_hi - max(s.N - s.L, tok_lo));
  const int n_own = tot_sel - nI - nL;
  const int n_win = (int)blockIdx.x < s.I + s.L ? (s.I + s.L - (int)blockIdx.x + s.nblkC - 1) / s.nblkC : 0;
  const int n_att = n_own + n_win;
  auto att_at = [&](int p) -> int {
    if (p < n_own) return sel_at(p + nI);
    const int wt = (int)blockIdx.x + (p - n_own) * s.nblkC;
    return wt < s.I ? wt : s.N - s.L + (wt - s.I);
  };
  if constexpr (ATTN) {
    if constexpr (kMfma) {
      bf16x8_t qf[4];
      load_q_frags(reinterpret_cast<const bf16_t*>(q) + ((size_t)b * s.Hq + (size_t)g * G) * kD, G, qf);
      MfmaState st;
      st.init();
      mfma_attend(reinterpret_cast<const bf16_t*>(kbase), reinterpret_cast<const bf16_t*>(vbase), s.N, att_at, n_att,
                  w * 16 * kMfmaTiles, NW * 16 * kMfmaTiles, s.scale_log2e, qf, vtile + w * kVTileBytes, st);
      PQC_MARK(ws, 1, 4);
      mfma_stash_wave_state<G>(st, red);
    } else {
      float qr[G][8];
      load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
      AttnState<G> st;
      st.init();
      constexpr int R = (G >= 8 || sizeof(T) == 4) ? 2 : 4;
      attend_rows<T, G, R>(kbase, vbase, s.N, att_at, n_att, w * 4 * R, NW * 4 * R, qr, st);
      PQC_MARK(ws, 1, 4);
      stash_wave_state<T, G>(st, red);
    }
    __syncthreads();
    // this workgroup's partial state: the accumulators as 128 floats per head ([j][h][kD] over the unit's workgroups j),
    // the (m, l) pairs in a dense array per head behind all accumulators ([units][h][j]); see finalize_kernel
    float* pacc = ws.partials + (((size_t)u * s.npart + blockIdx.x) * G) * kD;
    float2* pml = reinterpret_cast<float2*>(ws.partials + (size_t)s.B * s.Hkv * s.npart * G * kD) + (size_t)u * G * s.npart + blockIdx.x;
    for (int o = tid; o < G * kD; o += NT) {
      const int h = o / kD, d = o % kD;
      float m, l, acc;
      combine_waves<G, NW>(red, h, d, m, l, acc);
      pacc[h * kD + d] = acc;
      if (d == 0) pml[(size_t)h * s.npart] = make_float2(m, l);
    }
  }
  // (written after the attention: stores issued while the K/V loads of the co-resident workgroup
  // fill the memory pipeline would only delay this workgroup's own first loads)
  for (int p = tid; p < tot_sel; p += NT) stage32[p] = sel_at(p);
  if (tid == 0) ws.stage_cnt[(size_t)u * s.nblkC + blockIdx.x] = make_int2(tot_sel, tot_cand);
  PQC_MARK(ws, 1, 5);
  PQC_NOTE(ws, 1, 14, tot_sel);
  PQC_NOTE(ws, 1, 15, tot_cand);

  // candidates (few): composite for the generic path, and a full record while slots last
  if (tot_cand > 0) {  // workgroup-uniform
    if (tid == 0) scan_sm[0] = rec_base;
    __syncthreads();
    const int base = scan_sm[0];
    for (int c = grp; c < tot_cand; c += NT / 16) {
      int t = c0_t;
      CandKey key = c0_key;
      RowRaw<T> kr = c0_k, vr = c0_v;
      if (c >= NT / 16) {  // beyond the candidates whose loads went out before the attention
        t = cand_token(c);
        key = cand_key_load(t);
        if constexpr (ATTN) {
          kr.load(kbase, t, sub);
          vr.load(vbase, t, sub);
        }
      }
      const unsigned long long comp = make_composite(cand_score(key), t);
      if (sub == 0) stage[s.tokC - 1 - c] = comp;
      if (base + c < kCandRec) {
        const CandView cv = cand_view(ws.cand_rec + (size_t)u * ws.rec_stride, ATTN ? G : 1);
        if (sub == 0) cv.composite[base + c] = comp;
        if constexpr (ATTN) {
          float kf[8];
          kr.unpack(kf);
#pragma unroll
          for (int h = 0; h < G; ++h) {
            float d = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(qlds[h * kD + owned_dim<T>(sub, e)], kf[e], d);
            d = group16_sum(d);
            if (sub == 0) cv.logit[h * kCandRec + base + c] = d;
          }
          vr.store(cv.v + (size_t)(base + c) * kD * sizeof(T), sub);
        }
      }
    }
  }
}

// ------------------------------------------------------------- 3. finalize
// Grid (heads * SL + kCopyWgs, units), 256 threads; heads = the group's query heads, SL = Shape::slices (one
// head, one slice for the stand-alone top-k).
//   blockIdx.x <  heads * SL  slice blockIdx.x % SL of head blockIdx.x / SL: ranks the candidates and
//                        folds the admitted ones and all partial softmax states into kD / SL dimensions
//                        of this head's output; workgroup 0 also writes the admitted candidates'
//                        indices (best first)
//   blockIdx.x >= heads * SL  copy workgroups: concatenate the staged lists into out_idx; the
//                        first one also zeroes the unit's histogram and record counter
// The staged "selected" lists already hold the two windows: in workgroup order they read
//   [0..I) , tokens above the threshold bin (ascending) , [N-L..N).
// Fast path (at most kCandRec candidates): all a head needs is in the candidate records,
// which sit densely in order of arrival.  That order differs from run to run, so every
// sum over candidates is taken in rank order.  Generic path: candidates are the
// composites staged per select workgroup; admitted rows are gathered from the K/V cache.
template <int NT>
__device__ __forceinline__ float block_max(float v, float* sm /* [NT/64] */) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sm[0];
#pragma unroll
  for (int i = 1; i < NT / 64; ++i) r = fmaxf(r, sm[i]);
  __syncthreads();
  return r;
}
template <int NT>
__device__ __forceinline__ float block_sum(float v, float* sm /* [NT/64] */) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sm[0];
#pragma unroll
  for (int i = 1; i < NT / 64; ++i) r += sm[i];
  __syncthreads();
  return r;
}

constexpr int kHdrPerThread = kCandRec / 256;  // candidate record headers per thread
constexpr int kAccPer = 8;                     // partial states a thread keeps in flight at once (every eighth state is its own)
constexpr int kVPer = 12;                      // candidate records per thread whose V values are requested before the ranking knows which are admitted (96 records
                                               // with eight threads per dimension: tie classes of two-partition tables reach 70 tokens at 128K)
constexpr int kVPerFew = 8;                    // the same with fewer threads per dimension (many units; there the tie classes are small)
constexpr int kManyCand = 4096;                // candidates whose composites the path for large tie classes keeps in LDS
constexpr int kRankStep = 8;                    // composites read per step of the ranking loop
constexpr int kFoldRanks = 96;                 // admitted rows whose terms meet in LDS by rank (beyond: fetched by rank from the records)
constexpr int kMaxSlices = 4;                  // workgroups per query head, at most (32 output dimensions each)
constexpr int kIdxLists = 4;                   // staged index lists a wave copies with loads issued up front
constexpr int kCopyWgs = 4;                    // copy workgroups per unit

// dynamic LDS of finalize_kernel
inline size_t finalize_lds_bytes(const Shape& s, bool attn) {
  const size_t terms = attn ? (size_t)kFoldRanks * (kD / s.slices) * sizeof(float) : 0;
  const size_t many = (size_t)kManyCand * (sizeof(unsigned long long) + sizeof(int));  // the same region, when a unit has more than kCandRec candidates
  return (size_t)(4 * s.nblkC + 2) * sizeof(int) + (terms > many ? terms : many);
}

// The code of one appended token per unit (Section 3.1: nearest centroid of each partition): nothing in the
// step depends on it, so one more workgroup per unit of the finalize kernel computes it beside the others.
struct AppendArgs {
  const void* key;    // [units][kD] in the cache's element type, or null: nothing to append
  const float* cent;  // [units][M][C][Dm]
  uint8_t* codes;     // the code tensor; written at `position` of every unit
  int position;
  unsigned* pair_counts;  // two partitions: [units][C*C] counts that gain the token's code pair, or null
};

// WIDE: four workgroups per head (eight threads per output dimension); they request more candidate records up front.
template <typename T, int G, bool ATTN, bool WIDE = false>
__global__ __launch_bounds__(256) void finalize_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                       const T* __restrict__ kc, const T* __restrict__ vc,
                                                       int* __restrict__ out_idx, float* __restrict__ out_attn, AppendArgs ap) {
  constexpr int NT = 256, NW = 4;
  constexpr int heads = ATTN ? G : 1;
  constexpr int VPER = WIDE ? kVPer : kVPerFew;
  const int SL = ATTN ? s.slices : 1;  // head workgroups per head
  if ((int)blockIdx.x == heads * SL + kCopyWgs) {
    // -------------------------------------------------------------- append workgroup
    // one thread per centroid, the distance chain of pq_assign_kernel, the smallest (distance, centroid) pair
    // of each partition through a 64-bit LDS minimum
    __shared__ float ax[kD];
    __shared__ unsigned long long abest[8];
    const int u = blockIdx.y, c = threadIdx.x;
    if (c < kD) ax[c] = load_as_float<T>(static_cast<const T*>(ap.key), (size_t)u * kD + c);
    if (c < 8) abest[c] = ~0ull;
    __syncthreads();
    if (c < s.C) {
      for (int j = 0; j < s.M; ++j) {
        const float* cr = ap.cent + (((size_t)u * s.M + j) * s.C + c) * s.Dm;
        const float* xj = ax + j * s.Dm;
        float d2 = 0.0f;
        for (int e = 0; e < s.Dm; e += 4) {  // Dm is a multiple of 4
          const float4 cv = *reinterpret_cast<const float4*>(cr + e);
          float df = xj[e] - cv.x;
          d2 = fmaf(df, df, d2);
          df = xj[e + 1] - cv.y;
          d2 = fmaf(df, df, d2);
          df = xj[e + 2] - cv.z;
          d2 = fmaf(df, df, d2);
          df = xj[e + 3] - cv.w;
          d2 = fmaf(df, df, d2);
        }
        atomicMin(&abest[j], ((unsigned long long)__float_as_uint(d2) << 32) | (unsigned)c);  // d2 >= 0: bits order like values
      }
    }
    __syncthreads();
    if (c < s.M) ap.codes[((size_t)u * s.cap + ap.position) * s.M + c] = (uint8_t)(abest[c] & 0xffu);
    if (c == 0 && ap.pair_counts) ap.pair_counts[(size_t)u * s.C * s.C + (abest[0] & 0xffu) + s.C * (abest[1] & 0xffu)] += 1u;
    return;
  }
  extern __shared__ int dyn[];  // pre_sel[nblkC+1], pre_cand[nblkC+1], pm[nblkC], pl[nblkC], then terms[kFoldRanks][kD/slices] or, with
                                // more than kCandRec candidates, their composites and the admitted tokens (finalize_lds_bytes)
  __shared__ int scan_sm[2 * NW + 1];
  __shared__ float fsm[NW];
  __shared__ int ism[2 * NW];
  __shared__ unsigned long long comp[kCandRec + kRankStep];  // candidate composites, in record order
  __shared__ float lgk[kCandRec];                // by rank: logit, then softmax weight of the admitted ones
  __shared__ unsigned short ordv[kCandRec];      // by rank: record
  __shared__ unsigned short rankv[kCandRec];     // by record: rank
  __shared__ unsigned mkey;                      // order-preserving key of the largest logit (states and admitted rows)
  __shared__ unsigned rhist[256];
  __shared__ int digit_sm[2];
  __shared__ int rows_sm[NT];
  __shared__ float red[ATTN ? NW * (kD + 2) : 1];
  __shared__ float half_acc[ATTN ? kD : 1];
  __shared__ float slice_sm[ATTN ? 256 : 1];  // [threads per dimension][dimensions of the workgroup]
  __shared__ float lsm[8];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = u / s.Hkv, g = u % s.Hkv;
  int* pre_sel = dyn;
  int* pre_cand = dyn + (s.nblkC + 1);
  float* pm = reinterpret_cast<float*>(dyn + 2 * (s.nblkC + 1));
  float* pl = pm + s.nblkC;
  float* terms = pl + s.nblkC;  // [kFoldRanks][dimensions of the workgroup]: weighted V values of the admitted rows, by rank
  const int2* cnt = ws.stage_cnt + (size_t)u * s.nblkC;
  const unsigned long long* stage_u = ws.stage + (size_t)u * s.nblkC * s.stageStride;
  int* out = out_idx + (size_t)u * s.Ktot;
  PQC_MARK(ws, 2, 0);

  // exclusive prefix sums of the per-workgroup list sizes (into LDS); returns the totals
  auto scan_counts = [&](const int2 cnt0, int& n_list, int& n_cand) {
    int carry_s = 0, carry_c = 0;
    for (int j0 = 0; j0 < s.nblkC; j0 += NT) {
      const int j = j0 + tid;
      const int2 c = j < s.nblkC ? (j0 == 0 ? cnt0 : cnt[j]) : make_int2(0, 0);
      int ts, tc;
      const int ps = block_exclusive_scan<NT>(c.x, &ts, scan_sm);
      const int pc = block_exclusive_scan<NT>(c.y, &tc, scan_sm);
      if (j < s.nblkC) {
        pre_sel[j] = carry_s + ps;
        pre_cand[j] = carry_c + pc;
      }
      carry_s += ts;
      carry_c += tc;
    }
    if (tid == 0) {
      pre_sel[s.nblkC] = carry_s;
      pre_cand[s.nblkC] = carry_c;
    }
    __syncthreads();
    n_list = carry_s;
    n_cand = carry_c;
  };

  if ((int)blockIdx.x >= heads * SL) {
    // ---------------------------------------------------------------- copy workgroup
    // one wave per list, coalesced; the local window moves behind the admitted candidates
    const int cw = blockIdx.x - heads * SL, ncw = kCopyWgs;
    const int2 cnt0 = cnt[min(tid, s.nblkC - 1)];
    int ix[kIdxLists][4];  // first 256 entries of this wave's first kIdxLists lists
#pragma unroll
    for (int x = 0; x < kIdxLists; ++x) {
      const int j = min(cw * NW + w + x * ncw * NW, s.nblkC - 1);
      const int* src = reinterpret_cast<const int*>(stage_u + (size_t)j * s.stageStride);
#pragma unroll
      for (int y = 0; y < 4; ++y) ix[x][y] = src[min(y * 64 + lane, 2 * s.tokC - 1)];
    }
    PQC_LOADS_ISSUED();
    int n_list, n_cand;
    scan_counts(cnt0, n_list, n_cand);
    const int n_above = max(0, n_list - s.I - s.L);
    const int need = max(0, min(s.K - n_above, n_cand));
    PQC_MARK(ws, 2, 1);
    int x = 0;
    for (int j = cw * NW + w; j < s.nblkC; j += ncw * NW, ++x) {
      const int base = pre_sel[j], n = pre_sel[j + 1] - base;
      const int* src = reinterpret_cast<const int*>(stage_u + (size_t)j * s.stageStride);
      for (int p0 = 0; p0 < n; p0 += 256) {
        int v[4];
        if (x < kIdxLists && p0 == 0) {
#pragma unroll
          for (int y = 0; y < 4; ++y) v[y] = x == 0 ? ix[0][y] : x == 1 ? ix[1][y] : x == 2 ? ix[2][y] : ix[3][y];
        } else {
#pragma unroll
          for (int y = 0; y < 4; ++y)
            if (p0 + y * 64 + lane < n) v[y] = src[p0 + y * 64 + lane];
        }
#pragma unroll
        for (int y = 0; y < 4; ++y) {
          const int pos = base + p0 + y * 64 + lane;
          // (the bound only matters when the caller's pair counts do not belong to the codes: then n_above can exceed K)
          const int dst = pos < s.I + n_above ? pos : pos + need;
          if (p0 + y * 64 + lane < n && dst < s.Ktot) out[dst] = v[y];
        }
      }
    }
    PQC_MARK(ws, 2, 4);
    if (cw == 0) {  // the select kernel was their last reader: zero histogram and record counter for the next call
      unsigned* gh = ws.hist + (size_t)u * s.histCopies * kNB;
      for (int i = tid; i < s.histCopies * kNB; i += NT) gh[i] = 0u;
      if (tid == 0) ws.cand_count[u] = 0u;
    }
    PQC_MARK(ws, 2, 5);
    return;
  }

  // ------------------------------------------------------------------ head workgroup
  // One of SL workgroups of query head hq: it produces output dimensions [dims*sl, dims*sl + dims), dims = kD / SL.
  // A compute unit reads what other compute units wrote at a small fraction of the chip's bandwidth (about a hundred
  // cache lines per microsecond), so with few units the partial states of a head are spread over several workgroups,
  // each reading only its dimensions of every state, and everything a workgroup reads of the candidates is dense.
  const int hq = (int)blockIdx.x / SL, sl = (int)blockIdx.x % SL;
  const int dims = kD / SL, nps = NT / dims;   // output dimensions of this workgroup; threads per dimension (2, 4 or 8)
  const int dl = tid & (dims - 1), ps = tid / dims;  // dimension inside the slice; which share of the states and admitted rows
  const int d = dims * sl + dl;
  const int units = s.B * s.Hkv;
  // ---- everything whose address is known up front is requested first
  const CandView cv = cand_view(ws.cand_rec + (size_t)u * ws.rec_stride, heads);
  unsigned long long rc[kHdrPerThread];  // candidate x*NT + tid; the first NT are requested up front
  float rl[kHdrPerThread];
  rc[0] = cv.composite[tid];
  rl[0] = ATTN ? cv.logit[hq * kCandRec + tid] : 0.0f;
  const float* pacc = ws.partials + (size_t)u * s.npart * G * kD;                                   // [j][h][kD]
  const float2* pml = reinterpret_cast<const float2*>(ws.partials + (size_t)units * s.npart * G * kD) +
                      ((size_t)u * G + hq) * s.npart;                                                // [j] of this head
  const int jc = min(tid, s.nblkC - 1);
  const int2 cnt0 = cnt[jc];  // list sizes of the first NT select workgroups
  float2 ml0 = make_float2(kNegBig, 0.0f);
  float a0[kAccPer];  // this thread's first states: ps, ps + nps, ...
  float vv0[VPER];    // V values of the candidate records ps, ps + nps, ... (this thread's dimension)
  if constexpr (ATTN) {
    ml0 = pml[jc];
#pragma unroll
    for (int x = 0; x < kAccPer; ++x)  // states that do not exist re-read the first one (a cache hit, no extra traffic)
      a0[x] = pacc[((size_t)(ps + nps * x < s.nblkC ? ps + nps * x : 0) * G + hq) * kD + d];
    // the V values of the first candidates (in order of arrival), this workgroup's dimensions: which of them are
    // admitted is known only after the ranking, but requested now they are here by then
#pragma unroll
    for (int x = 0; x < VPER; ++x)
      vv0[x] = load_as_float<T>(reinterpret_cast<const T*>(cv.v) + (size_t)(ps + nps * x) * kD, d);
  }
  PQC_LOADS_ISSUED();
  float mpart = kNegBig;  // largest maximum of the partial states
  if constexpr (ATTN) {
    if (tid < s.nblkC) {
      pm[tid] = ml0.x;
      pl[tid] = ml0.y;
      mpart = ml0.x;
    }
    for (int j = NT + tid; j < s.nblkC; j += NT) {  // beyond the first NT lists (very long contexts)
      const float2 v = pml[j];
      pm[j] = v.x;
      pl[j] = v.y;
      mpart = fmaxf(mpart, v.x);
    }
  }
  // totals of the per-workgroup list sizes, and that maximum (one barrier)
  int n_list, n_cand;
  {
    int ss = tid < s.nblkC ? cnt0.x : 0, sc = tid < s.nblkC ? cnt0.y : 0;
    for (int j = NT + tid; j < s.nblkC; j += NT) {
      const int2 c = cnt[j];
      ss += c.x;
      sc += c.y;
    }
    ss = wave_last(wave_inclusive_scan(ss));
    sc = wave_last(wave_inclusive_scan(sc));
    mpart = wave_max(mpart);
    if (lane == 0) {
      ism[w] = ss;
      ism[NW + w] = sc;
      fsm[w] = mpart;
    }
    __syncthreads();  // also: pm, pl visible
    n_list = 0;
    n_cand = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      n_list += ism[i];
      n_cand += ism[NW + i];
      mpart = fmaxf(mpart, fsm[i]);
    }
  }
  const int n_above = max(0, n_list - s.I - s.L);  // n_list = I + (tokens above the bin) + L
  const int need = max(0, min(s.K - n_above, n_cand));
  PQC_MARK(ws, 2, 1);

  if (n_cand <= kCandRec) {
    // rank every candidate (count of larger composites); the admitted ones are the `need` best
    const bool meet = ATTN && need <= kFoldRanks;  // the admitted rows' terms meet in LDS, by rank
    if (need > 0) {
#pragma unroll
      for (int x = 1; x < kHdrPerThread; ++x) {
        rc[x] = 0ull;
        rl[x] = 0.0f;
        if (x * NT + tid < n_cand) {  // rare: more than NT candidates
          rc[x] = cv.composite[x * NT + tid];
          rl[x] = ATTN ? cv.logit[hq * kCandRec + x * NT + tid] : 0.0f;
        }
      }
      // (entries up to the next multiple of kRankStep are zero, which ranks behind everything: the loop below reads
      // kRankStep composites at a time, because one LDS read per step is a chain of latencies)
#pragma unroll
      for (int x = 0; x < kHdrPerThread; ++x)
        if (x * NT + tid < n_cand + kRankStep) comp[x * NT + tid] = x * NT + tid < n_cand ? rc[x] : 0ull;
      if (tid == 0) mkey = score_key(mpart);
      __syncthreads();
#pragma unroll
      for (int x = 0; x < kHdrPerThread; ++x) {
        const int k = x * NT + tid;
        if (k < n_cand) {
          const unsigned long long mine = rc[x];
          int rank = 0;
          for (int j0 = 0; j0 < n_cand; j0 += kRankStep) {
            unsigned long long c[kRankStep];
#pragma unroll
            for (int y = 0; y < kRankStep; ++y) c[y] = comp[j0 + y];
#pragma unroll
            for (int y = 0; y < kRankStep; ++y) rank += c[y] > mine ? 1 : 0;
          }
          rankv[k] = (unsigned short)rank;
          if (rank < need) {
            if (blockIdx.x == 0 && s.I + n_above + rank < s.Ktot) out[s.I + n_above + rank] = composite_token(mine);  // best first
            const float lg = rl[x] * s.scale_log2e;
            lgk[rank] = lg;
            ordv[rank] = (unsigned short)k;
            if constexpr (ATTN) atomicMax(&mkey, score_key(lg));
          }
        }
      }
      __syncthreads();
    }
    if constexpr (ATTN) {
      // out[d] = (sum_j w_j acc_j[d] + sum_r p_r V_r[d]) / l with w_j = exp2(m_j - m*), p_r = exp2(logit_r - m*):
      // nps threads per dimension, thread ps taking the states j = ps (mod nps) and the admitted rows r = ps (mod nps),
      // each in ascending order; the nps sums are added in order.  m* is the larger of the states' maximum (it came
      // with the totals above) and the admitted logits' maximum (an LDS maximum taken while ranking); the threads of
      // dimension 0 sum l alongside.
      const float mstar = need > 0 ? key_score(mkey) : mpart;
      if (meet && need > 0) {
        // the V values requested up front belong to the records ps + nps x in order of arrival; each admitted one's
        // term goes to the row of its rank, so that the sums below run in rank order whatever the order of arrival
        for (int k0 = 0; k0 < n_cand; k0 += nps * VPER) {
          if (k0 > 0) {  // rare: more candidates than the up-front loads cover
#pragma unroll
            for (int x = 0; x < VPER; ++x)
              vv0[x] = load_as_float<T>(reinterpret_cast<const T*>(cv.v) + (size_t)min(k0 + ps + nps * x, kCandRec - 1) * kD, d);
          }
#pragma unroll
          for (int x = 0; x < VPER; ++x) {
            const int k = k0 + ps + nps * x;
            if (k < n_cand) {
              const int r = rankv[k];
              if (r < need) terms[r * dims + dl] = __builtin_amdgcn_exp2f(lgk[r] - mstar) * vv0[x];
            }
          }
        }
      }
      float acc = 0.0f, lsum = 0.0f;
#pragma unroll
      for (int x = 0; x < kAccPer; ++x) {
        const int j = ps + nps * x;
        if (j < s.nblkC) {
          const float wj = __builtin_amdgcn_exp2f(pm[j] - mstar);
          acc = fmaf(wj, a0[x], acc);
          lsum = fmaf(wj, pl[j], lsum);
        }
      }
      for (int j0 = nps * kAccPer + ps; j0 < s.nblkC; j0 += nps * kAccPer) {
        float a[kAccPer];
#pragma unroll
        for (int x = 0; x < kAccPer; ++x) a[x] = pacc[((size_t)min(j0 + nps * x, s.nblkC - 1) * G + hq) * kD + d];
#pragma unroll
        for (int x = 0; x < kAccPer; ++x) {
          const int j = j0 + nps * x;
          if (j < s.nblkC) {
            const float wj = __builtin_amdgcn_exp2f(pm[j] - mstar);
            acc = fmaf(wj, a[x], acc);
            lsum = fmaf(wj, pl[j], lsum);
          }
        }
      }
      if (meet) {
        if (need > 0) __syncthreads();  // (need is uniform over the workgroup)
        for (int r0 = ps; r0 < need; r0 += nps * 4) {
          float t[4], lg[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const int r = min(r0 + nps * x, need - 1);
            t[x] = terms[r * dims + dl];
            lg[x] = lgk[r];
          }
#pragma unroll
          for (int x = 0; x < 4; ++x)
            if (r0 + nps * x < need) {
              acc += t[x];
              lsum += __builtin_amdgcn_exp2f(lg[x] - mstar);
            }
        }
      } else {
        // more admitted rows than the LDS rows hold (a large tie class at the threshold): fetched by rank
        for (int r0 = ps; r0 < need; r0 += nps * kAccPer) {
          float vv[kAccPer];
#pragma unroll
          for (int x = 0; x < kAccPer; ++x)
            vv[x] = load_as_float<T>(reinterpret_cast<const T*>(cv.v) + (size_t)ordv[min(r0 + nps * x, need - 1)] * kD, d);
#pragma unroll
          for (int x = 0; x < kAccPer; ++x) {
            const int r = r0 + nps * x;
            if (r < need) {
              acc += __builtin_amdgcn_exp2f(lgk[r] - mstar) * vv[x];
              lsum += __builtin_amdgcn_exp2f(lgk[r] - mstar);
            }
          }
        }
      }
      slice_sm[ps * dims + dl] = acc;
      if (dl == 0) lsm[ps] = lsum;
      __syncthreads();
      PQC_MARK(ws, 2, 2);
      if (tid < dims) {
        float ts[8], ls[8];  // nps <= 8
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          ts[x] = slice_sm[min(x, nps - 1) * dims + tid];
          ls[x] = lsm[min(x, nps - 1)];
        }
        float tot = ts[0], lstar = ls[0];
#pragma unroll
        for (int x = 1; x < 8; ++x)
          if (x < nps) {
            tot += ts[x];
            lstar += ls[x];
          }
        out_attn[((size_t)b * s.Hq + (size_t)g * G + hq) * kD + dims * sl + tid] = tot / lstar;
      }
      PQC_MARK(ws, 2, 3);
    }
  } else if (sl == 0) {
    // generic path (one workgroup per head does all 128 dimensions): radix select of the need-th largest staged
    // composite, 8 bits per pass
    const int d128 = tid & (kD - 1), half = tid >> 7;
    {
      int nl, nc;
      scan_counts(cnt0, nl, nc);
    }
    auto owner = [&](int p) -> int {  // largest j with pre_cand[j] <= p
      int lo = 0, hi = s.nblkC - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (pre_cand[mid] <= p) lo = mid; else hi = mid - 1;
      }
      return lo;
    };
    auto cand_global = [&](int i) -> unsigned long long {
      const int j = owner(i);
      return stage_u[(size_t)j * s.stageStride + s.tokC - 1 - (i - pre_cand[j])];
    };
    // Up to kManyCand composites are fetched once into LDS (every pass over them would otherwise be a chain of
    // memory round trips); the bytes that all of them share (the whole score, when the candidates are one tie
    // class) need no radix pass.
    unsigned long long* gcomp = reinterpret_cast<unsigned long long*>(terms);  // [kManyCand]
    int* gtok = reinterpret_cast<int*>(gcomp + kManyCand);                     // [kManyCand] admitted tokens, in candidate order
    const bool cached = n_cand <= kManyCand;
    unsigned long long varying = ~0ull, common = 0ull;
    if (cached && need > 0) {
      unsigned long long a_and = ~0ull, a_or = 0ull;
      for (int i0 = 0; i0 < n_cand; i0 += 4 * NT) {
        unsigned long long c[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) c[x] = cand_global(min(i0 + x * NT + tid, n_cand - 1));
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const int i = i0 + x * NT + tid;
          if (i < n_cand) {
            gcomp[i] = c[x];
            a_and &= c[x];
            a_or |= c[x];
          }
        }
      }
      if (tid < 4) rhist[tid] = tid < 2 ? 0xffffffffu : 0u;
      __syncthreads();
      atomicAnd(&rhist[0], (unsigned)a_and);
      atomicAnd(&rhist[1], (unsigned)(a_and >> 32));
      atomicOr(&rhist[2], (unsigned)a_or);
      atomicOr(&rhist[3], (unsigned)(a_or >> 32));
      __syncthreads();
      common = ((unsigned long long)rhist[1] << 32) | rhist[0];
      varying = common ^ (((unsigned long long)rhist[3] << 32) | rhist[2]);
      __syncthreads();
    }
    auto cand_at = [&](int i) -> unsigned long long { return cached ? gcomp[i] : cand_global(i); };
    unsigned long long thr = ~0ull;
    if (need > 0) {
      unsigned long long prefix = 0;
      int want = need;
      for (int shift = 56; shift >= 0; shift -= 8) {
        if (((varying >> shift) & 0xffull) == 0) {  // uniform: every candidate has this byte
          prefix |= common & (0xffull << shift);
          continue;
        }
        rhist[tid] = 0u;
        __syncthreads();
        for (int i = tid; i < n_cand; i += NT) {
          const unsigned long long c = cand_at(i);
          if (shift == 56 || (c >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&rhist[(unsigned)(c >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
          int cum = 0, dg = 255;
          for (; dg > 0; --dg) {
            if (cum + (int)rhist[dg] >= want) break;
            cum += (int)rhist[dg];
          }
          digit_sm[0] = dg;
          digit_sm[1] = want - cum;
        }
        __syncthreads();
        prefix |= (unsigned long long)digit_sm[0] << shift;
        want = digit_sm[1];
        __syncthreads();
      }
      thr = prefix;
    }
    // admitted candidates in token order: indices out, rows attended (all at once when they fit the LDS list, else
    // NT candidates per round)
    AttnState<1> st;
    st.init();
    float qr[1][8];
    if constexpr (ATTN) load_query<T, 1>(q + ((size_t)b * s.Hq + (size_t)g * G + hq) * kD, s.scale_log2e, qr);
    int carry = 0;
    for (int i0 = 0; i0 < (need > 0 ? n_cand : 0); i0 += NT) {
      const int i = i0 + tid;
      unsigned long long c = 0;
      if (i < n_cand) c = cand_at(i);
      const int flag = (i < n_cand && c >= thr) ? 1 : 0;
      int tot;
      const int pos = block_exclusive_scan<NT>(flag, &tot, scan_sm);
      if (flag) {
        if (cached) gtok[carry + pos] = composite_token(c); else rows_sm[pos] = composite_token(c);
        if (hq == 0 && s.I + n_above + carry + pos < s.Ktot) out[s.I + n_above + carry + pos] = composite_token(c);
      }
      if (!cached) {
        __syncthreads();
        if constexpr (ATTN) {
          auto row_at = [&](int p) -> int { return rows_sm[p]; };
          attend_rows<T, 1, 4>(kc + (size_t)u * s.cap * kD, vc + (size_t)u * s.cap * kD, s.N, row_at, tot, w * 16, NW * 16, qr, st);
        }
        __syncthreads();
      }
      carry += tot;
    }
    if (cached) {
      __syncthreads();
      if constexpr (ATTN) {
        auto row_at = [&](int p) -> int { return gtok[p]; };
        attend_rows<T, 1, 4>(kc + (size_t)u * s.cap * kD, vc + (size_t)u * s.cap * kD, s.N, row_at, carry, w * 16, NW * 16, qr, st);
      }
    }
    if constexpr (ATTN) {
      stash_wave_state<T, 1>(st, red);
      __syncthreads();
      float m_own, l_own, acc;
      combine_waves<1, NW>(red, 0, d128, m_own, l_own, acc);
      float mx = m_own;
      for (int j = tid; j < s.nblkC; j += NT) mx = fmaxf(mx, pm[j]);
      const float mstar = block_max<NT>(mx, fsm);
      float lsum = 0.0f;
      for (int j = tid; j < s.nblkC; j += NT) {
        const float wj = __builtin_amdgcn_exp2f(pm[j] - mstar);
        pm[j] = wj;
        lsum = fmaf(wj, pl[j], lsum);
      }
      const float f_own = __builtin_amdgcn_exp2f(m_own - mstar);
      const float lstar = block_sum<NT>(lsum, fsm) + l_own * f_own;
      acc = half == 0 ? acc * f_own : 0.0f;
      for (int j = half; j < s.nblkC; j += 2) acc = fmaf(pm[j], pacc[((size_t)j * G + hq) * kD + d128], acc);
      if (half == 1) half_acc[d128] = acc;
      __syncthreads();
      if (half == 0) out_attn[((size_t)b * s.Hq + (size_t)g * G + hq) * kD + d128] = (acc + half_acc[d128]) / lstar;
    }
  }
  PQC_NOTE(ws, 2, 13, n_above);
  PQC_NOTE(ws, 2, 14, n_cand);
  PQC_NOTE(ws, 2, 15, need);
}

// ---------------------------------------------- stand-alone attention over a list
// pqc_gather_attn: workgroup x of unit u attends list positions [x*rowsP, +rowsP).
template <typename T, int G>
__global__ __launch_bounds__(256) void attn_list_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                        const T* __restrict__ kc, const T* __restrict__ vc,
                                                        const int* __restrict__ idx) {
  constexpr int NT = 256, NW = 4;
  constexpr bool kMfma = sizeof(T) == 2 && kMatrixCoreAttention;
  __shared__ float red[NW * G * (kD + 2)];
  __shared__ __attribute__((aligned(16))) unsigned char vtile[kMfma ? NW * kVTileBytes : 16];
  const int u = blockIdx.y, tid = threadIdx.x, w = tid >> 6;
  const int b = u / s.Hkv, g = u % s.Hkv;
  const int p0 = blockIdx.x * s.rowsP;
  const int count = min(s.rowsP, s.Ktot - p0);
  // this workgroup's slice of the list goes to LDS first: one coalesced load instead of a
  // dependent global load in front of every stage of row loads
  extern __shared__ int lst[];  // [rowsP]
  for (int p = tid; p < count; p += NT) lst[p] = idx[(size_t)u * s.Ktot + p0 + p];
  __syncthreads();
  auto row_at = [&](int p) -> int { return lst[p]; };
  const T* kbase = kc + (size_t)u * s.cap * kD;
  const T* vbase = vc + (size_t)u * s.cap * kD;
  if constexpr (kMfma) {
    bf16x8_t qf[4];
    load_q_frags(reinterpret_cast<const bf16_t*>(q) + ((size_t)b * s.Hq + (size_t)g * G) * kD, G, qf);
    MfmaState st;
    st.init();
    mfma_attend(reinterpret_cast<const bf16_t*>(kbase), reinterpret_cast<const bf16_t*>(vbase), s.N, row_at, count,
                w * 16 * kMfmaTiles, NW * 16 * kMfmaTiles, s.scale_log2e, qf, vtile + w * kVTileBytes, st);
    mfma_stash_wave_state<G>(st, red);
  } else {
    float qr[G][8];
    load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
    AttnState<G> st;
    st.init();
    constexpr int R = G >= 8 ? 2 : 4;
    attend_rows<T, G, R>(kbase, vbase, s.N, row_at, count, w * 4 * R, NW * 4 * R, qr, st);
    stash_wave_state<T, G>(st, red);
  }
  __syncthreads();
  float* part = ws.partials + ((size_t)u * s.npart + blockIdx.x) * G * (kD + 2);
  for (int o = tid; o < G * kD; o += NT) {
    const int h = o / kD, d = o % kD;
    float m, l, acc;
    combine_waves<G, NW>(red, h, d, m, l, acc);
    part[h * (kD + 2) + 2 + d] = acc;
    if (d == 0) {
      part[h * (kD + 2)] = m;
      part[h * (kD + 2) + 1] = l;
    }
  }
}

// Folds the partial softmax states of a unit into the outputs: grid (G, units), one
// workgroup per query head, two threads per output dimension.
template <int G>
__global__ __launch_bounds__(256) void merge_kernel(Shape s, Workspace ws, int nparts, float* __restrict__ out_attn) {
  constexpr int NT = 256, NW = 4, kBatch = 16;
  extern __shared__ float wsm[];  // [nparts] weights
  __shared__ float fsm[NW];
  __shared__ float half_acc[kD];
  const int u = blockIdx.y, hq = blockIdx.x, b = u / s.Hkv, g = u % s.Hkv, tid = threadIdx.x;
  const int d = tid & (kD - 1), half = tid >> 7;
  const float* parts = ws.partials + ((size_t)u * s.npart * G + hq) * (kD + 2);
  const size_t stride = (size_t)G * (kD + 2);
  float mx = kNegBig;
  for (int j = tid; j < nparts; j += NT) {
    const float m = parts[j * stride];
    wsm[j] = m;
    mx = fmaxf(mx, m);
  }
  const float mstar = block_max<NT>(mx, fsm);  // its barriers make wsm visible
  float lsum = 0.0f;
  for (int j = tid; j < nparts; j += NT) {
    const float wj = __builtin_amdgcn_exp2f(wsm[j] - mstar);
    wsm[j] = wj;
    lsum = fmaf(wj, parts[j * stride + 1], lsum);
  }
  const float lstar = block_sum<NT>(lsum, fsm);
  float acc = 0.0f;
  for (int j0 = half; j0 < nparts; j0 += 2 * kBatch) {
    float a[kBatch];
#pragma unroll
    for (int x = 0; x < kBatch; ++x) a[x] = parts[(size_t)min(j0 + 2 * x, nparts - 1) * stride + 2 + d];
#pragma unroll
    for (int x = 0; x < kBatch; ++x) acc = fmaf(j0 + 2 * x < nparts ? wsm[j0 + 2 * x] : 0.0f, a[x], acc);
  }
  if (half == 1) half_acc[d] = acc;
  __syncthreads();
  if (half == 0) out_attn[((size_t)b * s.Hq + (size_t)g * G + hq) * kD + d] = (acc + half_acc[d]) / lstar;
}

}  // namespace pqc
