// Kernels of libpqcache (gfx950).  Grid layout: blockIdx.y = unit (sequence b, KV
// head g); blockIdx.x = workgroup inside the unit.
//
// Decode path (pqc_decode), two launches; the one dependency between all workgroups of a
// unit that needs every one of them to be done sits at the kernel boundary, the other is
// settled by whichever workgroup finishes last (nobody ever waits inside a kernel):
//   hist_kernel      table -> scan codes -> histogram of scores over kNB bins, and every
//                    token's bin number left behind for the next kernel
//   select_kernel    threshold bin from the histogram -> tokens whose stored bin lies
//                    above it (and the two windows) are listed in ascending order
//                    without atomics and attended at once; tokens inside the bin
//                    ("candidates") are recorded with their logits and V row.  The unit's
//                    last workgroup to finish then ranks the candidates, folds the
//                    admitted ones and all partial softmax states into the output, writes
//                    the indices and zeroes the unit's histogram and counters again:
//                    every call leaves them as it found them
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
template <typename T, class SRC>
__global__ __launch_bounds__(1024) void hist_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                    const float* __restrict__ cent, const void* __restrict__ src_ptr) {
  constexpr int NT = 1024, P = SRC::P;
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
  typename SRC::Raw raw[kMaxVecA];
  typename SRC::One sample;
  const bool have_sample = tid < s.sampleN;
  auto issue_loads = [&]() {
#pragma unroll
    for (int v = 0; v < kMaxVecA; ++v) raw[v] = src.load(chunk0 + min(v * NT + tid, chunks - 1));
    const int sample_i = min(tid, s.sampleN - 1);
    sample = src.load_one(min(s.N - 1, s.I + (int)(((long long)sample_i * max(0, s.N - s.I - s.L)) / s.sampleN)), u, src_stride);
  };
  float2 bounds;
  if constexpr (SRC::kFromCodes) {
    const int b = u / s.Hkv, g = u % s.Hkv;
    for (int i = tid; i < kNB; i += NT) hist[i] = 0u;
    bounds = build_lut<T, NT, LM>(
        q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * LM * s.C * (kD / LM), s.G, s.C, lut, qs, red, tile,
        [&](int slot) { PQC_MARK(ws, 0, slot); }, issue_loads);
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
  for (int v = 0; v < kMaxVecA; ++v) src.fix_tail(raw[v], chunk0 + min(v * NT + tid, chunks - 1));
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
  for (int v = 0; v < kMaxVecA; ++v) {
    if (v * NT + tid < chunks) {
      const int t0 = (chunk0 + v * NT + tid) * P - src.lead;
      unsigned st[P];  // what the select kernel will read back: bin + 1, or the window mark
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

// ------------------------------------------------------ 2. finishing a unit
// The select workgroups of a unit each leave a partial softmax state per query head and their boundary-bin
// candidates behind.  Nobody ever waits for anybody inside the kernel: whoever finishes last does the next step,
// which it learns from a ticket drawn with one returning atomic.
//   - Groups of grpC consecutive workgroups: the last one of a group folds the group's partial states into one
//     (fold_group), so that the unit's last workgroup has few states to read: a single compute unit reads
//     memory that other compute units wrote at a small fraction of the chip's bandwidth, so what it reads must be small.
//     (Units with at most grpC workgroups skip this level.)
//   - The unit's last workgroup (finalize_unit) ranks the candidates and admits the K - n_above best (at most
//     kCandRec candidates: all that is needed sits in their records, which arrive in a different order on every
//     run, so every sum over candidates is taken in rank order; more candidates: an 8-bit radix select over the
//     composites staged per workgroup, the admitted rows being attended from the K/V cache), folds the group
//     states (in order) and the admitted rows into out_attn, writes the admitted candidates' indices, and zeroes
//     the unit's histogram and counters again, which nothing reads after this point: every call leaves them as it
//     found them.
// Index output: every select workgroup publishes its list sizes as soon as it has classified its tokens; when it
// is done attending it reads the sizes of all workgroups of the unit and, if they are all there (they practically
// always are), writes its list straight into out_idx behind those of the workgroups before it.  Otherwise it
// stages the list and the unit's last workgroup copies it.  In workgroup order the lists read
//     [0..I) , tokens above the threshold bin (ascending) , [N-L..N)
// and the admitted candidates go between the second and the third part.
constexpr int kVBatch = 32;                     // admitted candidates' V elements a thread keeps in flight
constexpr int kMaxGroups = 128;                 // groups per unit, at most (kMaxBlkC / 4)
constexpr unsigned kStagedFlag = 0x40000000u;   // in a stored list size: the list sits in its staging slot, not in out_idx
template <int G>
constexpr int fold_width() { return G >= 8 ? 4 : 8; }  // states folded at once = workgroups per group (about 16 KB of states)

// The code of one appended token per unit (Section 3.1: nearest centroid of each partition): nothing in the
// step depends on it, so one more workgroup per unit of the select kernel computes it beside the others.
struct AppendArgs {
  const void* key;    // [units][kD] in the cache's element type, or null: nothing to append
  const float* cent;  // [units][M][C][Dm]
  uint8_t* codes;     // the code tensor; written at `position` of every unit
  int position;
  unsigned* pair_counts;  // two partitions: [units][C*C] counts that gain the token's code pair, or null
};

// Softmax states of the heads a thread owns (heads hb, hb + 2, ... of the group; one head when the group has one),
// for output dimension d.
template <int G>
struct Folded {
  static constexpr int HPT = G >= 2 ? G / 2 : 1;
  float m[HPT], l[HPT], acc[HPT];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int i = 0; i < HPT; ++i) {
      m[i] = kNegBig;
      l[i] = 0.0f;
      acc[i] = 0.0f;
    }
  }
};

// Folds `count` states -- per state G heads of { m, l, acc[kD] } -- into r, in order, fold_width() states at a time
// (all their loads in flight together).  The result depends on the states and their order alone.
template <int G>
__device__ __forceinline__ void fold_states(const float* __restrict__ src, int count, int d, int hb, Folded<G>& r) {
  constexpr int F = fold_width<G>(), HPT = Folded<G>::HPT;
  constexpr size_t stride = (size_t)G * (kD + 2);
#pragma unroll 1
  for (int j0 = 0; j0 < count; j0 += F) {
    float2 ml[HPT][F];
    float a[HPT][F];
#pragma unroll
    for (int x = 0; x < F; ++x) {
      const float* p = src + (size_t)min(j0 + x, count - 1) * stride;
#pragma unroll
      for (int i = 0; i < HPT; ++i) {
        const float* ph = p + (G >= 2 ? hb + 2 * i : 0) * (kD + 2);
        ml[i][x] = *reinterpret_cast<const float2*>(ph);
        a[i][x] = ph[2 + d];
      }
    }
    PQC_LOADS_ISSUED();
#pragma unroll
    for (int i = 0; i < HPT; ++i) {
      float mc = r.m[i];
#pragma unroll
      for (int x = 0; x < F; ++x) mc = j0 + x < count ? fmaxf(mc, ml[i][x].x) : mc;
      const float f = __builtin_amdgcn_exp2f(r.m[i] - mc);
      r.l[i] *= f;
      r.acc[i] *= f;
      r.m[i] = mc;
#pragma unroll
      for (int x = 0; x < F; ++x) {
        const float wv = j0 + x < count ? __builtin_amdgcn_exp2f(ml[i][x].x - mc) : 0.0f;
        r.l[i] = fmaf(wv, ml[i][x].y, r.l[i]);
        r.acc[i] = fmaf(wv, a[i][x], r.acc[i]);
      }
    }
  }
}

template <int G, bool ATTN>
struct TailLds {
  static constexpr int NW = 4, GA = ATTN ? G : 1, GG = GA > 4 ? 4 : GA;
  struct Few {                            // at most kCandRec candidates: ranked here
    unsigned long long comp[kCandRec];    // composites in record order
    float lg[GA][kCandRec];               // by rank: logit of head h (log2 domain)
    unsigned short ordv[kCandRec];        // by rank: record
  };
  struct Many {                           // more: radix select, admitted rows attended from the cache
    unsigned rhist[256];
    int digit[2];
    int rows[256];
    float red[ATTN ? NW * GG * (kD + 2) : 1];
    float xacc[GA][kD];                   // one more state per head: the admitted rows
    float xm[8], xl[8];
  };
  union {
    Few few;
    Many many;
  };
  int lsize[kMaxBlkC];                    // list sizes as stored (with kStagedFlag); only when a list was staged
  int pre_sel[kMaxBlkC + 1];              // exclusive prefix sums of the list sizes; likewise
  int pre_cand[kMaxBlkC + 1];             // and of the staged candidate counts (radix path)
  int scan_sm[2 * (2 * NW + 1)];
  int tot[3 * NW];
};

template <typename T, int G, bool ATTN>
__device__ __forceinline__ void finalize_unit(const Shape& s, const Workspace& ws, int u, const T* __restrict__ q,
                                              const T* __restrict__ kc, const T* __restrict__ vc, int* __restrict__ out_idx,
                                              float* __restrict__ out_attn, const AppendArgs& ap, TailLds<G, ATTN>& L,
                                              Folded<ATTN ? G : 1>& r /* the unit's folded states, for this thread's heads */) {
  constexpr int NT = 256, NW = 4;
  constexpr int GA = ATTN ? G : 1;
  constexpr int HPT = Folded<GA>::HPT;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = u / s.Hkv, g = u % s.Hkv, nb = s.nblkC;
  const int2* cnt = ws.stage_cnt + (size_t)u * nb;
  const unsigned long long* stage_u = ws.stage + (size_t)u * nb * s.stageStride;
  const unsigned char* recs = ws.cand_rec + (size_t)u * kCandRec * ws.rec_stride;
  int* out = out_idx + (size_t)u * s.Ktot;
  const int d = tid & (kD - 1), hb = tid >> 7;  // output dimension; first head of this thread
  const bool owner = GA >= 2 || hb == 0;        // this thread owns outputs
  PQC_MARK(ws, 2, 0);

  // ---- everything whose address is known up front is requested first
  const int2 c0 = cnt[min(tid, nb - 1)], c1 = cnt[min(tid + NT, nb - 1)];  // nb <= 2 * NT
  unsigned long long rc[kCandRec / NT];  // record x*NT + tid
  float rl[kCandRec / NT][GA];
  {
    const CandHeader* hd = reinterpret_cast<const CandHeader*>(recs + (size_t)tid * ws.rec_stride);
    rc[0] = hd->composite;
#pragma unroll
    for (int h = 0; h < GA; ++h) rl[0][h] = ATTN ? hd->logit[h] : 0.0f;
  }
  // ---- totals of the list sizes
  int n_list, n_cand;
  bool any_staged;
  {
    int vs = 0, vc2 = 0, vf = 0;
    if (tid < nb) {
      vs = c0.x & (int)~kStagedFlag;
      vc2 = c0.y;
      vf = (c0.x & (int)kStagedFlag) ? 1 : 0;
    }
    if (tid + NT < nb) {
      vs += c1.x & (int)~kStagedFlag;
      vc2 += c1.y;
      vf += (c1.x & (int)kStagedFlag) ? 1 : 0;
    }
    vs = wave_last(wave_inclusive_scan(vs));
    vc2 = wave_last(wave_inclusive_scan(vc2));
    vf = wave_last(wave_inclusive_scan(vf));
    if (lane == 0) {
      L.tot[w] = vs;
      L.tot[NW + w] = vc2;
      L.tot[2 * NW + w] = vf;
    }
    __syncthreads();
    n_list = 0;
    n_cand = 0;
    int nf = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      n_list += L.tot[i];
      n_cand += L.tot[NW + i];
      nf += L.tot[2 * NW + i];
    }
    any_staged = nf > 0;
  }
  const int n_above = max(0, n_list - s.I - s.L);  // n_list = I + (tokens above the bin) + L
  const int need = max(0, min(s.K - n_above, n_cand));
  PQC_MARK(ws, 2, 1);

  const bool few = n_cand <= kCandRec;
  if (__builtin_expect(any_staged || !few, 0)) {
    // exclusive prefix sums of list sizes and candidate counts
    int2 t0, t1 = make_int2(0, 0);
    const int2 p0 = block_exclusive_scan2<NT>(tid < nb ? c0.x & (int)~kStagedFlag : 0, tid < nb ? c0.y : 0, &t0, L.scan_sm);
    if (tid < nb) {
      L.pre_sel[tid] = p0.x;
      L.pre_cand[tid] = p0.y;
      L.lsize[tid] = c0.x;
    }
    if (nb > NT) {  // uniform
      const int2 p1 = block_exclusive_scan2<NT>(tid + NT < nb ? c1.x & (int)~kStagedFlag : 0, tid + NT < nb ? c1.y : 0, &t1, L.scan_sm);
      if (tid + NT < nb) {
        L.pre_sel[tid + NT] = t0.x + p1.x;
        L.pre_cand[tid + NT] = t0.y + p1.y;
        L.lsize[tid + NT] = c1.x;
      }
    }
    if (tid == 0) {
      L.pre_sel[nb] = n_list;
      L.pre_cand[nb] = n_cand;
    }
    __syncthreads();
    // staged lists (rare: a workgroup that could not see every other workgroup's list size when it was done)
#pragma unroll 1
    for (int j = w; j < nb; j += NW) {
      if (L.lsize[j] & (int)kStagedFlag) {
        const int base = L.pre_sel[j], n = L.pre_sel[j + 1] - base;
        const int* src = reinterpret_cast<const int*>(stage_u + (size_t)j * s.stageStride);
#pragma unroll 1
        for (int p = lane; p < n; p += 64) {
          const int pos = base + p, dst = pos < s.I + n_above ? pos : pos + need;
          if (dst < s.Ktot) out[dst] = src[p];
        }
      }
    }
  }
  PQC_MARK(ws, 2, 2);

  int need_few = 0;          // admitted candidates whose logits and V rows come from the records
  bool extra_state = false;  // the radix path left one more state per head in LDS
  if (__builtin_expect(few, 1)) {
    // rank every candidate (count of larger composites); the admitted ones are the `need` best
    if (need > 0) {
#pragma unroll
      for (int x = 1; x < kCandRec / NT; ++x) {
        rc[x] = 0ull;
#pragma unroll
        for (int h = 0; h < GA; ++h) rl[x][h] = 0.0f;
        if (x * NT + tid < n_cand) {  // rare: more than NT candidates
          const CandHeader* hd = reinterpret_cast<const CandHeader*>(recs + (size_t)(x * NT + tid) * ws.rec_stride);
          rc[x] = hd->composite;
#pragma unroll
          for (int h = 0; h < GA; ++h) rl[x][h] = ATTN ? hd->logit[h] : 0.0f;
        }
      }
#pragma unroll
      for (int x = 0; x < kCandRec / NT; ++x)
        if (x * NT + tid < n_cand) L.few.comp[x * NT + tid] = rc[x];
      __syncthreads();
#pragma unroll
      for (int x = 0; x < kCandRec / NT; ++x) {
        const int k = x * NT + tid;
        if (k < n_cand) {
          const unsigned long long mine = rc[x];
          int rank = 0;
#pragma unroll 1
          for (int j0 = 0; j0 < n_cand; j0 += 8) {  // eight independent LDS reads per round
            unsigned long long o[8];
#pragma unroll
            for (int y = 0; y < 8; ++y) o[y] = L.few.comp[min(j0 + y, n_cand - 1)];
#pragma unroll
            for (int y = 0; y < 8; ++y) rank += (j0 + y < n_cand && o[y] > mine) ? 1 : 0;
          }
          if (rank < need) {
            const int dst = s.I + n_above + rank;  // best first
            if (dst < s.Ktot) out[dst] = composite_token(mine);
#pragma unroll
            for (int h = 0; h < GA; ++h) L.few.lg[h][rank] = rl[x][h] * s.scale_log2e;
            L.few.ordv[rank] = (unsigned short)k;
          }
        }
      }
    }
    need_few = need;
  } else {
    // radix select of the need-th largest staged composite, 8 bits per pass
    auto owner_of = [&](int p) -> int {  // largest j with pre_cand[j] <= p
      int lo = 0, hi = nb - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (L.pre_cand[mid] <= p) lo = mid; else hi = mid - 1;
      }
      return lo;
    };
    auto cand_at = [&](int i) -> unsigned long long {
      const int j = owner_of(i);
      return stage_u[(size_t)j * s.stageStride + s.tokC - 1 - (i - L.pre_cand[j])];
    };
    unsigned long long thr = ~0ull;
    if (need > 0) {
      unsigned long long prefix = 0;
      int want = need;
      for (int shift = 56; shift >= 0; shift -= 8) {
        L.many.rhist[tid] = 0u;
        __syncthreads();
        for (int i = tid; i < n_cand; i += NT) {
          const unsigned long long c = cand_at(i);
          if (shift == 56 || (c >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&L.many.rhist[(unsigned)(c >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
          int cum = 0, dg = 255;
          for (; dg > 0; --dg) {
            if (cum + (int)L.many.rhist[dg] >= want) break;
            cum += (int)L.many.rhist[dg];
          }
          L.many.digit[0] = dg;
          L.many.digit[1] = want - cum;
        }
        __syncthreads();
        prefix |= (unsigned long long)L.many.digit[0] << shift;
        want = L.many.digit[1];
        __syncthreads();
      }
      thr = prefix;
    }
    // admitted candidates in staged order, NT candidates per round: indices out, rows attended for up to four heads
    // at a time (the rounds are repeated for the next four)
    constexpr int GG = TailLds<G, ATTN>::GG;
    for (int h0 = 0; h0 < GA; h0 += GG) {
      AttnState<GG> st;
      st.init();
      float qr[GG][8];
      if constexpr (ATTN) load_query<T, GG>(q + ((size_t)b * s.Hq + (size_t)g * G + h0) * kD, s.scale_log2e, qr);
      int carry = 0;
      for (int i0 = 0; i0 < (need > 0 ? n_cand : 0); i0 += NT) {
        const int i = i0 + tid;
        unsigned long long c = 0;
        if (i < n_cand) c = cand_at(i);
        const int flag = (i < n_cand && c >= thr) ? 1 : 0;
        int tot;
        const int pos = block_exclusive_scan<NT>(flag, &tot, L.scan_sm);
        if (flag) {
          L.many.rows[pos] = composite_token(c);
          const int dst = s.I + n_above + carry + pos;
          if (h0 == 0 && dst < s.Ktot) out[dst] = composite_token(c);
        }
        __syncthreads();
        if constexpr (ATTN) {
          constexpr int R = sizeof(T) == 4 ? 2 : 4;
          auto row_at = [&](int p) -> int { return L.many.rows[p]; };
          attend_rows<T, GG, R>(kc + (size_t)u * s.cap * kD, vc + (size_t)u * s.cap * kD, s.N, row_at, tot, w * 4 * R, NW * 4 * R, qr, st);
        }
        __syncthreads();
        carry += tot;
      }
      if constexpr (ATTN) {
        stash_wave_state<T, GG>(st, L.many.red);
        __syncthreads();
        for (int o = tid; o < GG * kD; o += NT) {
          const int h = o / kD, dd = o % kD;
          float m, l, acc;
          combine_waves<GG, NW>(L.many.red, h, dd, m, l, acc);
          L.many.xacc[h0 + h][dd] = acc;
          if (dd == 0) {
            L.many.xm[h0 + h] = m;
            L.many.xl[h0 + h] = l;
          }
        }
        __syncthreads();
        extra_state = true;
      }
    }
  }
  __syncthreads();
  PQC_MARK(ws, 2, 3);

  if constexpr (ATTN) {
    // ---- out[h][d] = (folded states + admitted candidates, in rank order) / l
    if (owner) {
      int hh[HPT];
#pragma unroll
      for (int i = 0; i < HPT; ++i) hh[i] = G >= 2 ? hb + 2 * i : 0;
      if (extra_state) {
#pragma unroll
        for (int i = 0; i < HPT; ++i) {
          const float xm = L.many.xm[hh[i]], mc = fmaxf(r.m[i], xm);
          const float f = __builtin_amdgcn_exp2f(r.m[i] - mc), fx = __builtin_amdgcn_exp2f(xm - mc);
          r.l[i] = fmaf(L.many.xl[hh[i]], fx, r.l[i] * f);
          r.acc[i] = fmaf(L.many.xacc[hh[i]][d], fx, r.acc[i] * f);
          r.m[i] = mc;
        }
      }
      if (need_few > 0) {
#pragma unroll
        for (int i = 0; i < HPT; ++i) {
          float mc = r.m[i];
#pragma unroll 4
          for (int k = 0; k < need_few; ++k) mc = fmaxf(mc, L.few.lg[hh[i]][k]);
          const float f = __builtin_amdgcn_exp2f(r.m[i] - mc);
          r.l[i] *= f;
          r.acc[i] *= f;
          r.m[i] = mc;
        }
#pragma unroll 1
        for (int r0 = 0; r0 < need_few; r0 += kVBatch) {
          float vv[kVBatch];
#pragma unroll
          for (int x = 0; x < kVBatch; ++x) {
            const int k = L.few.ordv[min(r0 + x, need_few - 1)];
            vv[x] = load_as_float<T>(reinterpret_cast<const T*>(recs + (size_t)k * ws.rec_stride + sizeof(CandHeader)), d);
          }
          PQC_LOADS_ISSUED();
#pragma unroll
          for (int x = 0; x < kVBatch; ++x)
#pragma unroll
            for (int i = 0; i < HPT; ++i) {
              const float p = r0 + x < need_few ? __builtin_amdgcn_exp2f(L.few.lg[hh[i]][min(r0 + x, need_few - 1)] - r.m[i]) : 0.0f;
              r.l[i] += p;
              r.acc[i] = fmaf(p, vv[x], r.acc[i]);
            }
        }
      }
#pragma unroll
      for (int i = 0; i < HPT; ++i) out_attn[((size_t)b * s.Hq + (size_t)g * G + hh[i]) * kD + d] = r.acc[i] / r.l[i];
    }
    PQC_MARK(ws, 2, 5);
  }

  // ---- every select workgroup of the unit is done with them: zero the histogram and the unit's counters
  {
    uint4* gh = reinterpret_cast<uint4*>(ws.hist + (size_t)u * s.histCopies * kNB);
    for (int i = tid; i < s.histCopies * (kNB / 4); i += NT) gh[i] = make_uint4(0u, 0u, 0u, 0u);
    for (int i = tid; i < nb; i += NT) ws.pub[(size_t)u * nb + i] = 0ull;
    if (tid < kMaxGroups) ws.gticket[(size_t)u * kMaxGroups + tid] = 0u;
    if (tid == 0) {
      ws.cand_count[u] = 0u;
      ws.ticket[u] = 0u;
      if (ap.key && ap.pair_counts) {  // the appended token's code pair joins the counts now that nobody reads them
        const uint8_t* cp = ap.codes + ((size_t)u * s.cap + ap.position) * 2;
        const unsigned a0c = cp[0], a1c = cp[1];
        if (a0c < (unsigned)s.C && a1c < (unsigned)s.C) ap.pair_counts[(size_t)u * s.C * s.C + a0c + (size_t)s.C * a1c] += 1u;
      }
    }
  }
  PQC_MARK(ws, 2, 6);
  PQC_NOTE(ws, 2, 13, n_above);
  PQC_NOTE(ws, 2, 14, n_cand);
  PQC_NOTE(ws, 2, 15, need);
}

// The code of the appended token of unit u (one thread per centroid, the distance chain of pq_assign_kernel, the
// smallest (distance, centroid) pair of each partition through a 64-bit LDS minimum).
struct AppendLds {
  float ax[kD];
  unsigned long long abest[8];
};
template <typename T>
__device__ __forceinline__ void append_token(const Shape& s, const AppendArgs& ap, int u, AppendLds& A) {
  const int c = threadIdx.x;
  if (c < kD) A.ax[c] = load_as_float<T>(static_cast<const T*>(ap.key), (size_t)u * kD + c);
  if (c < 8) A.abest[c] = ~0ull;
  __syncthreads();
  if (c < s.C) {
    for (int j = 0; j < s.M; ++j) {
      const float* cr = ap.cent + (((size_t)u * s.M + j) * s.C + c) * s.Dm;
      const float* xj = A.ax + j * s.Dm;
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
      atomicMin(&A.abest[j], ((unsigned long long)__float_as_uint(d2) << 32) | (unsigned)c);  // d2 >= 0: bits order like values
    }
  }
  __syncthreads();
  if (c < s.M) store_through(&ap.codes[((size_t)u * s.cap + ap.position) * s.M + c], (uint8_t)(A.abest[c] & 0xffu));
}

// Draws a ticket from `counter`; true for the workgroup that draws the last of `total`.  What a workgroup leaves
// for whoever draws the last ticket was stored with store_through(); those stores have completed (every wave waits
// for its own, then the barrier) before the ticket is drawn, and the last workgroup drops whatever its caches hold
// before it reads the others' data.
__device__ __forceinline__ bool last_ticket(unsigned* counter, int total, int* ticket_sm) {
  __builtin_amdgcn_s_waitcnt(0);  // all counters at zero: this wave's stores are acknowledged
  __syncthreads();
  if (threadIdx.x == 0) *ticket_sm = (int)atomicAdd(counter, 1u);
  __syncthreads();
  const bool last = *ticket_sm == total - 1;
  if (last) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return last;
}

// ---------------------------------------------------- 3. select (+ attention)
// One workgroup owns tokens [bx*tokC, +tokC) of its unit (bx: its number inside the unit); its 4 waves each own
// a contiguous quarter.  The histogram kernel left every token's bin behind, so a token
// is classified by comparing that number with the threshold bin.  Per wave, lanes hold
// 8 consecutive tokens, counts are prefix-summed across lanes, and the wave appends to
// its own LDS segment: selected tokens (ascending) from the front, boundary-bin
// candidates from the back.  SRC is only used to score the few candidates exactly.
constexpr int kMaxVecC = 4;  // 8-token groups per lane (tokC <= 8192)

// PAIRS (M = 2 only): there is no histogram kernel in front; the threshold comes from the
// code-pair counts (pair_threshold) and tokens are classified by their exact score keys.
//
// Grid (nblkC [+ 1], units): workgroup nblkC of a unit, present when a token is appended, computes
// that token's code.  The last workgroup of a unit to finish completes the unit (finalize_unit);
// the LDS of that step overlays the LDS of the selection, which is dead by then.
template <typename T, int G, bool ATTN, bool PAIRS>
struct SelectLds {
  static constexpr int NW = 4;
  static constexpr bool kMfma = ATTN && sizeof(T) == 2;
  std::conditional_t<PAIRS, PairLds, int> pl;
  int scan_sm[2 * NW + 1 + 4];
  int wcnt[2 * NW];
  float red[ATTN ? NW * G * (kD + 2) : 1];
  float qlds[ATTN ? G * kD : 1];
  __attribute__((aligned(16))) unsigned char vtile[kMfma ? NW * kVTileBytes : 16];
};
template <class A, class B, class C>
constexpr size_t max_size() {
  return sizeof(A) > sizeof(B) ? (sizeof(A) > sizeof(C) ? sizeof(A) : sizeof(C)) : (sizeof(B) > sizeof(C) ? sizeof(B) : sizeof(C));
}

// All arguments of the select kernel in one block, so that the step that completes a unit can read them again
// from the kernel-argument segment when it runs (late_kernel_args) instead of holding them in registers throughout.
struct SelectArgs {
  Shape s;
  Workspace ws;
  const void* q;            // [B][Hq][kD]
  const void* kc;           // K cache
  const void* vc;           // V cache
  const void* src;          // codes, or the score array of the stand-alone top-k
  int* out_idx;
  float* out_attn;
  AppendArgs ap;
  const float* cent;            // PAIRS: centroids
  const unsigned* pair_counts;  // PAIRS: tokens per code pair
  int uncounted;                // PAIRS: a window token not in the counts yet, or -1
};

// The kernel's argument block (its only parameter), read where this is called: scalar loads from the
// kernel-argument segment.  The pointer is made opaque first, so that the loads stay behind this point.
template <class A>
__device__ __forceinline__ const A& late_kernel_args() {
  auto p = (const __attribute__((address_space(4))) A*)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(p));
  return *(const A*)p;
}

// What a workgroup does when it is done with its own part: draw a ticket; the last of a group folds the group's
// states into one and draws a ticket of the unit; the last of the unit folds the groups' states and completes the
// unit.  Both levels run the same loop body, so that the second pass finds its instructions in the cache.
// level: 0 for a select workgroup of a unit with groups, 1 otherwise (units without groups, the appending workgroup).
template <typename T, int G, bool ATTN>
__device__ __forceinline__ void finish_late(int u, int bx, unsigned char* smem, int* ticket_sm) {
  constexpr int GA = ATTN ? G : 1, HPT = Folded<GA>::HPT;
  const SelectArgs& a = late_kernel_args<SelectArgs>();
  const int grpC = ATTN ? a.s.grpC : 0, extra = a.ap.key ? 1 : 0;
  const int tid = threadIdx.x, d = tid & (kD - 1), hb = tid >> 7;
  const bool owner = GA >= 2 || hb == 0;
  const int grp = grpC > 0 ? bx / max(grpC, 1) : 0;
  Folded<GA> r;
#pragma unroll 1
  for (int level = (grpC > 0 && bx < a.s.nblkC) ? 0 : 1; level < 2; ++level) {
    unsigned* counter = level == 0 ? &a.ws.gticket[(size_t)u * kMaxGroups + grp] : &a.ws.ticket[u];
    const int total = level == 0 ? min(grpC, a.s.nblkC - grp * grpC) : (grpC > 0 ? a.s.ngrp : a.s.nblkC) + extra;
    if (!last_ticket(counter, total, ticket_sm)) return;
    r.init();
    if constexpr (ATTN) {
      const bool from_groups = level == 1 && grpC > 0;
      const float* src = from_groups ? a.ws.gparts + (size_t)u * kMaxGroups * G * (kD + 2)
                                     : a.ws.partials + ((size_t)u * a.s.npart + (level == 0 ? grp * grpC : 0)) * G * (kD + 2);
      const int count = level == 0 ? total : (grpC > 0 ? a.s.ngrp : a.s.nblkC);
      if (owner) {
        fold_states<G>(src, count, d, hb, r);
        if (level == 0) {
          float* dst = a.ws.gparts + ((size_t)u * kMaxGroups + grp) * G * (kD + 2);
#pragma unroll
          for (int i = 0; i < HPT; ++i) {
            float* dh = dst + (G >= 2 ? hb + 2 * i : 0) * (kD + 2);
            store_through(&dh[2 + d], r.acc[i]);
            if (d == 0) {
              store_through(&dh[0], r.m[i]);
              store_through(&dh[1], r.l[i]);
            }
          }
        }
      }
    }
  }
  finalize_unit<T, G, ATTN>(a.s, a.ws, u, static_cast<const T*>(a.q), static_cast<const T*>(a.kc), static_cast<const T*>(a.vc),
                            a.out_idx, a.out_attn, a.ap, *reinterpret_cast<TailLds<G, ATTN>*>(smem), r);
}

template <typename T, int G, class SRC, bool ATTN, bool PAIRS = false>
__global__ __launch_bounds__(256, 2) void select_kernel(SelectArgs args) {
  const Shape& s = args.s;
  const Workspace& ws = args.ws;
  const T* __restrict__ q = static_cast<const T*>(args.q);
  const T* __restrict__ kc = static_cast<const T*>(args.kc);
  const T* __restrict__ vc = static_cast<const T*>(args.vc);
  const void* __restrict__ src_ptr = args.src;
  const float* __restrict__ cent = args.cent;
  const unsigned* __restrict__ pair_counts = args.pair_counts;
  const int uncounted = args.uncounted;
  constexpr int NT = 256, NW = 4;
  constexpr bool kMfma = ATTN && sizeof(T) == 2;
  static_assert(!PAIRS || (SRC::kFromCodes && SRC::M == 2), "pair counts exist for two partitions only");
  using SelLds = SelectLds<T, G, ATTN, PAIRS>;
  using EndLds = TailLds<G, ATTN>;
  extern __shared__ unsigned short list[];  // [tokC] token offsets from the workgroup's first token
  __shared__ __attribute__((aligned(16))) unsigned char smem[max_size<SelLds, EndLds, AppendLds>()];
  __shared__ int ticket_sm;
  SelLds& S = *reinterpret_cast<SelLds*>(smem);
  auto& pl = S.pl;
  int* scan_sm = S.scan_sm;
  int* wcnt = S.wcnt;
  float* red = S.red;
  float* qlds = S.qlds;
  unsigned char* vtile = S.vtile;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // Workgroups are handed to the 8 XCDs round-robin in launch order (x fastest).  Eight units at a time are
  // interleaved, so that the workgroups of one unit share an XCD: what they leave for the unit's last workgroup
  // is then found in that XCD's L2 (a matter of speed only: the exchange is correct wherever they run).
  int u = blockIdx.y, bx = blockIdx.x;
  {
    const int nx = gridDim.x, lin = blockIdx.y * nx + blockIdx.x, units = s.B * s.Hkv;
    if (lin < (units & ~7) * nx) {
      const int i = lin % (8 * nx);
      u = (lin / (8 * nx)) * 8 + (i & 7);
      bx = i >> 3;
    }
  }
  const int b = u / s.Hkv, g = u % s.Hkv;
  auto select_and_attend = [&]() {
  PQC_MARK(ws, 1, 0);
  // this wave's stored bins, the query and the histogram: all requested up front
  const int tpw = s.tokC / NW;           // tokens per wave, in groups of 8 per lane
  const int gpw = (tpw + 511) / 512;     // groups per lane: 1, 2 or 4 (the last lanes idle when tpw < 512)
  const int wave_t0 = bx * s.tokC + w * tpw;
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
  const int wg_t0 = bx * s.tokC;
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
  // this workgroup's list sizes, for the other workgroups of the unit to place their lists in out_idx
  if (tid == 0) store_through(&ws.pub[(size_t)u * s.nblkC + bx], ((unsigned long long)(unsigned)tot_cand << 32) | (unsigned)(tot_sel + 1));
  // put away (in LDS) once the attention's first loads are back, which arrive after it: no wait, and no register
  // held through the attention
  // Likewise the list sizes of the unit's first 64 workgroups (wave 0, one per lane) are requested there: the
  // workgroups of a unit start together and publish their sizes long before anyone's first rows are back.
  unsigned long long pw0 = 0ull;
  auto put_rec_base = [&]() {
    if (tid == 0 && tot_cand > 0) scan_sm[0] = rec_base;  // scan_sm is idle since the threshold search
    if (w == 0) pw0 = __hip_atomic_load(&ws.pub[(size_t)u * s.nblkC + min(lane, s.nblkC - 1)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
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

  // selected list for the index output
  unsigned long long* stage = ws.stage + ((size_t)u * s.nblkC + bx) * s.stageStride;
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
  const int tok_lo = bx * s.tokC, tok_hi = min(s.N, (bx + 1) * s.tokC);
  const int nI = max(0, min(s.I, tok_hi) - tok_lo), nL = max(0, tok_hi - max(s.N - s.L, tok_lo));
  const int n_own = tot_sel - nI - nL;
  const int n_win = bx < s.I + s.L ? (s.I + s.L - bx + s.nblkC - 1) / s.nblkC : 0;
  const int n_att = n_own + n_win;
  auto att_at = [&](int p) -> int {
    if (p < n_own) return sel_at(p + nI);
    const int wt = bx + (p - n_own) * s.nblkC;
    return wt < s.I ? wt : s.N - s.L + (wt - s.I);
  };
  // the list sizes of the unit's workgroups (wave 0): requested when the attention is done, read further down
  constexpr int PWX = kMaxBlkC / 64;
  unsigned long long pw[PWX];
  auto poll_sizes = [&]() {
    if (w == 0) {
      pw[0] = pw0;
      const bool again = __any(lane < s.nblkC && (unsigned)pw0 == 0u) != 0;  // uniform: some size was not there yet
#pragma unroll
      for (int x = 0; x < PWX; ++x) {
        if (x > 0) pw[x] = 0ull;
        if (x * 64 < s.nblkC && (x > 0 || again))  // uniform
          pw[x] = __hip_atomic_load(&ws.pub[(size_t)u * s.nblkC + min(x * 64 + lane, s.nblkC - 1)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  };
  if constexpr (ATTN) {
    if constexpr (kMfma) {
      bf16x8_t qf[4];
      load_q_frags(reinterpret_cast<const bf16_t*>(q) + ((size_t)b * s.Hq + (size_t)g * G) * kD, G, qf);
      MfmaState st;
      st.init();
      mfma_attend(reinterpret_cast<const bf16_t*>(kbase), reinterpret_cast<const bf16_t*>(vbase), s.N, att_at, n_att,
                  w * 16 * kMfmaTiles, NW * 16 * kMfmaTiles, s.scale_log2e, qf, vtile + w * kVTileBytes, st, put_rec_base);
      PQC_MARK(ws, 1, 4);
      poll_sizes();
      mfma_stash_wave_state<G>(st, red);
    } else {
      float qr[G][8];
      load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
      AttnState<G> st;
      st.init();
      constexpr int R = (G >= 8 || sizeof(T) == 4) ? 2 : 4;
      attend_rows<T, G, R>(kbase, vbase, s.N, att_at, n_att, w * 4 * R, NW * 4 * R, qr, st);
      put_rec_base();
      PQC_MARK(ws, 1, 4);
      poll_sizes();
      stash_wave_state<T, G>(st, red);
    }
    __syncthreads();
    float* part = ws.partials + ((size_t)u * s.npart + bx) * G * (kD + 2);
    for (int o = tid; o < G * kD; o += NT) {
      const int h = o / kD, d = o % kD;
      float m, l, acc;
      combine_waves<G, NW>(red, h, d, m, l, acc);
      store_through(&part[h * (kD + 2) + 2 + d], acc);
      if (d == 0) {
        store_through(&part[h * (kD + 2)], m);
        store_through(&part[h * (kD + 2) + 1], l);
      }
    }
  } else {
    put_rec_base();
    poll_sizes();
  }
  // Where this workgroup's list goes in out_idx: behind the lists of the workgroups before it, if every
  // workgroup's sizes are known by now; otherwise the list is staged for the unit's last workgroup.
  if (w == 0) {
    int before = 0, all_sel = 0, all_cand = 0;
    bool known = true;
#pragma unroll
    for (int x = 0; x < PWX; ++x) {
      if (x * 64 < s.nblkC) {  // uniform
        const int j = x * 64 + lane;
        const unsigned lo = (unsigned)pw[x], hi = (unsigned)(pw[x] >> 32);
        if (j < s.nblkC) {
          known = known && lo != 0u;
          const int sz = lo != 0u ? (int)lo - 1 : 0;
          all_sel += sz;
          all_cand += (int)hi;
          before += j < bx ? sz : 0;
        }
      }
    }
    known = __all(known) != 0;
    before = wave_last(wave_inclusive_scan(before));
    all_sel = wave_last(wave_inclusive_scan(all_sel));
    all_cand = wave_last(wave_inclusive_scan(all_cand));
    if (lane == 0) {
      scan_sm[1] = known ? before : -1;
      scan_sm[2] = all_sel;
      scan_sm[3] = all_cand;
    }
  }
  __syncthreads();
  const int my_off = scan_sm[1];
  if (my_off >= 0) {  // uniform
    const int n_above_u = max(0, scan_sm[2] - s.I - s.L);
    const int need_u = max(0, min(s.K - n_above_u, scan_sm[3]));
    int* out = args.out_idx + (size_t)u * s.Ktot;
    for (int p = tid; p < tot_sel; p += NT) {
      const int pos = my_off + p, dst = pos < s.I + n_above_u ? pos : pos + need_u;  // the local window goes behind the admitted candidates
      if (dst < s.Ktot) out[dst] = sel_at(p);
    }
  } else {
    for (int p = tid; p < tot_sel; p += NT) store_through(&stage32[p], sel_at(p));
  }
  if (tid == 0)
    store_through(reinterpret_cast<unsigned long long*>(ws.stage_cnt + (size_t)u * s.nblkC + bx),
                  ((unsigned long long)(unsigned)tot_cand << 32) | ((unsigned)tot_sel | (my_off >= 0 ? 0u : kStagedFlag)));
  PQC_MARK(ws, 1, 5);
  PQC_NOTE(ws, 1, 14, tot_sel);
  PQC_NOTE(ws, 1, 15, tot_cand);

  // candidates (few): composite for the generic path, and a full record while slots last
  if (tot_cand > 0) {  // workgroup-uniform
    __syncthreads();  // rec_base was put away by thread 0 (put_rec_base)
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
      if (sub == 0) store_through(&stage[s.tokC - 1 - c], comp);
      if (base + c < kCandRec) {
        unsigned char* rec = ws.cand_rec + ((size_t)u * kCandRec + base + c) * ws.rec_stride;
        CandHeader* hd = reinterpret_cast<CandHeader*>(rec);
        if (sub == 0) store_through(&hd->composite, comp);
        if constexpr (ATTN) {
          float kf[8];
          kr.unpack(kf);
#pragma unroll
          for (int h = 0; h < G; ++h) {
            float d = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(qlds[h * kD + owned_dim<T>(sub, e)], kf[e], d);
            d = group16_sum(d);
            if (sub == 0) store_through(&hd->logit[h], d);
          }
          vr.store_through(rec + sizeof(CandHeader), sub);
        }
      }
    }
  }
  PQC_MARK(ws, 1, 6);
  };  // select_and_attend
  if (bx == s.nblkC)  // the appended token's code; nothing in the step reads it
    append_token<T>(s, args.ap, u, *reinterpret_cast<AppendLds*>(smem));
  else
    select_and_attend();
  // whoever finishes last does the next step: fold the group's states, complete the unit
  finish_late<T, G, ATTN>(u, bx, smem, &ticket_sm);
}

// ------------------------------------------------------------ block reductions
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

// ---------------------------------------------- stand-alone attention over a list
// pqc_gather_attn: workgroup x of unit u attends list positions [x*rowsP, +rowsP).
template <typename T, int G>
__global__ __launch_bounds__(256) void attn_list_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                        const T* __restrict__ kc, const T* __restrict__ vc,
                                                        const int* __restrict__ idx) {
  constexpr int NT = 256, NW = 4;
  constexpr bool kMfma = sizeof(T) == 2;
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
                w * 16 * kMfmaTiles, NW * 16 * kMfmaTiles, s.scale_log2e, qf, vtile + w * kVTileBytes, st, []() {});
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
