// Kernels of libpqcache (gfx950).  Grid layout everywhere: blockIdx.y = unit
// (sequence b, KV head g), blockIdx.x = workgroup inside the unit.
//
// Decode path (pqc_decode), three launches, every dependency at a kernel boundary:
//   hist_kernel      table -> scan codes -> histogram of scores over kNB bins
//   select_kernel    threshold bin from the histogram -> scan codes again -> tokens
//                    above the bin (and the two windows) are listed in ascending order
//                    without atomics and attended at once; tokens inside the bin are
//                    staged as candidates
//   finalize_kernel  ranks the candidates, attends the admitted ones, merges all
//                    partial softmax states, writes indices and output, and leaves
//                    the histogram zeroed for the next call
//
// Codes are read 16 bytes at a time (P = 16/M tokens).  A unit's codes start at byte
// u*N*M, which need not be 16-byte aligned: chunks are laid over the aligned-down
// address, so chunk 0 may begin with up to P-1 "phantom" tokens of the previous unit
// and the last chunk may end with phantoms; both are masked by the token range check.
#pragma once
#include "pqc_device.h"

namespace pqc {

constexpr int kMaxVecA = 4;   // 16-byte code chunks per thread, histogram kernel
constexpr int kMaxVecC = 16;  // 16-byte code chunks per lane, select kernel

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
  __device__ __forceinline__ void init(const void* ptr, int u, int N, int units, const float* lut_) {
    all = static_cast<const uint8_t*>(ptr);
    total_bytes = (long long)units * N * M;
    const long long ob = (long long)u * N * M;
    unit_byte0 = ob & ~15ll;
    lead = (int)((ob - unit_byte0) / M);
    lut = lut_;
  }
  __device__ __forceinline__ Raw load(int chunk) const {
    const long long off = unit_byte0 + 16ll * chunk;
    if (off + 16 <= total_bytes) return *reinterpret_cast<const uint4*>(all + off);
    unsigned w[4] = {0u, 0u, 0u, 0u};  // the tensor's last, partial chunk (or beyond it)
    for (int b = 0; b < 16; ++b)
      if (off + b < total_bytes) w[b >> 2] |= (unsigned)all[off + b] << (8 * (b & 3));
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
  __device__ __forceinline__ float score(const Raw& r, int i) const { return score_from_word<M>(chunk_word<M>(r, i), lut); }
  __device__ __forceinline__ float score_of_token(int t, int u, int N) const {
    const uint8_t* p = all + ((long long)u * N + t) * M;
    typename CodeWord<M>::type w = 0;
#pragma unroll
    for (int j = 0; j < M; ++j) w |= (typename CodeWord<M>::type)p[j] << (8 * j);
    return score_from_word<M>(w, lut);
  }
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
  __device__ __forceinline__ void init(const void* ptr, int u, int N, int, const float*) {
    scores = static_cast<const float*>(ptr) + (size_t)u * N;
    n = N;
    lead = 0;
  }
  __device__ __forceinline__ Raw load(int chunk) const {
    Raw r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long long t = (long long)chunk * 4 + i;
      r.f[i] = t < n ? scores[t] : 0.0f;
    }
    return r;
  }
  __device__ __forceinline__ float score(const Raw& r, int i) const { return r.f[i]; }
  __device__ __forceinline__ float score_of_token(int t, int, int) const { return scores[t]; }
};

// ------------------------------------------------------------------ utilities
__global__ void reset_kernel(unsigned* hist, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) hist[i] = 0u;
}

// Stand-alone table (pqc_lut).
template <typename T, int M>
__global__ __launch_bounds__(256) void lut_kernel(Shape s, const T* __restrict__ q, const float* __restrict__ cent,
                                                  float* __restrict__ table) {
  __shared__ float lut[M * kLutRow];
  __shared__ float qs[kD];
  __shared__ float red[32];
  __shared__ float tile[kLutTileFloats + kLutTileFloats / (kD / M)];
  const int u = blockIdx.y, b = u / s.Hkv, g = u % s.Hkv;
  build_lut<T, 256, M>(q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * M * s.C * (kD / M), s.G, s.C, lut,
                       qs, red, tile);
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
  const W* cw = reinterpret_cast<const W*>(codes) + (size_t)u * s.N;
  const int t0 = blockIdx.x * 2048;
  for (int t = t0 + threadIdx.x; t < min(t0 + 2048, s.N); t += 256) {
    const bool mid = t >= s.I && t < s.N - s.L;
    scores[(size_t)u * s.N + t] = mid ? score_from_word<M>(cw[t], lut) : -INFINITY;
  }
}

// Bin layout from the middle tokens of a score array (stand-alone top-k only): range,
// mean and spread, reduced in a fixed order by one workgroup per unit.
__global__ __launch_bounds__(1024) void score_stats_kernel(Shape s, const float* __restrict__ scores,
                                                           BinParams* __restrict__ ctl) {
  __shared__ float smn[16], smx[16];
  __shared__ double ssum[16], ssq[16];
  const int u = blockIdx.y;
  float mn = INFINITY, mx = -INFINITY;
  double sum = 0.0, sq = 0.0;
  for (int t = s.I + threadIdx.x; t < s.N - s.L; t += 1024) {
    const float v = scores[(size_t)u * s.N + t];
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
    sum += (double)v;
    sq += (double)v * (double)v;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, o));
    mx = fmaxf(mx, __shfl_xor(mx, o));
    sum += __shfl_xor(sum, o);
    sq += __shfl_xor(sq, o);
  }
  if ((threadIdx.x & 63) == 0) {
    smn[threadIdx.x >> 6] = mn;
    smx[threadIdx.x >> 6] = mx;
    ssum[threadIdx.x >> 6] = sum;
    ssq[threadIdx.x >> 6] = sq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w) {
      mn = fminf(mn, smn[w]);
      mx = fmaxf(mx, smx[w]);
      sum += ssum[w];
      sq += ssq[w];
    }
    const double n = (double)max(1, s.N - s.L - s.I);
    const double mean = sum / n, var = fmax(0.0, sq / n - mean * mean);
    const bool finite = mn > -3.0e38f && mx < 3.0e38f && mean == mean && var == var;
    ctl[u] = finite ? make_bins(mn, mx, (float)mean, (float)sqrt(var)) : make_bins(mn, mx, mn, 0.0f);
  }
}

// ------------------------------------------------------------- 1. histogram
// SRC = CodeChunks<M>: builds the unit's table first (workgroup 0 also publishes it
// together with the bin layout).  SRC = ScoreChunks: layout comes from score_stats_kernel.
template <typename T, class SRC>
__global__ __launch_bounds__(1024) void hist_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                    const float* __restrict__ cent, const void* __restrict__ src_ptr) {
  constexpr int NT = 1024, P = SRC::P;
  constexpr int LM = SRC::kFromCodes ? SRC::M : 1;
  __shared__ float lut[LM * kLutRow];
  __shared__ float qs[kD];
  __shared__ float red[32];
  __shared__ float tile[SRC::kFromCodes ? kLutTileFloats + kLutTileFloats / (kD / LM) : 1];
  __shared__ unsigned hist[kNB];
  const int u = blockIdx.y, tid = threadIdx.x;
  PQC_MARK(ws, 0, 0);
  SRC src;
  src.init(src_ptr, u, s.N, s.B * s.Hkv, lut);
  // this workgroup's chunks: issue the loads before anything else
  const int chunks = s.tokA / P, chunk0 = blockIdx.x * chunks;
  typename SRC::Raw raw[kMaxVecA];
#pragma unroll
  for (int v = 0; v < kMaxVecA; ++v)
    if (v * NT + tid < chunks) raw[v] = src.load(chunk0 + v * NT + tid);
  for (int i = tid; i < kNB; i += NT) hist[i] = 0u;
  BinParams bp;
  if constexpr (SRC::kFromCodes) {
    const int b = u / s.Hkv, g = u % s.Hkv;
    bp = build_lut<T, NT, LM>(q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * LM * s.C * (kD / LM), s.G,
                              s.C, lut, qs, red, tile);
    if (blockIdx.x == 0) {
      for (int e = tid; e < LM * s.C; e += NT) ws.lut[(size_t)u * LM * s.C + e] = lut[(e / s.C) * kLutRow + (e % s.C)];
      if (tid == 0) ws.ctl[u] = bp;
    }
  } else {
    bp = ws.ctl[u];
    __syncthreads();
  }
  PQC_MARK(ws, 0, 1);
#pragma unroll
  for (int v = 0; v < kMaxVecA; ++v) {
    if (v * NT + tid < chunks) {
      const int t0 = (chunk0 + v * NT + tid) * P - src.lead;
#pragma unroll
      for (int i = 0; i < P; ++i) {
        const int t = t0 + i;
        if (t >= s.I && t < s.N - s.L) atomicAdd(&hist[score_bin(src.score(raw[v], i), bp)], 1u);
      }
    }
  }
  __syncthreads();
  PQC_MARK(ws, 0, 2);
  unsigned* gh = ws.hist + (size_t)u * kNB;
  for (int i = tid; i < kNB; i += NT)
    if (hist[i]) atomicAdd(&gh[i], hist[i]);
  PQC_MARK(ws, 0, 3);
}

// ---------------------------------------------------- 2. select (+ attention)
// One workgroup owns virtual tokens [blockIdx.x*tokC, +tokC) of its unit; its 4 waves
// each own a contiguous quarter.  Per wave, lanes hold consecutive chunks, counts are
// prefix-summed across lanes, and the wave appends to its own LDS segment: selected
// tokens (ascending) from the front, boundary-bin candidates from the back.
template <typename T, int G, class SRC, bool ATTN>
__global__ __launch_bounds__(256) void select_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                     const T* __restrict__ kc, const T* __restrict__ vc,
                                                     const void* __restrict__ src_ptr) {
  constexpr int NT = 256, NW = 4, P = SRC::P;
  constexpr int LM = SRC::kFromCodes ? SRC::M : 1;
  extern __shared__ int list[];  // [tokC]
  __shared__ float lut[LM * kLutRow];
  __shared__ int scan_sm[2 * NW + 1 + 4];
  __shared__ int wcnt[2 * NW];
  __shared__ float red[ATTN ? NW * G * (kD + 2) : 1];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  PQC_MARK(ws, 1, 0);
  SRC src;
  src.init(src_ptr, u, s.N, s.B * s.Hkv, lut);
  // this wave's chunks, loaded up front
  const int cpw = s.tokC / (NW * P);  // chunks per wave
  const int chunk0 = blockIdx.x * (s.tokC / P) + w * cpw;
  typename SRC::Raw raw[kMaxVecC];
#pragma unroll
  for (int v = 0; v < kMaxVecC; ++v)
    if (v * 64 + lane < cpw) raw[v] = src.load(chunk0 + v * 64 + lane);
  if constexpr (SRC::kFromCodes)
    for (int e = tid; e < LM * s.C; e += NT) lut[(e / s.C) * kLutRow + (e % s.C)] = ws.lut[(size_t)u * LM * s.C + e];
  const BinParams bp = ws.ctl[u];
  const Threshold th = find_threshold<NT>(ws.hist + (size_t)u * kNB, s.K, scan_sm);  // syncs: lut is ready after it

  PQC_MARK(ws, 1, 1);
  const int segN = s.tokC / NW;
  int* seg = list + w * segN;
  int nsel = 0, ncand = 0;
#pragma unroll
  for (int v = 0; v < kMaxVecC; ++v) {
    if (v * 64 < cpw) {  // wave-uniform
      const bool live = v * 64 + lane < cpw;
      const int t0 = (chunk0 + v * 64 + lane) * P - src.lead;
      unsigned selm = 0u, candm = 0u;
      if (live) {
#pragma unroll
        for (int i = 0; i < P; ++i) {
          const int t = t0 + i;
          if (t >= 0 && t < s.N) {
            if (t < s.I || t >= s.N - s.L) {
              selm |= 1u << i;
            } else {
              const int bin = score_bin(src.score(raw[v], i), bp);
              selm |= (bin > th.bstar ? 1u : 0u) << i;
              candm |= (bin == th.bstar ? 1u : 0u) << i;
            }
          }
        }
      }
      const int cnt = __popc(selm) | (__popc(candm) << 16);
      int inc = cnt;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int n = __shfl_up(inc, o);
        if (lane >= o) inc += n;
      }
      const int tot = __shfl(inc, 63);
      int ps = nsel + ((inc - cnt) & 0xffff), pc = ncand + ((inc - cnt) >> 16);
#pragma unroll
      for (int i = 0; i < P; ++i) {
        if (selm & (1u << i)) seg[ps++] = t0 + i;
        if (candm & (1u << i)) seg[segN - 1 - (pc++)] = t0 + i;
      }
      nsel += tot & 0xffff;
      ncand += tot >> 16;
    }
  }
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
  auto sel_at = [&](int p) -> int {
    int i = 0;
#pragma unroll
    for (int x = 1; x < NW; ++x) i += (p >= csel[x]) ? 1 : 0;
    return list[i * segN + (p - csel[i])];
  };

  // stage lists for the finalize kernel
  unsigned long long* stage = ws.stage + ((size_t)u * s.nblkC + blockIdx.x) * s.tokC;
  int* stage32 = reinterpret_cast<int*>(stage);
  for (int p = tid; p < tot_sel; p += NT) stage32[p] = sel_at(p);
  for (int c = tid; c < tot_cand; c += NT) {
    int i = 0;
#pragma unroll
    for (int x = 1; x < NW; ++x) i += (c >= ccand[x]) ? 1 : 0;
    const int t = list[i * segN + segN - 1 - (c - ccand[i])];
    stage[s.tokC - 1 - c] = make_composite(src.score_of_token(t, u, s.N), t);
  }
  if (tid == 0) ws.stage_cnt[(size_t)u * s.nblkC + blockIdx.x] = make_int2(tot_sel, tot_cand);
  PQC_MARK(ws, 1, 3);

  if constexpr (ATTN) {
    const int b = u / s.Hkv, g = u % s.Hkv;
    float qr[G][8];
    load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
    AttnState<G> st;
    st.init();
    constexpr int R = (G >= 8 || sizeof(T) == 4) ? 2 : 4;
    attend_rows<T, G, R>(kc + (size_t)u * s.N * kD, vc + (size_t)u * s.N * kD, s.N, sel_at, tot_sel, w * 4 * R,
                         NW * 4 * R, qr, st);
    PQC_MARK(ws, 1, 4);
    stash_wave_state<T, G, NW>(st, red);
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
    PQC_MARK(ws, 1, 5);
#ifdef PQC_TRACE
    if (tid == 0 && (size_t)blockIdx.y * gridDim.x + blockIdx.x < (size_t)kTraceWgs) {
      unsigned long long* tr = ws.trace + ((size_t)1 * kTraceWgs + (size_t)blockIdx.y * gridDim.x + blockIdx.x) * kTraceSlots;
      tr[14] = (unsigned long long)tot_sel;
      tr[15] = (unsigned long long)tot_cand;
    }
#endif
  }
}

// ------------------------------------------------------------- 3. finalize
// One workgroup (512 threads, so that 8 query heads fit the register file) per unit.
// The staged "selected" lists already hold the two windows: concatenated in workgroup
// order they read  [0..I) , tokens above the threshold bin (ascending) , [N-L..N).
template <typename T, int G, bool ATTN>
__global__ __launch_bounds__(512) void finalize_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                       const T* __restrict__ kc, const T* __restrict__ vc,
                                                       int* __restrict__ out_idx, float* __restrict__ out_attn) {
  constexpr int NT = 512, NW = 8;
  extern __shared__ int pre[];  // [2*(nblkC+1)]: prefix of selected counts, prefix of candidate counts
  __shared__ int scan_sm[2 * NW + 1];
  __shared__ unsigned long long comp[kCandLds];
  __shared__ int adm[kCandLds];
  __shared__ unsigned rhist[256];
  __shared__ unsigned long long thr_sm;
  __shared__ int digit_sm[2];
  __shared__ float red[ATTN ? NW * G * (kD + 2) : 1];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  PQC_MARK(ws, 2, 0);
  int* pre_sel = pre;
  int* pre_cand = pre + (s.nblkC + 1);
  unsigned* gh = ws.hist + (size_t)u * kNB;
  for (int i = tid; i < kNB; i += NT) gh[i] = 0u;  // all readers finished with the previous launch: ready for the next call

  // prefix sums of the per-workgroup list sizes
  const int2* cnt = ws.stage_cnt + (size_t)u * s.nblkC;
  int carry_s = 0, carry_c = 0;
  for (int j0 = 0; j0 < s.nblkC; j0 += NT) {
    const int j = j0 + tid;
    const int2 c = j < s.nblkC ? cnt[j] : make_int2(0, 0);
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
  const int n_list = carry_s;  // I + (tokens above the bin) + L
  const int n_above = max(0, n_list - s.I - s.L);
  const int n_cand = carry_c;
  const int need = max(0, min(s.K - n_above, n_cand));
  auto owner = [&](const int* prefix, int p) -> int {  // largest j with prefix[j] <= p
    int lo = 0, hi = s.nblkC - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (prefix[mid] <= p) lo = mid; else hi = mid - 1;
    }
    return lo;
  };
  const unsigned long long* stage_u = ws.stage + (size_t)u * s.nblkC * s.tokC;
  int* out = out_idx + (size_t)u * s.Ktot;
  PQC_MARK(ws, 2, 1);

  // indices of the staged lists: one wave per list, coalesced; the local window moves
  // behind the admitted candidates
  for (int j = w; j < s.nblkC; j += NW) {
    const int base = pre_sel[j], n = pre_sel[j + 1] - base;
    const int* src = reinterpret_cast<const int*>(stage_u + (size_t)j * s.tokC);
    for (int p = lane; p < n; p += 64) {
      const int pos = base + p;
      out[pos < s.I + n_above ? pos : pos + need] = src[p];
    }
  }

  PQC_MARK(ws, 2, 2);
  // candidates: the `need` best by (score desc, token asc) are admitted, listed in token order
  auto cand_at = [&](int i) -> unsigned long long {
    const int j = owner(pre_cand, i);
    return stage_u[(size_t)j * s.tokC + s.tokC - 1 - (i - pre_cand[j])];
  };
  const bool in_lds = n_cand <= kCandLds;
  if (need > 0) {
    if (in_lds) {
      for (int i = tid; i < n_cand; i += NT) comp[i] = cand_at(i);
      __syncthreads();
      for (int i = tid; i < n_cand; i += NT) {
        const unsigned long long mine = comp[i];
        int rank = 0;
        for (int j = 0; j < n_cand; ++j) rank += comp[j] > mine ? 1 : 0;
        if (rank == need - 1) thr_sm = mine;
      }
      __syncthreads();
    } else {
      // radix select of the need-th largest composite, 8 bits per pass, through global memory
      unsigned long long prefix = 0;
      int want = need;
      for (int shift = 56; shift >= 0; shift -= 8) {
        if (tid < 256) rhist[tid] = 0u;
        __syncthreads();
        for (int i = tid; i < n_cand; i += NT) {
          const unsigned long long c = cand_at(i);
          if (shift == 56 || (c >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&rhist[(unsigned)(c >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
          int cum = 0, d = 255;
          for (; d > 0; --d) {
            if (cum + (int)rhist[d] >= want) break;
            cum += (int)rhist[d];
          }
          digit_sm[0] = d;
          digit_sm[1] = want - cum;
        }
        __syncthreads();
        prefix |= (unsigned long long)digit_sm[0] << shift;
        want = digit_sm[1];
        __syncthreads();
      }
      if (tid == 0) thr_sm = prefix;
      __syncthreads();
    }
    const unsigned long long thr = thr_sm;
    int carry = 0;
    for (int i0 = 0; i0 < n_cand; i0 += NT) {
      const int i = i0 + tid;
      unsigned long long c = 0;
      if (i < n_cand) c = in_lds ? comp[i] : cand_at(i);
      const int flag = (i < n_cand && c >= thr) ? 1 : 0;
      int tot;
      const int pos = block_exclusive_scan<NT>(flag, &tot, scan_sm);
      if (flag && carry + pos < need) {
        const int t = composite_token(c);
        out[s.I + n_above + carry + pos] = t;
        if (need <= kCandLds) adm[carry + pos] = t;
      }
      carry += tot;
    }
  }

  PQC_MARK(ws, 2, 3);
  if constexpr (ATTN) {
    __syncthreads();  // admitted list (LDS, or this workgroup's own global writes) visible to all its threads
    const int b = u / s.Hkv, g = u % s.Hkv;
    AttnState<G> st;
    st.init();
    if (need > 0) {
      float qr[G][8];
      load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
      constexpr int R = 2;
      if (need <= kCandLds) {
        auto row_at = [&](int p) -> int { return adm[p]; };
        attend_rows<T, G, R>(kc + (size_t)u * s.N * kD, vc + (size_t)u * s.N * kD, s.N, row_at, need, w * 4 * R, NW * 4 * R,
                             qr, st);
      } else {
        auto row_at = [&](int p) -> int { return out[s.I + n_above + p]; };
        attend_rows<T, G, R>(kc + (size_t)u * s.N * kD, vc + (size_t)u * s.N * kD, s.N, row_at, need, w * 4 * R, NW * 4 * R,
                             qr, st);
      }
    }
    PQC_MARK(ws, 2, 4);
    stash_wave_state<T, G, NW>(st, red);
    __syncthreads();
    const float* parts = ws.partials + (size_t)u * s.npart * G * (kD + 2);
    for (int o = tid; o < G * kD; o += NT) {
      const int h = o / kD, d = o % kD;
      float m, l, acc;
      combine_waves<G, NW>(red, h, d, m, l, acc);
      for (int j0 = 0; j0 < s.nblkC; j0 += 8) {
        float mj[8], lj[8], aj[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const bool ok = j0 + x < s.nblkC;
          const float* pj = parts + ((size_t)(ok ? j0 + x : j0) * G + h) * (kD + 2);
          mj[x] = ok ? pj[0] : kNegBig;
          lj[x] = ok ? pj[1] : 0.0f;
          aj[x] = ok ? pj[2 + d] : 0.0f;
        }
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const float mn = fmaxf(m, mj[x]);
          const float fa = __builtin_amdgcn_exp2f(m - mn), fb = __builtin_amdgcn_exp2f(mj[x] - mn);
          l = l * fa + lj[x] * fb;
          acc = acc * fa + aj[x] * fb;
          m = mn;
        }
      }
      out_attn[((size_t)b * s.Hq + (size_t)g * G + h) * kD + d] = acc / l;
    }
    PQC_MARK(ws, 2, 5);
#ifdef PQC_TRACE
    if (tid == 0 && (size_t)blockIdx.y * gridDim.x + blockIdx.x < (size_t)kTraceWgs) {
      unsigned long long* tr = ws.trace + ((size_t)2 * kTraceWgs + (size_t)blockIdx.y * gridDim.x + blockIdx.x) * kTraceSlots;
      tr[13] = (unsigned long long)n_above;
      tr[14] = (unsigned long long)n_cand;
      tr[15] = (unsigned long long)need;
    }
#endif
  }
}

// ---------------------------------------------- stand-alone attention over a list
// pqc_gather_attn: workgroup x of unit u attends list positions [x*rowsP, +rowsP).
template <typename T, int G>
__global__ __launch_bounds__(256) void attn_list_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                        const T* __restrict__ kc, const T* __restrict__ vc,
                                                        const int* __restrict__ idx) {
  constexpr int NT = 256, NW = 4;
  __shared__ float red[NW * G * (kD + 2)];
  const int u = blockIdx.y, tid = threadIdx.x, w = tid >> 6;
  const int b = u / s.Hkv, g = u % s.Hkv;
  const int p0 = blockIdx.x * s.rowsP;
  const int count = min(s.rowsP, s.Ktot - p0);
  const int* lst = idx + (size_t)u * s.Ktot + p0;
  float qr[G][8];
  load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
  AttnState<G> st;
  st.init();
  constexpr int R = (G >= 8 || sizeof(T) == 4) ? 2 : 4;
  auto row_at = [&](int p) -> int { return lst[p]; };
  attend_rows<T, G, R>(kc + (size_t)u * s.N * kD, vc + (size_t)u * s.N * kD, s.N, row_at, count, w * 4 * R, NW * 4 * R,
                       qr, st);
  stash_wave_state<T, G, NW>(st, red);
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

template <int G>
__global__ __launch_bounds__(256) void merge_kernel(Shape s, Workspace ws, int nparts, float* __restrict__ out_attn) {
  const int u = blockIdx.y, b = u / s.Hkv, g = u % s.Hkv;
  const float* parts = ws.partials + (size_t)u * s.npart * G * (kD + 2);
  for (int o = threadIdx.x; o < G * kD; o += 256) {
    const int h = o / kD, d = o % kD;
    float m = kNegBig, l = 0.0f, acc = 0.0f;
    for (int j = 0; j < nparts; ++j) {
      const float* pj = parts + ((size_t)j * G + h) * (kD + 2);
      const float mj = pj[0], lj = pj[1], aj = pj[2 + d];
      const float mn = fmaxf(m, mj);
      const float fa = __builtin_amdgcn_exp2f(m - mn), fb = __builtin_amdgcn_exp2f(mj - mn);
      l = l * fa + lj * fb;
      acc = acc * fa + aj * fb;
      m = mn;
    }
    out_attn[((size_t)b * s.Hq + (size_t)g * G + h) * kD + d] = acc / l;
  }
}

}  // namespace pqc
