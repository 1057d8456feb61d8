// Kernels of libpqcache (gfx950).  Grid layout everywhere: blockIdx.y = unit
// (sequence b, KV head g), blockIdx.x = workgroup inside the unit.
//
// Decode path (pqc_decode), three launches, every dependency at a kernel boundary:
//   hist_kernel      table -> scan codes -> histogram of scores over kNB bins
//   select_kernel    threshold bin from the histogram -> scan codes again -> tokens
//                    above the bin are selected (ordered, no atomics) and attended at
//                    once; tokens inside the bin are staged as candidates
//   finalize_kernel  ranks the candidates, attends them and the two windows, merges
//                    all partial softmax states, writes indices and output, and
//                    leaves the histogram zeroed for the next call
#pragma once
#include "pqc_device.h"

namespace pqc {

// ------------------------------------------------------------------ utilities
__global__ void reset_kernel(unsigned* hist, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) hist[i] = 0u;
}

// Stand-alone table (pqc_lut).
template <typename T>
__global__ __launch_bounds__(256) void lut_kernel(Shape s, const T* __restrict__ q, const float* __restrict__ cent,
                                                  float* __restrict__ table) {
  __shared__ float lut[8 * kLutRow];
  __shared__ float qs[kD];
  __shared__ float red[16];
  const int u = blockIdx.y, b = u / s.Hkv, g = u % s.Hkv;
  float lo, inv_w;
  build_lut<T, 256>(q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * s.M * s.C * s.Dm, s.G, s.M, s.C,
                    s.Dm, lut, qs, red, &lo, &inv_w);
  for (int e = threadIdx.x; e < s.M * s.C; e += 256) table[(size_t)u * s.M * s.C + e] = lut[(e / s.C) * kLutRow + (e % s.C)];
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

// Score range of the middle tokens of a score array (stand-alone top-k only).
__global__ __launch_bounds__(1024) void minmax_kernel(Shape s, const float* __restrict__ scores, float2* __restrict__ ctl) {
  __shared__ float smn[16], smx[16];
  const int u = blockIdx.y;
  float mn = INFINITY, mx = -INFINITY;
  for (int t = s.I + threadIdx.x; t < s.N - s.L; t += 1024) {
    float v = scores[(size_t)u * s.N + t];
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, o));
    mx = fmaxf(mx, __shfl_xor(mx, o));
  }
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
    const float width = mx - mn;
    ctl[u] = make_float2(mn, (width > 1e-30f && width < 3.0e38f) ? (float)kNB / width : 0.0f);
  }
}

// ------------------------------------------------------------- 1. histogram
// SRC = CodeSource<M>: builds the unit's table first (workgroup 0 also publishes it
// together with the score bounds).  SRC = ScoreSource: bounds come from minmax_kernel.
template <typename T, class SRC>
__global__ __launch_bounds__(1024) void hist_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                    const float* __restrict__ cent, const void* __restrict__ src_ptr) {
  constexpr int NT = 1024;
  __shared__ float lut[SRC::kFromCodes ? 8 * kLutRow : 1];
  __shared__ float qs[kD];
  __shared__ float red[16];
  __shared__ unsigned hist[kNB];
  const int u = blockIdx.y, tid = threadIdx.x;
  for (int i = tid; i < kNB; i += NT) hist[i] = 0u;
  float lo, inv_w;
  SRC src;
  if constexpr (SRC::kFromCodes) {
    const int b = u / s.Hkv, g = u % s.Hkv;
    build_lut<T, NT>(q + ((size_t)b * s.Hq + (size_t)g * s.G) * kD, cent + (size_t)u * s.M * s.C * s.Dm, s.G, s.M,
                     s.C, s.Dm, lut, qs, red, &lo, &inv_w);
    if (blockIdx.x == 0) {
      for (int e = tid; e < s.M * s.C; e += NT) ws.lut[(size_t)u * s.M * s.C + e] = lut[(e / s.C) * kLutRow + (e % s.C)];
      if (tid == 0) ws.ctl[u] = make_float2(lo, inv_w);
    }
    src.codes = reinterpret_cast<const typename CodeWord<SRC::M>::type*>(src_ptr) + (size_t)u * s.N;
    src.lut = lut;
  } else {
    const float2 c = ws.ctl[u];
    lo = c.x;
    inv_w = c.y;
    src.scores = reinterpret_cast<const float*>(src_ptr) + (size_t)u * s.N;
  }
  __syncthreads();
  const int t0 = blockIdx.x * s.tokA;
  const int lo_t = max(t0, s.I), hi_t = min(min(t0 + s.tokA, s.N - s.L), s.N);
  for (int t = t0 + tid; t < hi_t; t += NT)
    if (t >= lo_t) atomicAdd(&hist[score_bin(src.score(t), lo, inv_w)], 1u);
  __syncthreads();
  unsigned* gh = ws.hist + (size_t)u * kNB;
  for (int i = tid; i < kNB; i += NT)
    if (hist[i]) atomicAdd(&gh[i], hist[i]);
}

// ---------------------------------------------------- 2. select (+ attention)
// One workgroup owns tokens [blockIdx.x*tokC, +tokC).  Its 4 waves each scan a
// contiguous quarter and compact with wave ballots, so every list is in ascending
// token order without atomics.  LDS list: per wave segment of tokC/4 slots, selected
// tokens from the front, candidates from the back.
template <typename T, int G, class SRC, bool ATTN>
__global__ __launch_bounds__(256) void select_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                     const T* __restrict__ kc, const T* __restrict__ vc,
                                                     const void* __restrict__ src_ptr) {
  constexpr int NT = 256, NW = 4;
  extern __shared__ int list[];  // [tokC]
  __shared__ float lut[SRC::kFromCodes ? 8 * kLutRow : 1];
  __shared__ int scan_sm[2 * NW + 1 + 4];
  __shared__ int wcnt[2 * NW];
  __shared__ float red[ATTN ? NW * G * (kD + 2) : 1];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  SRC src;
  if constexpr (SRC::kFromCodes) {
    for (int e = tid; e < s.M * s.C; e += NT) lut[(e / s.C) * kLutRow + (e % s.C)] = ws.lut[(size_t)u * s.M * s.C + e];
    src.codes = reinterpret_cast<const typename CodeWord<SRC::M>::type*>(src_ptr) + (size_t)u * s.N;
    src.lut = lut;
  } else {
    src.scores = reinterpret_cast<const float*>(src_ptr) + (size_t)u * s.N;
  }
  const float2 ctl = ws.ctl[u];
  const Threshold th = find_threshold<NT>(ws.hist + (size_t)u * kNB, s.K, scan_sm);  // syncs: lut is ready after it

  // scan this wave's quarter
  const int segN = s.tokC / NW;
  int* seg = list + w * segN;
  const int wt0 = blockIdx.x * s.tokC + w * segN;
  const int lo_t = max(wt0, s.I), hi_t = min(wt0 + segN, s.N - s.L);
  int nsel = 0, ncand = 0;
  for (int tb = wt0; tb < hi_t; tb += 64) {
    const int t = tb + lane;
    int bin = -1;
    if (t >= lo_t && t < hi_t) bin = score_bin(src.score(t), ctl.x, ctl.y);
    const bool sel = bin > th.bstar, cand = bin == th.bstar;
    const unsigned long long ms = __ballot(sel), mc = __ballot(cand);
    const unsigned long long below = (1ull << lane) - 1ull;
    if (sel) seg[nsel + __popcll(ms & below)] = t;
    if (cand) seg[segN - 1 - (ncand + __popcll(mc & below))] = t;
    nsel += __popcll(ms);
    ncand += __popcll(mc);
  }
  if (lane == 0) {
    wcnt[w] = nsel;
    wcnt[NW + w] = ncand;
  }
  __syncthreads();
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
    stage[s.tokC - 1 - c] = make_composite(src.score(t), t);
  }
  if (tid == 0) ws.stage_cnt[(size_t)u * s.nblkC + blockIdx.x] = make_int2(tot_sel, tot_cand);

  if constexpr (ATTN) {
    const int b = u / s.Hkv, g = u % s.Hkv;
    float qr[G][8];
    load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
    AttnState<G> st;
    st.init();
    constexpr int R = (G >= 8 || sizeof(T) == 4) ? 2 : 4;
    attend_rows<T, G, R>(kc + (size_t)u * s.N * kD, vc + (size_t)u * s.N * kD, s.N, sel_at, tot_sel, w * 4 * R,
                         NW * 4 * R, qr, st);
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
}

// ------------------------------------------------------------- 3. finalize
// One workgroup (512 threads, so that 8 query heads fit the register file) per unit.
template <typename T, int G, bool ATTN>
__global__ __launch_bounds__(512) void finalize_kernel(Shape s, Workspace ws, const T* __restrict__ q,
                                                        const T* __restrict__ kc, const T* __restrict__ vc,
                                                        int* __restrict__ out_idx, float* __restrict__ out_attn) {
  constexpr int NT = 512, NW = 8;
  extern __shared__ int pre[];  // [2*(nblkC+1)]: prefix of selected counts, prefix of candidate counts
  __shared__ int scan_sm[2 * NW + 1 + 4];
  __shared__ unsigned long long comp[kCandLds];
  __shared__ unsigned rhist[256];
  __shared__ unsigned long long thr_sm;
  __shared__ int digit_sm[2];
  __shared__ float red[ATTN ? NW * G * (kD + 2) : 1];
  const int u = blockIdx.y, tid = threadIdx.x;
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
  const int n_sel = min(carry_s, s.K);   // == th.n_above by construction
  const int n_cand = carry_c;            // == th.n_cand
  const int need = min(s.K - n_sel, n_cand);
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

  // indices: initial window, tokens above the threshold bin, local window
  for (int p = tid; p < s.I; p += NT) out[p] = p;
  for (int p = tid; p < s.L; p += NT) out[s.I + s.K + p] = s.N - s.L + p;
  for (int p = tid; p < n_sel; p += NT) {
    const int j = owner(pre_sel, p);
    out[s.I + p] = reinterpret_cast<const int*>(stage_u + (size_t)j * s.tokC)[p - pre_sel[j]];
  }

  // candidates: the `need` best by (score desc, token asc) are admitted
  auto cand_at = [&](int i) -> unsigned long long {
    const int j = owner(pre_cand, i);
    return stage_u[(size_t)j * s.tokC + s.tokC - 1 - (i - pre_cand[j])];
  };
  if (need > 0) {
    if (n_cand <= kCandLds) {
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
      if (i < n_cand) c = (n_cand <= kCandLds) ? comp[i] : cand_at(i);
      const int flag = (i < n_cand && c >= thr) ? 1 : 0;
      int tot;
      const int pos = block_exclusive_scan<NT>(flag, &tot, scan_sm);
      if (flag && carry + pos < need) out[s.I + n_sel + carry + pos] = composite_token(c);
      carry += tot;
    }
  }

  if constexpr (ATTN) {
    __syncthreads();  // this workgroup's index writes are visible to all its threads
    const int b = u / s.Hkv, g = u % s.Hkv;
    const int w = tid >> 6;
    float qr[G][8];
    load_query<T, G>(q + ((size_t)b * s.Hq + (size_t)g * G) * kD, s.scale_log2e, qr);
    AttnState<G> st;
    st.init();
    // rows attended here: initial window, admitted candidates, local window
    const int n_rows = s.I + need + s.L;
    auto row_at = [&](int p) -> int { return out[p < s.I ? p : p + n_sel]; };
    constexpr int R = 2;
    attend_rows<T, G, R>(kc + (size_t)u * s.N * kD, vc + (size_t)u * s.N * kD, s.N, row_at, n_rows, w * 4 * R,
                         NW * 4 * R, qr, st);
    stash_wave_state<T, G, NW>(st, red);
    __syncthreads();
    const float* parts = ws.partials + (size_t)u * s.npart * G * (kD + 2);
    for (int o = tid; o < G * kD; o += NT) {
      const int h = o / kD, d = o % kD;
      float m, l, acc;
      combine_waves<G, NW>(red, h, d, m, l, acc);
      for (int j = 0; j < s.nblkC; ++j) {
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
