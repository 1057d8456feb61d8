// PQ construction on the GPU (paper, Section 2.2 "index construction" and Section 3.1
// step 2): per (sequence, KV head, partition) Lloyd K-Means over the keys' sub-vectors,
// and the nearest-centroid code of a token that leaves the local window (Section 3.1,
// last paragraph; Algorithm 2 "PQArgNearest").
//
// Grid layout: blockIdx.y = unit * M + partition j, blockIdx.x = token chunk.
// Distances are evaluated in fp32 as sum_e (x_e - c_e)^2, e ascending; the lowest
// centroid index wins ties.  Centroid sums are accumulated in 64-bit fixed point
// (2^-20 resolution), which makes the update independent of summation order and
// therefore reproducible; an empty cluster keeps its centroid.
#pragma once
#include "pqc_device.h"

namespace pqc {

constexpr int kFixShift = 20;
constexpr int kAssignTok = 256;   // tokens per workgroup of the assignment kernel

struct BuildShape {
  int units, N, M, C, Dm;
  int cap;  // tokens the key and code tensors hold per unit (>= N): their stride between units
};

// centroids[u][j][c][:] = keys[u][init_idx[u][j][c]][j*Dm : (j+1)*Dm]
template <typename T>
__global__ __launch_bounds__(256) void pq_init_kernel(BuildShape s, const T* __restrict__ keys,
                                                      const int* __restrict__ init_idx, float* __restrict__ cent) {
  const int uj = blockIdx.y, u = uj / s.M, j = uj % s.M;
  for (int i = threadIdx.x; i < s.C * s.Dm; i += 256) {
    const int c = i / s.Dm, e = i % s.Dm;
    int t = init_idx[(size_t)uj * s.C + c];
    t = max(0, min(s.N - 1, t));
    cent[(size_t)uj * s.C * s.Dm + i] = load_as_float<T>(keys, ((size_t)u * s.cap + t) * kD + j * s.Dm + e);
  }
}

// codes[u][t][j] = argmin_c || keys[u][t][j*Dm..] - cent[u][j][c] ||^2
// One thread per token; centroids staged through LDS 32 at a time.
template <typename T, int DM>
__global__ __launch_bounds__(256) void pq_assign_kernel(BuildShape s, const T* __restrict__ keys, int64_t key_unit_stride,
                                                        int n_tokens, int code_pos0, const float* __restrict__ cent,
                                                        uint8_t* __restrict__ codes) {
  constexpr int CG = 32;
  __shared__ float cs[CG * DM];
  const int uj = blockIdx.y, u = uj / s.M, j = uj % s.M;
  const int t = blockIdx.x * kAssignTok + threadIdx.x;
  const bool live = t < n_tokens;
  float x[DM];
  if (live) {
#pragma unroll
    for (int e = 0; e < DM; ++e) x[e] = load_as_float<T>(keys, (size_t)u * key_unit_stride + (size_t)t * kD + j * DM + e);
  } else {
#pragma unroll
    for (int e = 0; e < DM; ++e) x[e] = 0.0f;
  }
  float best = INFINITY;
  int arg = 0;
  for (int c0 = 0; c0 < s.C; c0 += CG) {
    const int nc = min(CG, s.C - c0);
    __syncthreads();
    for (int i = threadIdx.x; i < nc * DM; i += 256) cs[i] = cent[((size_t)uj * s.C + c0) * DM + i];
    __syncthreads();
    for (int c = 0; c < nc; ++c) {
      float d2 = 0.0f;
#pragma unroll
      for (int e = 0; e < DM; ++e) {
        const float df = x[e] - cs[c * DM + e];
        d2 = fmaf(df, df, d2);
      }
      if (d2 < best) {
        best = d2;
        arg = c0 + c;
      }
    }
  }
  if (live) codes[((size_t)u * s.cap + code_pos0 + t) * s.M + j] = (uint8_t)arg;
}

// One token per unit (the code of an appended token): one thread per centroid, the same distance chain
// as pq_assign_kernel, the smallest (distance, centroid) pair through a 64-bit LDS minimum.
template <typename T>
__global__ __launch_bounds__(256) void pq_encode_kernel(BuildShape s, const T* __restrict__ key /* [units][kD] */, int position,
                                                        const float* __restrict__ cent, uint8_t* __restrict__ codes) {
  __shared__ float x[kD];
  __shared__ unsigned long long best;
  const int uj = blockIdx.x, u = uj / s.M, j = uj % s.M, c = threadIdx.x;
  if (c < s.Dm) x[c] = load_as_float<T>(key, (size_t)u * kD + j * s.Dm + c);
  if (c == 0) best = ~0ull;
  __syncthreads();
  if (c < s.C) {
    const float* cr = cent + ((size_t)uj * s.C + c) * s.Dm;
    float d2 = 0.0f;
    for (int e = 0; e < s.Dm; e += 4) {  // Dm is a multiple of 4
      const float4 cv = *reinterpret_cast<const float4*>(cr + e);
      float df = x[e] - cv.x;
      d2 = fmaf(df, df, d2);
      df = x[e + 1] - cv.y;
      d2 = fmaf(df, df, d2);
      df = x[e + 2] - cv.z;
      d2 = fmaf(df, df, d2);
      df = x[e + 3] - cv.w;
      d2 = fmaf(df, df, d2);
    }
    atomicMin(&best, ((unsigned long long)__float_as_uint(d2) << 32) | (unsigned)c);  // d2 >= 0: its bits order like its value
  }
  __syncthreads();
  if (c == 0) codes[((size_t)u * s.cap + position) * s.M + j] = (uint8_t)(best & 0xffu);
}

// The same assignment on the matrix cores, for bf16 keys and sub-vectors of 32, 64 or 128
// dimensions: this step is a dense contraction (tokens x dimensions by dimensions x
// centroids).  The nearest centroid minimises |c|^2 - 2 x.c.  Keys are bf16 already; an fp32
// centroid is split into three bf16 terms that add up to it exactly, so the products are
// exact and only the fp32 accumulation rounds.  Per wave: 16-token tiles as the A operand
// (kept in registers), 16-centroid tiles as the B operand (from LDS), D[token][centroid];
// each lane keeps the best centroid of its column per token, the columns are merged with DPP
// row operations at the end (equal values: lower centroid index).
constexpr int kAssignTiles = 8;                          // 16-token tiles per wave and batch
constexpr int kAssignBatchTok = 4 * 16 * kAssignTiles;   // tokens per workgroup and batch
constexpr int kAssignBatches = 4;                        // batches per workgroup (the staged centroids are reused)
constexpr int kAssignMfmaTok = kAssignBatchTok * kAssignBatches;
template <int DM>
__global__ __launch_bounds__(256) void pq_assign_mfma_kernel(BuildShape s, const bf16_t* __restrict__ keys,
                                                             int64_t key_unit_stride, int n_tokens, int code_pos0,
                                                             const float* __restrict__ cent, uint8_t* __restrict__ codes) {
  constexpr int KK = DM / 32;            // k steps of 32 dimensions
  constexpr int CG = 8192 / DM;          // centroids staged at a time (48 KB of bf16 terms)
  constexpr int RS = DM + 8;             // LDS row stride in bf16 (16 bytes of padding)
  __shared__ __attribute__((aligned(16))) unsigned short ct[3][CG * RS];  // hi, mid, lo terms
  __shared__ float cn[CG];
  const int uj = blockIdx.y, u = uj / s.M, j = uj % s.M, tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6, col = lane & 15, quad = lane >> 4;
  const bool one_group = s.C <= CG;  // then the centroids are staged once for all batches
  for (int batch = 0; batch < kAssignBatches; ++batch) {
    const int tok0 = (blockIdx.x * kAssignBatches + batch) * kAssignBatchTok + w * 16 * kAssignTiles;
    if (blockIdx.x * kAssignMfmaTok + batch * kAssignBatchTok >= n_tokens) break;  // workgroup-uniform
    // this wave's keys: tile tt, row col, dims 32*kk + 8*quad .. +7
    bf16x8_t a[kAssignTiles][KK];
#pragma unroll
    for (int tt = 0; tt < kAssignTiles; ++tt) {
      const int t = min(tok0 + tt * 16 + col, n_tokens - 1);
      const uint4* kp =
          reinterpret_cast<const uint4*>(keys + (size_t)u * key_unit_stride + (size_t)t * kD + j * DM + 8 * quad);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const uint4 raw = kp[4 * kk];
        __builtin_memcpy(&a[tt][kk], &raw, 16);
      }
    }
    float best[kAssignTiles][4];
    int bidx[kAssignTiles][4];
#pragma unroll
    for (int tt = 0; tt < kAssignTiles; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        best[tt][i] = INFINITY;
        bidx[tt][i] = 0;
      }
    for (int c0 = 0; c0 < s.C; c0 += CG) {
      const int nc = min(CG, s.C - c0);
      if (!(one_group && batch > 0)) {
        __syncthreads();
        // stage: split every centroid value into three bf16 terms that add up to it exactly
        for (int i = tid; i < nc * DM; i += 256) {
          const float v = cent[((size_t)uj * s.C + c0) * DM + i];
          const unsigned h = bf16_round_bits(v);
          const float r1 = v - __uint_as_float(h << 16);
          const unsigned m = bf16_round_bits(r1);
          const float r2 = r1 - __uint_as_float(m << 16);
          const unsigned l = bf16_round_bits(r2);
          const int o = (i / DM) * RS + (i % DM);
          ct[0][o] = (unsigned short)h;
          ct[1][o] = (unsigned short)m;
          ct[2][o] = (unsigned short)l;
        }
        // squared norms: four threads per centroid, a quarter of the dimensions each
        for (int cb = 0; cb < nc; cb += 64) {
          const int c = cb + (tid >> 2), seg = tid & 3;
          const float4* cr = reinterpret_cast<const float4*>(cent + ((size_t)uj * s.C + c0 + min(c, nc - 1)) * DM + seg * (DM / 4));
          float n2 = 0.0f;
#pragma unroll
          for (int e = 0; e < DM / 16; ++e) {
            const float4 v = cr[e];
            n2 = fmaf(v.x, v.x, n2);
            n2 = fmaf(v.y, v.y, n2);
            n2 = fmaf(v.z, v.z, n2);
            n2 = fmaf(v.w, v.w, n2);
          }
          n2 += dpp_f<0xB1>(0.0f, n2);
          n2 += dpp_f<0x4E>(0.0f, n2);
          if (seg == 0 && c < nc) cn[c] = n2;
        }
        __syncthreads();
      }
      for (int nt = 0; nt * 16 < nc; ++nt) {
        const int c = nt * 16 + col;  // this lane's centroid column
        const bool live = c < nc;
        bf16x8_t b[3][KK];
#pragma unroll
        for (int term = 0; term < 3; ++term)
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) {
            const uint4 raw = *reinterpret_cast<const uint4*>(&ct[term][min(c, nc - 1) * RS + 32 * kk + 8 * quad]);
            __builtin_memcpy(&b[term][kk], &raw, 16);
          }
        const float cnv = live ? cn[c] : INFINITY;
#pragma unroll
        for (int tt = 0; tt < kAssignTiles; ++tt) {
          f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int term = 2; term >= 0; --term)  // small terms first
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tt][kk], b[term][kk], acc, 0, 0, 0);
#pragma unroll
          for (int i = 0; i < 4; ++i) {  // token 4*quad + i of the tile against centroid c
            const float sc = fmaf(-2.0f, acc[i], cnv);
            if (sc < best[tt][i]) {  // strict: an earlier (lower) centroid of this lane keeps a tie
              best[tt][i] = sc;
              bidx[tt][i] = c0 + c;
            }
          }
        }
      }
    }
    // merge the 16 columns of a row of lanes; equal values: lower centroid index
#pragma unroll
    for (int tt = 0; tt < kAssignTiles; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float v = best[tt][i];
        int x = bidx[tt][i];
        auto take = [&](float ov, int ox) {
          const bool t = ov < v || (ov == v && ox < x);
          v = t ? ov : v;
          x = t ? ox : x;
        };
        take(dpp_f<0xB1>(v, v), dpp_i<0xB1>(x, x));
        take(dpp_f<0x4E>(v, v), dpp_i<0x4E>(x, x));
        take(dpp_f<0x141>(v, v), dpp_i<0x141>(x, x));
        take(dpp_f<0x140>(v, v), dpp_i<0x140>(x, x));
        const int t = tok0 + tt * 16 + 4 * quad + i;
        if (col == 0 && t < n_tokens) codes[((size_t)u * s.cap + code_pos0 + t) * s.M + j] = (uint8_t)x;
      }
  }
}

__global__ void pq_zero_kernel(unsigned long long* p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

// sums[u][j][c][e] += fix(keys[u][t][j*Dm+e]) for every token t with code c; counts[u][j][c] += 1.
// A workgroup first sorts its tokens by code (a counting sort in LDS: one 32-bit atomic per token), then each wave
// takes centroids in turn and sums the centroid's members in registers: a lane loads 16 bytes of a member's
// sub-vector (8 bf16 or 4 fp32 values), a group of Dm*sizeof(T)/16 lanes covers one member and a wave several
// members per load; the lane groups' partial sums meet in a wave-private LDS tile.  (Adding every value to an LDS
// accumulator with an atomic, as a first version did, is bound by the LDS atomic rate of about one lane per clock.)
// Sums are 64-bit integers of the values in fixed point (2^-20), so the result does not depend on the order of
// the members, of the waves or of the workgroups.
__host__ __device__ constexpr int accum_tokens_per_wg(int C) { return 32 * C < 2048 ? 2048 : (32 * C > 8192 ? 8192 : 32 * C); }
template <typename T, int DM>
__global__ __launch_bounds__(256) void pq_accum_kernel(BuildShape s, const T* __restrict__ keys,
                                                       const uint8_t* __restrict__ codes,
                                                       unsigned long long* __restrict__ sums,
                                                       unsigned* __restrict__ counts) {
  constexpr int EPV = 16 / (int)sizeof(T);  // values per lane
  constexpr int LPT = DM / EPV;             // lanes per member
  constexpr int MPW = 64 / LPT;             // members a wave loads at a time
  constexpr int U = 4;                      // such loads in flight
  constexpr int NW = 4;
  static_assert(DM % EPV == 0 && LPT >= 1 && LPT <= 64, "a sub-vector is a whole number of 16-byte pieces");
  extern __shared__ unsigned short order[];  // [tokens per workgroup] token offsets, sorted by code
  __shared__ unsigned cnt[256];
  __shared__ int start[257];
  __shared__ int scan_sm[2 * NW + 1];
  __shared__ long long part[NW][MPW * DM];   // per wave: [member slot][dimension]
  const int uj = blockIdx.y, u = uj / s.M, j = uj % s.M, tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6, sub = lane % LPT, slot = lane / LPT;
  const int tpw = accum_tokens_per_wg(s.C);
  const int t0 = blockIdx.x * tpw, nt = min(tpw, s.N - t0);
  const uint8_t* cp = codes + ((size_t)u * s.cap + t0) * s.M + j;
  // ---- counting sort of the workgroup's tokens by code
  cnt[tid] = 0u;
  __syncthreads();
  for (int t = tid; t < nt; t += 256) {
    const unsigned c = cp[(size_t)t * s.M];
    if (c < (unsigned)s.C) atomicAdd(&cnt[c], 1u);  // (a code that names no centroid is left out)
  }
  __syncthreads();
  {
    const int mine = (int)cnt[tid];
    int total;
    const int ex = block_exclusive_scan<256>(mine, &total, scan_sm);
    start[tid] = ex;
    if (tid == 255) start[256] = total;
    cnt[tid] = (unsigned)ex;  // now the bucket's fill position
  }
  __syncthreads();
  for (int t = tid; t < nt; t += 256) {
    const unsigned c = cp[(size_t)t * s.M];
    if (c < (unsigned)s.C) order[atomicAdd(&cnt[c], 1u)] = (unsigned short)t;
  }
  __syncthreads();
  // ---- one centroid at a time per wave
  const T* kbase = keys + ((size_t)u * s.cap + t0) * kD + j * DM + sub * EPV;
  long long* mypart = part[w];
  for (int c = w; c < s.C; c += NW) {
    const int base = start[c], n = start[c + 1] - base;  // wave-uniform
    if (n == 0) continue;
    long long acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = 0;
    for (int m0 = 0; m0 < n; m0 += MPW * U) {
      uint4 raw[U];
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const int t = order[base + min(m0 + k * MPW + slot, n - 1)];  // clamped: straight-line loads, masked below
        raw[k] = *reinterpret_cast<const uint4*>(kbase + (size_t)t * kD);
      }
#pragma unroll
      for (int k = 0; k < U; ++k) {
        if (m0 + k * MPW + slot < n) {
          const unsigned rw[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
          float x[EPV];
          if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              x[2 * e] = __uint_as_float(rw[e] << 16);
              x[2 * e + 1] = __uint_as_float(rw[e] & 0xffff0000u);
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = __uint_as_float(rw[e]);
          }
#pragma unroll
          for (int e = 0; e < EPV; ++e) {
            const float xs = x[e] * (float)(1 << kFixShift);
            // the usual case in 32-bit arithmetic (a 64-bit conversion is a long instruction sequence)
            long long fx = (long long)__float2int_rn(xs);
            if (__builtin_expect(!(fabsf(xs) < 2147483520.0f), 0)) fx = __float2ll_rn(xs);  // |x| >= 2048, or not a number
            acc[e] += fx;
          }
        }
      }
    }
    // the lane groups' sums meet in the wave's tile; then one lane per dimension adds them up
#pragma unroll
    for (int e = 0; e < EPV; ++e) mypart[slot * DM + sub * EPV + e] = acc[e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int used = min(MPW, n);  // slots beyond the members hold zeros; skipping them is only quicker
    for (int d = lane; d < DM; d += 64) {
      long long tot = 0;
      for (int sl = 0; sl < used; ++sl) tot += mypart[sl * DM + d];
      if (tot) atomicAdd(&sums[((size_t)uj * s.C + c) * DM + d], (unsigned long long)tot);
    }
    if (lane == 0) atomicAdd(&counts[(size_t)uj * s.C + c], (unsigned)n);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// cent = sums / counts where counts > 0
__global__ __launch_bounds__(256) void pq_mean_kernel(BuildShape s, const unsigned long long* __restrict__ sums,
                                                      const unsigned* __restrict__ counts, float* __restrict__ cent) {
  const size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  const size_t n = (size_t)s.units * s.M * s.C * s.Dm;
  if (i >= n) return;
  const unsigned k = counts[i / s.Dm];
  if (k) cent[i] = (float)((double)(long long)sums[i] * (1.0 / (double)(1 << kFixShift)) / (double)k);
}

// ------------------------------------------------------------ block statistics
// Section 3.4: the block-level cache is refreshed with the k_cache blocks that hold the
// most retrieved tokens.  One workgroup per unit: counts per block (global atomics, read
// back through the L2 with returning atomics), a histogram of the count values (a count
// never exceeds the block size when the listed tokens are distinct), the cut c* and the
// number of blocks to admit at the cut, then the blocks in the order in which the cache
// refresh serves them: fullest first, the lower block number first among equal counts.  A
// block's place is (blocks with a larger count) + (blocks before it with the same count);
// the second term comes from a counter per count value that the waves of a chunk of 1024
// blocks advance one after the other, lanes with equal counts being ranked inside a wave
// by ballots.
constexpr int kCountBins = 2048;
__global__ __launch_bounds__(1024) void block_stats_kernel(const int* __restrict__ idx, long long n_idx, int N, int bt,
                                                           int nb, int k_cache, int* __restrict__ counts,
                                                           int* __restrict__ blocks) {
  constexpr int NT = 1024, NW = NT / 64;
  __shared__ unsigned hist[kCountBins];
  __shared__ int above[kCountBins];  // blocks with a larger count
  __shared__ int run[kCountBins];    // blocks with this count placed so far
  __shared__ int scan_sm[2 * NW + 1];
  __shared__ int res[2];
  __shared__ int any_sm;
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int* cu = counts + (size_t)u * nb;
  for (int i = tid; i < nb; i += NT) cu[i] = 0;
  for (int i = tid; i < kCountBins; i += NT) {
    hist[i] = 0u;
    run[i] = 0;
  }
  if (tid == 0) {
    res[0] = kCountBins;  // cut (no block reaches it when k_cache == 0)
    res[1] = 0;           // blocks above the cut
  }
  __threadfence();
  __syncthreads();
  const int* lst = idx + (size_t)u * n_idx;
  for (long long i = tid; i < n_idx; i += NT) {
    const int t = lst[i];
    if (t >= 0 && t < N) atomicAdd(&cu[t / bt], 1);
  }
  __threadfence();
  __syncthreads();
  for (int i = tid; i < nb; i += NT) atomicAdd(&hist[min(atomicAdd(&cu[i], 0), kCountBins - 1)], 1u);
  __syncthreads();
  // thread tid owns count values kCountBins-1-2*tid and kCountBins-2-2*tid (descending)
  const int h0 = (int)hist[kCountBins - 1 - 2 * tid], h1 = (int)hist[kCountBins - 2 - 2 * tid];
  int total;
  int cum = block_exclusive_scan<NT>(h0 + h1, &total, scan_sm);
  above[kCountBins - 1 - 2 * tid] = cum;
  above[kCountBins - 2 - 2 * tid] = cum + h0;
  if (k_cache > 0 && cum < k_cache && cum + h0 >= k_cache) {
    res[0] = kCountBins - 1 - 2 * tid;
    res[1] = cum;
  } else if (k_cache > 0 && cum + h0 < k_cache && cum + h0 + h1 >= k_cache) {
    res[0] = kCountBins - 2 - 2 * tid;
    res[1] = cum + h0;
  }
  __syncthreads();
  const int cut = res[0], n_above = res[1], need = k_cache - n_above;
  int* out = blocks + (size_t)u * k_cache;
  int carry_t = 0;
  for (int i0 = 0; i0 < (k_cache > 0 ? nb : 0); i0 += NT) {
    const int i = i0 + tid;
    const int c = i < nb ? min(atomicAdd(&cu[i], 0), kCountBins - 1) : -1;
    const bool a = c > cut;
    // blocks at the cut: the lowest-numbered `need` of them, behind all blocks above the cut
    int tt;
    const int pt = block_exclusive_scan<NT>(c == cut ? 1 : 0, &tt, scan_sm);
    if (c == cut && carry_t + pt < need) out[n_above + carry_t + pt] = i;
    carry_t += tt;
    // blocks above the cut (chunks without any skip the ordered part)
    if (tid == 0) any_sm = 0;
    __syncthreads();
    if (a) any_sm = 1;
    __syncthreads();
    if (any_sm) {  // uniform
      // rank among the wave's lanes with the same count (lanes ascend with the block number), one count value per round
      int rank_w = 0, cnt_w = 0;
      bool leader = false;
      unsigned long long todo = __ballot(a);
      while (todo) {  // wave-uniform
        const int src = __ffsll((long long)todo) - 1;
        const int k0 = __shfl(c, src);
        const unsigned long long m = __ballot(a && c == k0);
        if (a && c == k0) {
          rank_w = __popcll(m & ((1ull << lane) - 1ull));
          cnt_w = __popcll(m);
          leader = lane == src;
        }
        todo &= ~m;
      }
      // the waves advance the per-count counters one after the other (a wave's LDS accesses stay in program order:
      // every lane has read the counter before the leader of its count value moves it on)
      int base = 0;
      for (int ww = 0; ww < NW; ++ww) {
        if (w == ww && a) {
          base = run[c];
          if (leader) run[c] = base + cnt_w;
        }
        __syncthreads();
      }
      if (a) out[above[c] + base + rank_w] = i;
    }
  }
}

// ------------------------------------------------------------ block cache refresh
// Section 3.4: the block-level cache is looked up with this step's retrieved tokens, then refreshed
// with the step's requested blocks under an LRU or LFU policy.  One workgroup per unit.  Sequentially,
// each absent block would take the lowest empty slot or else the policy's victim among the slots not
// requested in this step; since the order of those slots (empty ones by index, then by (uses,) last
// use, slot) does not change while the step is served, the i-th absent block simply takes the slot of
// rank i in that order, which is found by counting.
constexpr int kCacheSlots = 1024;  // most slots, and most requested blocks, per unit
__global__ __launch_bounds__(256) void block_cache_kernel(int nb, int n_slots, int k_cache, int lfu, int step,
                                                          const int* __restrict__ counts, const int* __restrict__ blocks,
                                                          int* __restrict__ slot_block, int* __restrict__ slot_stamp,
                                                          int* __restrict__ slot_uses, int* __restrict__ stats) {
  constexpr int NT = 256, NW = NT / 64;
  __shared__ int blk[kCacheSlots], stamp[kCacheSlots], uses[kCacheSlots];
  __shared__ int req[kCacheSlots], req_slot[kCacheSlots], miss_rank[kCacheSlots];
  __shared__ int by_rank[kCacheSlots];                 // slot of rank r among the slots not requested in this step
  __shared__ unsigned long long key[kCacheSlots];      // ordering key of a slot; ~0 = requested in this step
  __shared__ int scan_sm[2 * NW + 1];
  __shared__ int red[4];
  const int u = blockIdx.x, tid = threadIdx.x;
  int* sb = slot_block + (size_t)u * n_slots;
  int* ss = slot_stamp + (size_t)u * n_slots;
  int* su = slot_uses + (size_t)u * n_slots;
  const int* cu = counts + (size_t)u * nb;
  if (tid < 4) red[tid] = 0;
  for (int s = tid; s < n_slots; s += NT) {
    blk[s] = sb[s];
    stamp[s] = ss[s];
    uses[s] = su[s];
  }
  for (int i = tid; i < k_cache; i += NT) req[i] = blocks[(size_t)u * k_cache + i];
  __syncthreads();
  // look-up against the cache as it stands: retrieved tokens inside resident blocks
  int ht = 0;
  for (int s = tid; s < n_slots; s += NT)
    if (blk[s] >= 0 && blk[s] < nb) ht += cu[blk[s]];
  if (ht) atomicAdd(&red[0], ht);
  // requested blocks that are resident: mark them used
  int hb = 0;
  for (int i = tid; i < k_cache; i += NT) {
    int found = -1;
    for (int s = 0; s < n_slots; ++s) found = blk[s] == req[i] ? s : found;
    if (req[i] < 0 || req[i] >= nb) found = -2;  // not a block: neither a hit nor a request
    req_slot[i] = found;
    hb += found >= 0;
  }
  if (hb) atomicAdd(&red[1], hb);
  __syncthreads();
  for (int s = tid; s < n_slots; s += NT) {
    const unsigned long long st = (unsigned)stamp[s] ^ 0x80000000u;  // signed order as unsigned order
    const unsigned long long k1 = lfu ? ((unsigned long long)(unsigned)uses[s] << 32) | st : st;
    key[s] = blk[s] < 0 ? 0ull : (1ull << 63) | k1;
  }
  __syncthreads();
  for (int i = tid; i < k_cache; i += NT) {
    const int s = req_slot[i];
    if (s >= 0) {
      key[s] = ~0ull;
      stamp[s] = step;
      atomicAdd(&uses[s], 1);
    }
  }
  __syncthreads();
  // rank of every other slot in victim order
  int n_free_local = 0;
  for (int s = tid; s < n_slots; s += NT) {
    const unsigned long long ks = key[s];
    if (ks == ~0ull) continue;
    int r = 0;
    for (int t = 0; t < n_slots; ++t) {
      const unsigned long long kt = key[t];
      r += (kt != ~0ull) && (kt < ks || (kt == ks && t < s));
    }
    by_rank[r] = s;
    ++n_free_local;
  }
  if (n_free_local) atomicAdd(&red[2], n_free_local);
  // absent requests, numbered in request order
  int carry = 0;
  for (int i0 = 0; i0 < k_cache; i0 += NT) {
    const int i = i0 + tid;
    const int miss = i < k_cache && req_slot[i] == -1;
    int total;
    const int pos = block_exclusive_scan<NT>(miss, &total, scan_sm);
    if (i < k_cache) miss_rank[i] = miss ? carry + pos : -1;
    carry += total;
  }
  __syncthreads();
  const int n_free = red[2], n_ins = min(carry, n_free);
  int evicted = 0;
  for (int i = tid; i < k_cache; i += NT) {
    const int r = miss_rank[i];
    if (r >= 0 && r < n_ins) {
      const int s = by_rank[r];
      evicted += blk[s] >= 0;
      blk[s] = req[i];
      stamp[s] = step;
      uses[s] = 1;
    }
  }
  if (evicted) atomicAdd(&red[3], evicted);
  __syncthreads();
  for (int s = tid; s < n_slots; s += NT) {
    sb[s] = blk[s];
    ss[s] = stamp[s];
    su[s] = uses[s];
  }
  if (tid == 0) {
    int* o = stats + (size_t)u * 4;
    o[0] = red[0];
    o[1] = red[1];
    o[2] = n_ins;
    o[3] = red[3];
  }
}

// -------------------------------------------------------------- code-pair counts
// M = 2: how many tokens of a unit carry each pair of codes (c0 + C*c1), over all N tokens.
// A statistic of the codes alone; pqc_decode_indexed takes its threshold from it.
constexpr int kPairTok = 8192;  // tokens per workgroup
__global__ __launch_bounds__(256) void pair_count_kernel(const uint8_t* __restrict__ codes, int N, int cap, int C,
                                                         unsigned* __restrict__ counts) {
  __shared__ unsigned h[4096];
  const int u = blockIdx.y, tid = threadIdx.x, np = C * C;
  for (int i = tid; i < np; i += 256) h[i] = 0u;
  __syncthreads();
  const unsigned short* cu = reinterpret_cast<const unsigned short*>(codes) + (size_t)u * cap;
  const int t1 = min(N, ((int)blockIdx.x + 1) * kPairTok);
  for (int t = blockIdx.x * kPairTok + tid; t < t1; t += 256) {
    const unsigned cw = cu[t];
    const int c0 = (int)(cw & 0xffu), c1 = (int)(cw >> 8);
    if (c0 < C && c1 < C) atomicAdd(&h[c0 + C * c1], 1u);  // a code outside [0, C) names no pair: not counted
  }
  __syncthreads();
  for (int i = tid; i < np; i += 256)
    if (h[i]) atomicAdd(&counts[(size_t)u * np + i], h[i]);
}

// one appended token per unit: its pair gains a token
__global__ void pair_count_add_kernel(const uint8_t* __restrict__ codes, int cap, int C, int units, int position,
                                      unsigned* __restrict__ counts) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= units) return;
  const uint8_t* cp = codes + ((size_t)u * cap + position) * 2;
  const int c0 = (int)cp[0], c1 = (int)cp[1];
  if (c0 < C && c1 < C) counts[(size_t)u * C * C + c0 + C * c1] += 1u;
}

}  // namespace pqc
