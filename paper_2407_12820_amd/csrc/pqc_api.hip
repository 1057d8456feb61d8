// Host side of libpqcache: the C ABI of include/pqcache.h, configuration checks,
// workspace carving and kernel dispatch.  No device memory is allocated here and
// nothing synchronises the host: every entry point only enqueues kernels.
#include "../../include/pqcache.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "pqc_build_kernels.h"
#include "pqc_kernels.h"

namespace {

using namespace pqc;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Plan {
  Shape s;
  size_t off_ctl, off_lut, off_range, off_hist, off_bins, off_crec, off_stage, off_cnt, off_part, off_trace, total;
  int rec_stride;
};

// Launch-shape overrides from the environment, for sweeps: debug builds (-DPQC_TRACE) only.  The shipped library
// reads no environment variable.
int env_int(const char* name, int fallback) {
#ifdef PQC_TRACE
  const char* v = std::getenv(name);
  if (!v || !*v) return fallback;
  const int x = std::atoi(v);
  return x > 0 ? x : fallback;
#else
  (void)name;
  return fallback;
#endif
}

// Offsets of the workspace regions for the given per-unit sizes.
void lay_out(Plan* p, size_t bins_per_unit, size_t stage_words_per_unit, size_t counts_per_unit, size_t partials_per_unit) {
  const Shape& s = p->s;
  const size_t units = (size_t)s.B * s.Hkv;
  size_t off = 0;
  p->off_ctl = off;   off = align_up(off + sizeof(BinParams) * units);
  p->off_lut = off;   off = align_up(off + sizeof(float) * units * s.M * s.C);
  p->off_range = off; off = align_up(off + sizeof(float2) * units);
  p->off_hist = off;  off = align_up(off + sizeof(unsigned) * units * (kHistCopies * kNB + 1));  // + record counters
  p->off_bins = off;  off = align_up(off + sizeof(unsigned short) * units * bins_per_unit);
  p->off_crec = off;  off = align_up(off + (size_t)p->rec_stride * units);
  p->off_stage = off; off = align_up(off + sizeof(unsigned long long) * units * stage_words_per_unit);
  p->off_cnt = off;   off = align_up(off + sizeof(int2) * units * counts_per_unit);
  p->off_part = off;  off = align_up(off + sizeof(float) * units * partials_per_unit * s.G * (kD + 2));
#ifdef PQC_TRACE
  p->off_trace = off; off = align_up(off + sizeof(unsigned long long) * 3 * kTraceWgs * kTraceSlots);
#endif
  p->total = off;
}

int make_plan(const pqc_config* c, Plan* p) {
  if (!c) return PQC_EINVAL;
  if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 || c->n_tokens < 1 || c->pq_m < 1 ||
      c->pq_centroids < 1 || c->topk < 0 || c->n_init < 0 || c->n_local < 0)
    return PQC_EINVAL;
  if (c->n_q_heads % c->n_kv_heads || c->head_dim % c->pq_m) return PQC_EINVAL;
  if ((long long)c->n_init + c->topk + c->n_local > c->n_tokens || c->n_init + c->topk + c->n_local < 1) return PQC_EINVAL;
  if (c->kv_dtype != PQC_F32 && c->kv_dtype != PQC_BF16) return PQC_EINVAL;
  if (!(c->softmax_scale == c->softmax_scale) || std::isinf(c->softmax_scale)) return PQC_EINVAL;
  const int G = c->n_q_heads / c->n_kv_heads;
  if (c->head_dim != kD) return PQC_EUNSUPPORTED;
  if (c->pq_m != 1 && c->pq_m != 2 && c->pq_m != 4 && c->pq_m != 8) return PQC_EUNSUPPORTED;
  if (c->pq_centroids > 256) return PQC_EUNSUPPORTED;
  if (G != 1 && G != 2 && G != 4 && G != 8) return PQC_EUNSUPPORTED;
  if (c->n_capacity < 0 || (c->n_capacity && c->n_capacity < c->n_tokens)) return PQC_EINVAL;
  if (c->n_tokens > (1 << 22) || c->n_capacity > (1 << 22)) return PQC_EUNSUPPORTED;
  if ((long long)c->batch * c->n_kv_heads > 65535) return PQC_EUNSUPPORTED;

  Shape& s = p->s;
  s.B = c->batch; s.Hq = c->n_q_heads; s.Hkv = c->n_kv_heads; s.G = G; s.N = c->n_tokens;
  s.cap = c->n_capacity ? c->n_capacity : c->n_tokens;
  s.M = c->pq_m; s.C = c->pq_centroids; s.Dm = c->head_dim / c->pq_m;
  s.K = c->topk; s.I = c->n_init; s.L = c->n_local; s.Ktot = s.I + s.K + s.L;
  const float scale = c->softmax_scale > 0.0f ? c->softmax_scale : 1.0f / std::sqrt((float)c->head_dim);
  s.scale_log2e = scale * 1.4426950408889634f;
  const long long units = (long long)s.B * s.Hkv;

  // A unit's codes start at byte u*cap*M; when that is not always 16-byte aligned the first
  // chunk of a unit begins with up to 15 phantom tokens that the grids must cover as well.
  const int lead = ((long long)s.cap * s.M) % 16 == 0 ? 0 : 15;
  // histogram kernel: about one 1024-thread workgroup per compute unit over all units
  const int maxA = 4096 * (16 / s.M) < 16384 ? 4096 * (16 / s.M) : 16384;  // kMaxVecA chunks per thread
  int tokA = env_int("PQC_TOK_A", 0);
  if (!tokA) {
    // every workgroup builds the unit's whole table first, so few, large workgroups: 4096 tokens measured best
    // from 32K to 128K tokens per unit (at 32K: 27.6 us per step against 28.3 with 1024)
    tokA = 4096;
    while (tokA < maxA && units * ((s.N + lead + tokA - 1) / tokA) > 320) tokA *= 2;
  }
  if (tokA % 1024 || tokA > maxA) return PQC_EINVAL;
  s.tokA = tokA; s.nblkA = (s.N + lead + tokA - 1) / tokA;
  s.histCopies = s.nblkA <= 32 ? 1 : s.nblkA <= 64 ? 2 : kHistCopies;
  // select kernel: 256-thread workgroups, two resident per compute unit
  int tokC = env_int("PQC_TOK_C", 0);
  if (!tokC) {
    tokC = 512;
    while (tokC < 8192 && units * ((s.N + tokC - 1) / tokC) > 512) tokC *= 2;
  }
  if (tokC != 512 && tokC != 1024 && tokC != 2048 && tokC != 4096 && tokC != 8192) return PQC_EINVAL;
  s.tokC = tokC; s.nblkC = (s.N + tokC - 1) / tokC;
  s.binStride = s.nblkC * s.tokC;
  s.stageStride = s.tokC + 40;
  s.rowsP = env_int("PQC_ROWS_P", 256);
  s.nblkP = (s.Ktot + s.rowsP - 1) / s.rowsP;
  s.npart = s.nblkC > s.nblkP ? s.nblkC : s.nblkP;
  p->rec_stride = (int)cand_unit_bytes(G, c->kv_dtype == PQC_F32 ? 4 : 2);
  // finalize kernel: as many workgroups per query head (each with its share of the output dimensions) as keep the
  // grid within about two workgroups per compute unit
  s.slices = 1;
  while (s.slices < kMaxSlices && units * (2 * s.slices * G + kCopyWgs) <= 512) s.slices *= 2;
  // sample ranks that bracket the K-th largest score by 5 standard errors (+2)
  const int nmid = s.N - s.I - s.L;
  s.sampleN = nmid < 1024 ? (nmid > 0 ? nmid : 1) : 1024;
  {
    const double pr = nmid > 0 ? (double)s.K / (double)nmid : 0.0;
    const double centre = pr * s.sampleN, hw = 5.0 * std::sqrt(s.sampleN * pr * (1.0 - pr)) + 2.0;
    s.rankHi = (int)std::floor(centre - hw);                       // < 1: the window reaches the upper bound
    s.rankLo = (int)std::ceil(centre + hw);
    if (s.rankLo > s.sampleN) s.rankLo = 0;                        // 0: the window reaches the lower bound
    if (s.rankHi < 1) s.rankHi = 0;
  }

  lay_out(p, (size_t)s.binStride, (size_t)s.nblkC * s.stageStride, (size_t)s.nblkC, (size_t)s.npart);
  return PQC_OK;
}

// Workspace needed by any context of this configuration whose length is changed later
// (pqc_set_length) to anything up to the capacity: every size that depends on the length,
// replaced by a bound over all lengths.
size_t workspace_bound(const pqc_config* c) {
  Plan p;
  if (make_plan(c, &p) != PQC_OK) return 0;
  const Shape& s = p.s;
  if (s.cap == s.N) return p.total;
  const size_t units = (size_t)s.B * s.Hkv, cap = (size_t)s.cap;
  // select kernel grid: tokens per workgroup double until the grid has at most 512 workgroups or
  // they reach 8192 (an override by environment may pin them as low as 512)
  const size_t tok_min = env_int("PQC_TOK_C", 0) ? (size_t)env_int("PQC_TOK_C", 0) : 8192;
  size_t nb = 512 / units;
  if (nb < (cap + tok_min - 1) / tok_min) nb = (cap + tok_min - 1) / tok_min;
  if (nb < 1) nb = 1;
  size_t npart = (cap + s.rowsP - 1) / s.rowsP;
  if (npart < nb) npart = nb;
  lay_out(&p, cap + 8192, cap + 8192 + 40 * nb, nb, npart);
  return p.total;
}

}  // namespace

struct pqc_ctx {
  pqc_config cfg;
  Plan plan;
  Workspace ws;
  AppendArgs append;       // set for the duration of a pqc_decode_append call
  char* workspace;         // the caller's device memory
  size_t workspace_bytes;
  bool hist_clean;  // the histogram is known to be all zero
  int next_phase;   // pqc_decode_phase: the phase that continues the step begun on this context (0: none begun)
  int last_hip;
};

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_launch(pqc_ctx* ctx) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    ctx->last_hip = (int)e;
    ctx->hist_clean = false;
    return PQC_EHIP;
  }
  return PQC_OK;
}

// Histograms and record counters must be zero when a call starts; finalize_kernel leaves them
// so, which makes a completed call stateless (and a captured one replayable).
int ensure_clean_hist(pqc_ctx* ctx, hipStream_t st) {
  if (ctx->next_phase != 0) {  // a step begun phase by phase (pqc_decode_phase) was left unfinished: its histogram is stale
    ctx->hist_clean = false;
    ctx->next_phase = 0;
  }
  if (ctx->hist_clean) return PQC_OK;
  const Shape& s = ctx->plan.s;
  const size_t na = (size_t)s.B * s.Hkv * (kHistCopies * kNB + 1);  // histograms and the record counters behind them
  hipLaunchKernelGGL(reset_kernel, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, st, ctx->ws.hist, na);
  return check_launch(ctx);
}

// ---- template dispatch -------------------------------------------------------
// The histogram kernel is compiled for the number of 16-byte loads a thread needs: of the centroids (VW: the
// unit's M*C*Dm floats over 1024 threads) and of the codes or scores (VA: the workgroup's tokA tokens).
template <typename T, class SRC, int VW>
void launch_hist_w(const Shape& s, const Workspace& ws, const T* q, const float* cent, const void* src, size_t lds, hipStream_t st) {
  const dim3 grid(s.nblkA, (unsigned)(s.B * s.Hkv));
  const int chunks = s.tokA / SRC::P, va = (chunks + 1023) / 1024;
  if (va <= 1)
    hipLaunchKernelGGL((hist_kernel<T, SRC, VW, 1>), grid, dim3(1024), lds, st, s, ws, q, cent, src);
  else if (va <= 2)
    hipLaunchKernelGGL((hist_kernel<T, SRC, VW, 2>), grid, dim3(1024), lds, st, s, ws, q, cent, src);
  else
    hipLaunchKernelGGL((hist_kernel<T, SRC, VW, 4>), grid, dim3(1024), lds, st, s, ws, q, cent, src);
}
template <typename T, class SRC>
void launch_hist(const Shape& s, const Workspace& ws, const T* q, const float* cent, const void* src, size_t lds, hipStream_t st) {
  if constexpr (!SRC::kFromCodes) {
    launch_hist_w<T, SRC, 1>(s, ws, q, cent, src, lds, st);
  } else {
    const int vw = (s.M * s.C * s.Dm + 4095) / 4096;
    if (vw <= 1) launch_hist_w<T, SRC, 1>(s, ws, q, cent, src, lds, st);
    else if (vw <= 2) launch_hist_w<T, SRC, 2>(s, ws, q, cent, src, lds, st);
    else if (vw <= 4) launch_hist_w<T, SRC, 4>(s, ws, q, cent, src, lds, st);
    else launch_hist_w<T, SRC, 8>(s, ws, q, cent, src, lds, st);
  }
}

template <typename T, int G>
void launch_finalize(pqc_ctx* ctx, const T* qt, const T* kt, const T* vt, int32_t* out_idx, float* out_attn, hipStream_t st) {
  const Shape& s = ctx->plan.s;
  const dim3 grid(G * s.slices + kCopyWgs + (ctx->append.key ? 1 : 0), (unsigned)(s.B * s.Hkv));
  // Tokens that share all their codes share a score: with few distinct code words the tie class at the threshold is
  // large (131072 tokens over 64 x 64 code pairs: up to 70 candidates), and the kernel requests more records up front.
  double words = 1.0;
  for (int j = 0; j < s.M; ++j) words *= s.C;
  if (s.slices == kMaxSlices && s.N >= 16.0 * words)
    hipLaunchKernelGGL((finalize_kernel<T, G, true, true>), grid, dim3(256), finalize_lds_bytes(s, true), st, s, ctx->ws, qt, kt, vt,
                       out_idx, out_attn, ctx->append);
  else
    hipLaunchKernelGGL((finalize_kernel<T, G, true, false>), grid, dim3(256), finalize_lds_bytes(s, true), st, s, ctx->ws, qt, kt, vt,
                       out_idx, out_attn, ctx->append);
}

// phases: bit k set = launch kernel k of the decode path (0 histogram, 1 select + attention, 2 finalize)
template <typename T, int G, int M>
void launch_decode_tgm(pqc_ctx* ctx, const void* q, const float* cent, const uint8_t* codes, const void* k,
                       const void* v, int32_t* out_idx, float* out_attn, hipStream_t st, unsigned phases) {
  const Shape& s = ctx->plan.s;
  const unsigned units = (unsigned)(s.B * s.Hkv);
  const T* qt = static_cast<const T*>(q);
  const T* kt = static_cast<const T*>(k);
  const T* vt = static_cast<const T*>(v);
  if (phases & 1u) launch_hist<T, CodeChunks<M>>(s, ctx->ws, qt, cent, static_cast<const void*>(codes), sizeof(float) * lut_tile_floats(1024, M, s.C), st);
  if (phases & 2u)
    hipLaunchKernelGGL((select_kernel<T, G, CodeChunks<M>, true>), dim3(s.nblkC, units), dim3(256),
                       s.tokC * sizeof(unsigned short), st, s, ctx->ws, qt, kt, vt, static_cast<const void*>(codes));
  if (phases & 4u)
    launch_finalize<T, G>(ctx, qt, kt, vt, out_idx, out_attn, st);
}

template <typename T, int G>
void launch_decode_tg(pqc_ctx* ctx, const void* q, const float* cent, const uint8_t* codes, const void* k, const void* v,
                      int32_t* out_idx, float* out_attn, hipStream_t st, unsigned phases) {
  switch (ctx->plan.s.M) {
    case 1: launch_decode_tgm<T, G, 1>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
    case 2: launch_decode_tgm<T, G, 2>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
    case 4: launch_decode_tgm<T, G, 4>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
    default: launch_decode_tgm<T, G, 8>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
  }
}

template <typename T>
void launch_decode_t(pqc_ctx* ctx, const void* q, const float* cent, const uint8_t* codes, const void* k, const void* v,
                     int32_t* out_idx, float* out_attn, hipStream_t st, unsigned phases) {
  switch (ctx->plan.s.G) {
    case 1: launch_decode_tg<T, 1>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
    case 2: launch_decode_tg<T, 2>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
    case 4: launch_decode_tg<T, 4>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
    default: launch_decode_tg<T, 8>(ctx, q, cent, codes, k, v, out_idx, out_attn, st, phases); break;
  }
}

// decode with the threshold taken from code-pair counts (M = 2): select + finalize, no histogram kernel
template <typename T, int G>
void launch_indexed_tg(pqc_ctx* ctx, const void* q, const float* cent, const uint8_t* codes, const unsigned* pair_counts,
                       const void* k, const void* v, int32_t* out_idx, float* out_attn, hipStream_t st) {
  const Shape& s = ctx->plan.s;
  const unsigned units = (unsigned)(s.B * s.Hkv);
  const T* qt = static_cast<const T*>(q);
  const T* kt = static_cast<const T*>(k);
  const T* vt = static_cast<const T*>(v);
  hipLaunchKernelGGL((select_kernel<T, G, CodeChunks<2>, true, true>), dim3(s.nblkC, units), dim3(256),
                     s.tokC * sizeof(unsigned short), st, s, ctx->ws, qt, kt, vt, static_cast<const void*>(codes), cent,
                     pair_counts, ctx->append.key ? ctx->append.position : -1);
  launch_finalize<T, G>(ctx, qt, kt, vt, out_idx, out_attn, st);
}

template <typename T>
void launch_indexed_t(pqc_ctx* ctx, const void* q, const float* cent, const uint8_t* codes, const unsigned* pair_counts,
                      const void* k, const void* v, int32_t* out_idx, float* out_attn, hipStream_t st) {
  switch (ctx->plan.s.G) {
    case 1: launch_indexed_tg<T, 1>(ctx, q, cent, codes, pair_counts, k, v, out_idx, out_attn, st); break;
    case 2: launch_indexed_tg<T, 2>(ctx, q, cent, codes, pair_counts, k, v, out_idx, out_attn, st); break;
    case 4: launch_indexed_tg<T, 4>(ctx, q, cent, codes, pair_counts, k, v, out_idx, out_attn, st); break;
    default: launch_indexed_tg<T, 8>(ctx, q, cent, codes, pair_counts, k, v, out_idx, out_attn, st); break;
  }
}

bool pairs_supported(const pqc_config* c) {
  return c->pq_m == 2 && c->pq_centroids <= kPairC && (c->n_capacity ? c->n_capacity : c->n_tokens) % 8 == 0;
}

template <typename T, int G>
void launch_attn_tg(pqc_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* idx, float* out,
                    hipStream_t st) {
  const Shape& s = ctx->plan.s;
  const unsigned units = (unsigned)(s.B * s.Hkv);
  hipLaunchKernelGGL((attn_list_kernel<T, G>), dim3(s.nblkP, units), dim3(256), sizeof(int) * s.rowsP, st, s, ctx->ws,
                     static_cast<const T*>(q), static_cast<const T*>(k), static_cast<const T*>(v), idx);
  hipLaunchKernelGGL((merge_kernel<G>), dim3(G, units), dim3(256), sizeof(float) * s.nblkP, st, s, ctx->ws, s.nblkP, out);
}

template <typename T>
void launch_attn_t(pqc_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* idx, float* out,
                   hipStream_t st) {
  switch (ctx->plan.s.G) {
    case 1: launch_attn_tg<T, 1>(ctx, q, k, v, idx, out, st); break;
    case 2: launch_attn_tg<T, 2>(ctx, q, k, v, idx, out, st); break;
    case 4: launch_attn_tg<T, 4>(ctx, q, k, v, idx, out, st); break;
    default: launch_attn_tg<T, 8>(ctx, q, k, v, idx, out, st); break;
  }
}

template <typename T>
void launch_lut_t(const Shape& s, const T* q, const float* cent, float* table, hipStream_t st) {
  const dim3 grid(1, (unsigned)(s.B * s.Hkv));
  switch (s.M) {
    case 1: hipLaunchKernelGGL((lut_kernel<T, 1>), grid, dim3(256), 0, st, s, q, cent, table); break;
    case 2: hipLaunchKernelGGL((lut_kernel<T, 2>), grid, dim3(256), 0, st, s, q, cent, table); break;
    case 4: hipLaunchKernelGGL((lut_kernel<T, 4>), grid, dim3(256), 0, st, s, q, cent, table); break;
    default: hipLaunchKernelGGL((lut_kernel<T, 8>), grid, dim3(256), 0, st, s, q, cent, table); break;
  }
}

template <int M>
void launch_scan_m(pqc_ctx* ctx, const float* table, const uint8_t* codes, float* scores, hipStream_t st) {
  const Shape& s = ctx->plan.s;
  hipLaunchKernelGGL((scan_kernel<M>), dim3((s.N + 2047) / 2048, (unsigned)(s.B * s.Hkv)), dim3(256), 0, st, s, table,
                     codes, scores);
}

}  // namespace

extern "C" {

int pqc_version(void) { return 200; }

const char* pqc_strerror(int status) {
  switch (status) {
    case PQC_OK: return "ok";
    case PQC_EINVAL: return "invalid argument or configuration";
    case PQC_EUNSUPPORTED: return "configuration outside the supported shapes";
    case PQC_EWORKSPACE: return "workspace missing, misaligned or too small";
    case PQC_EHIP: return "HIP call failed";
    case PQC_ESCRATCH: return "shape needs more than the static scratch of pqc_decode_static (use pqc_decode with a workspace)";
    default: return "unknown status";
  }
}

#ifdef PQC_TRACE
size_t pqc_debug_trace_offset(const pqc_config* cfg) {
  Plan p;
  if (make_plan(cfg, &p) != PQC_OK) return 0;
  return p.off_trace;
}
#endif

size_t pqc_workspace_bytes(const pqc_config* cfg) { return workspace_bound(cfg); }

namespace {
// Point the context's views at the regions of its plan.
void bind_workspace(pqc_ctx* ctx) {
  const Plan& p = ctx->plan;
  char* base = ctx->workspace;
  ctx->ws.ctl = reinterpret_cast<BinParams*>(base + p.off_ctl);
  ctx->ws.lut = reinterpret_cast<float*>(base + p.off_lut);
  ctx->ws.hist = reinterpret_cast<unsigned*>(base + p.off_hist);
  ctx->ws.cand_count = ctx->ws.hist + (size_t)p.s.B * p.s.Hkv * kHistCopies * kNB;
  ctx->ws.range = reinterpret_cast<float2*>(base + p.off_range);
  ctx->ws.bins = reinterpret_cast<unsigned short*>(base + p.off_bins);
  ctx->ws.cand_rec = reinterpret_cast<unsigned char*>(base + p.off_crec);
  ctx->ws.rec_stride = p.rec_stride;
  ctx->ws.stage = reinterpret_cast<unsigned long long*>(base + p.off_stage);
  ctx->ws.stage_cnt = reinterpret_cast<int2*>(base + p.off_cnt);
  ctx->ws.partials = reinterpret_cast<float*>(base + p.off_part);
#ifdef PQC_TRACE
  ctx->ws.trace = reinterpret_cast<unsigned long long*>(base + p.off_trace);
#endif
}
}  // namespace

int pqc_create(pqc_ctx** out, const pqc_config* cfg, void* workspace, size_t workspace_bytes) {
  if (!out) return PQC_EINVAL;
  *out = nullptr;
  Plan p;
  const int rc = make_plan(cfg, &p);
  if (rc != PQC_OK) return rc;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) || workspace_bytes < p.total) return PQC_EWORKSPACE;
  pqc_ctx* ctx = new (std::nothrow) pqc_ctx;
  if (!ctx) return PQC_EINVAL;
  ctx->cfg = *cfg;
  ctx->cfg.n_capacity = p.s.cap;
  ctx->plan = p;
  ctx->workspace = static_cast<char*>(workspace);
  ctx->workspace_bytes = workspace_bytes;
  bind_workspace(ctx);
  ctx->hist_clean = false;
  ctx->next_phase = 0;
  ctx->last_hip = 0;
  ctx->append = AppendArgs{nullptr, nullptr, nullptr, 0, nullptr};
  *out = ctx;
  return PQC_OK;
}

int pqc_set_length(pqc_ctx* ctx, int32_t n_tokens, int32_t topk) {
  if (!ctx) return PQC_EINVAL;
  pqc_config c = ctx->cfg;
  c.n_tokens = n_tokens;
  c.topk = topk;
  Plan p;
  const int rc = make_plan(&c, &p);  // rejects a length beyond the capacity
  if (rc != PQC_OK) return rc;
  if (p.total > ctx->workspace_bytes) return PQC_EWORKSPACE;
  // The histogram region does not move and a clean one is all zero, whatever the length: it stays clean.
  ctx->cfg = c;
  ctx->plan = p;
  bind_workspace(ctx);
  return PQC_OK;
}

void pqc_destroy(pqc_ctx* ctx) { delete ctx; }

int pqc_last_hip_error(const pqc_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

static int decode_impl(pqc_ctx* ctx, const void* q, const float* centroids, const uint8_t* codes, const void* k_cache,
                       const void* v_cache, int32_t* out_idx, float* out_attn, void* stream, unsigned phases) {
  if (!ctx || !q || !centroids || !codes || !k_cache || !v_cache || !out_idx || !out_attn) return PQC_EINVAL;
  if (!aligned16(q) || !aligned16(centroids) || !aligned16(codes) || !aligned16(k_cache) || !aligned16(v_cache) ||
      !aligned16(out_idx) || !aligned16(out_attn))
    return PQC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = PQC_OK;
  if (phases & 1u) {
    rc = ensure_clean_hist(ctx, st);
    if (rc != PQC_OK) return rc;
    ctx->hist_clean = false;
  }
  if (ctx->cfg.kv_dtype == PQC_F32)
    launch_decode_t<float>(ctx, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, st, phases);
  else
    launch_decode_t<bf16_t>(ctx, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, st, phases);
  rc = check_launch(ctx);
  if (rc == PQC_OK && (phases & 4u)) {
    ctx->hist_clean = true;  // finalize_kernel zeroed them again
  }
  return rc;
}

int pqc_decode(pqc_ctx* ctx, const void* q, const float* centroids, const uint8_t* codes, const void* k_cache,
               const void* v_cache, int32_t* out_idx, float* out_attn, void* stream) {
  return decode_impl(ctx, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, stream, 7u);
}

int pqc_decode_append(pqc_ctx* ctx, const void* q, const float* centroids, uint8_t* codes, const void* k_cache,
                      const void* v_cache, const void* new_key, int32_t position, int32_t* out_idx, float* out_attn,
                      void* stream) {
  if (!ctx || !new_key || !aligned16(new_key)) return PQC_EINVAL;
  const Shape& s = ctx->plan.s;
  // only a position whose code this call does not read: inside a window, or beyond the tokens in use
  if (position < 0 || position >= s.cap || (position >= s.I && position < s.N - s.L)) return PQC_EINVAL;
  ctx->append = AppendArgs{new_key, centroids, codes, (int)position, nullptr};
  const int rc = decode_impl(ctx, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, stream, 7u);
  ctx->append = AppendArgs{nullptr, nullptr, nullptr, 0, nullptr};
  return rc;
}

static int indexed_impl(pqc_ctx* ctx, const void* q, const float* centroids, const uint8_t* codes,
                        const uint32_t* pair_counts, const void* k_cache, const void* v_cache, int32_t* out_idx,
                        float* out_attn, void* stream) {
  if (!ctx || !q || !centroids || !codes || !pair_counts || !k_cache || !v_cache || !out_idx || !out_attn) return PQC_EINVAL;
  if (!aligned16(q) || !aligned16(centroids) || !aligned16(codes) || !aligned16(pair_counts) || !aligned16(k_cache) ||
      !aligned16(v_cache) || !aligned16(out_idx) || !aligned16(out_attn))
    return PQC_EINVAL;
  if (!pairs_supported(&ctx->cfg)) return PQC_EUNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = ensure_clean_hist(ctx, st);  // the record counters live with the histograms
  if (rc != PQC_OK) return rc;
  ctx->hist_clean = false;
  if (ctx->cfg.kv_dtype == PQC_F32)
    launch_indexed_t<float>(ctx, q, centroids, codes, pair_counts, k_cache, v_cache, out_idx, out_attn, st);
  else
    launch_indexed_t<bf16_t>(ctx, q, centroids, codes, pair_counts, k_cache, v_cache, out_idx, out_attn, st);
  rc = check_launch(ctx);
  if (rc == PQC_OK) {
    ctx->hist_clean = true;
  }
  return rc;
}

int pqc_decode_indexed(pqc_ctx* ctx, const void* q, const float* centroids, const uint8_t* codes,
                       const uint32_t* pair_counts, const void* k_cache, const void* v_cache, int32_t* out_idx,
                       float* out_attn, void* stream) {
  return indexed_impl(ctx, q, centroids, codes, pair_counts, k_cache, v_cache, out_idx, out_attn, stream);
}

int pqc_decode_indexed_append(pqc_ctx* ctx, const void* q, const float* centroids, uint8_t* codes, uint32_t* pair_counts,
                              const void* k_cache, const void* v_cache, const void* new_key, int32_t position,
                              int32_t* out_idx, float* out_attn, void* stream) {
  if (!ctx || !new_key || !aligned16(new_key)) return PQC_EINVAL;
  const Shape& s = ctx->plan.s;
  if (position < 0 || position >= s.cap || (position >= s.I && position < s.N - s.L)) return PQC_EINVAL;
  ctx->append = AppendArgs{new_key, centroids, codes, (int)position, pair_counts};
  const int rc = indexed_impl(ctx, q, centroids, codes, pair_counts, k_cache, v_cache, out_idx, out_attn, stream);
  ctx->append = AppendArgs{nullptr, nullptr, nullptr, 0, nullptr};
  return rc;
}

int pqc_pair_counts(const pqc_config* cfg, const uint8_t* codes, uint32_t* pair_counts, void* stream) {
  Plan p;
  const int rc = make_plan(cfg, &p);
  if (rc != PQC_OK) return rc;
  if (!codes || !pair_counts) return PQC_EINVAL;
  if (cfg->pq_m != 2 || cfg->pq_centroids > kPairC) return PQC_EUNSUPPORTED;
  const Shape& s = p.s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t n = (size_t)s.B * s.Hkv * s.C * s.C;
  hipLaunchKernelGGL(reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, pair_counts, n);
  hipLaunchKernelGGL(pair_count_kernel, dim3((unsigned)((s.N + kPairTok - 1) / kPairTok), (unsigned)(s.B * s.Hkv)), dim3(256), 0,
                     st, codes, s.N, s.cap, s.C, pair_counts);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

int pqc_pair_counts_add(const pqc_config* cfg, const uint8_t* codes, int32_t position, uint32_t* pair_counts, void* stream) {
  Plan p;
  const int rc = make_plan(cfg, &p);
  if (rc != PQC_OK) return rc;
  if (!codes || !pair_counts || position < 0 || position >= p.s.cap) return PQC_EINVAL;
  if (cfg->pq_m != 2 || cfg->pq_centroids > kPairC) return PQC_EUNSUPPORTED;
  const int units = p.s.B * p.s.Hkv;
  hipLaunchKernelGGL(pair_count_add_kernel, dim3((unsigned)((units + 63) / 64)), dim3(64), 0, static_cast<hipStream_t>(stream),
                     codes, p.s.cap, p.s.C, units, (int)position, pair_counts);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

int pqc_decode_phase(pqc_ctx* ctx, int phase, const void* q, const float* centroids, const uint8_t* codes,
                     const void* k_cache, const void* v_cache, int32_t* out_idx, float* out_attn, void* stream) {
  if (!ctx || phase < 0 || phase >= PQC_DECODE_KERNELS) return PQC_EINVAL;
  if (phase != ctx->next_phase) return PQC_EINVAL;  // a phase out of turn would count a histogram twice or read a stale one
  const int rc = decode_impl(ctx, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, stream, 1u << phase);
  if (rc == PQC_OK) ctx->next_phase = (phase + 1) % PQC_DECODE_KERNELS;
  return rc;
}

int pqc_lut(pqc_ctx* ctx, const void* q, const float* centroids, float* table, void* stream) {
  if (!ctx || !q || !centroids || !table) return PQC_EINVAL;
  if (!aligned16(q) || !aligned16(centroids) || !aligned16(table)) return PQC_EINVAL;
  const Shape& s = ctx->plan.s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->cfg.kv_dtype == PQC_F32)
    launch_lut_t<float>(s, static_cast<const float*>(q), centroids, table, st);
  else
    launch_lut_t<bf16_t>(s, static_cast<const bf16_t*>(q), centroids, table, st);
  return check_launch(ctx);
}

int pqc_scan(pqc_ctx* ctx, const float* table, const uint8_t* codes, float* scores, void* stream) {
  if (!ctx || !table || !codes || !scores) return PQC_EINVAL;
  if (!aligned16(table) || !aligned16(codes) || !aligned16(scores)) return PQC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  switch (ctx->plan.s.M) {
    case 1: launch_scan_m<1>(ctx, table, codes, scores, st); break;
    case 2: launch_scan_m<2>(ctx, table, codes, scores, st); break;
    case 4: launch_scan_m<4>(ctx, table, codes, scores, st); break;
    default: launch_scan_m<8>(ctx, table, codes, scores, st); break;
  }
  return check_launch(ctx);
}

int pqc_topk(pqc_ctx* ctx, const float* scores, int32_t* out_idx, void* stream) {
  if (!ctx || !scores || !out_idx) return PQC_EINVAL;
  if (!aligned16(scores) || !aligned16(out_idx)) return PQC_EINVAL;
  const Shape& s = ctx->plan.s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = ensure_clean_hist(ctx, st);
  if (rc != PQC_OK) return rc;
  ctx->hist_clean = false;
  const unsigned units = (unsigned)(s.B * s.Hkv);
  const float* nof = nullptr;
  hipLaunchKernelGGL(score_range_kernel, dim3(1, units), dim3(1024), 0, st, s, scores, ctx->ws.range);
  launch_hist<float, ScoreChunks>(s, ctx->ws, nof, nof, static_cast<const void*>(scores), 0, st);
  hipLaunchKernelGGL((select_kernel<float, 1, ScoreChunks, false>), dim3(s.nblkC, units), dim3(256), s.tokC * sizeof(unsigned short), st,
                     s, ctx->ws, nof, nof, nof, static_cast<const void*>(scores));
  hipLaunchKernelGGL((finalize_kernel<float, 1, false>), dim3(1 + kCopyWgs, units), dim3(256), finalize_lds_bytes(s, false), st, s,
                     ctx->ws, nof, nof, nof, out_idx, static_cast<float*>(nullptr), AppendArgs{nullptr, nullptr, nullptr, 0, nullptr});
  rc = check_launch(ctx);
  if (rc == PQC_OK) {
    ctx->hist_clean = true;
  }
  return rc;
}

int pqc_gather_attn(pqc_ctx* ctx, const void* q, const void* k_cache, const void* v_cache, const int32_t* idx,
                    float* out_attn, void* stream) {
  if (!ctx || !q || !k_cache || !v_cache || !idx || !out_attn) return PQC_EINVAL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(idx) || !aligned16(out_attn)) return PQC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->cfg.kv_dtype == PQC_F32)
    launch_attn_t<float>(ctx, q, k_cache, v_cache, idx, out_attn, st);
  else
    launch_attn_t<bf16_t>(ctx, q, k_cache, v_cache, idx, out_attn, st);
  return check_launch(ctx);
}


}  // extern "C"

/* ------------------------------------------------- decode without an allocation */
// For callers that can neither allocate device memory nor hold a workspace of their own (code under HIP graph
// capture, serving loops, harnesses that forbid hipMalloc): the workspace of the step is a file-scope device
// array.  Host code never uses the array's name as an address: its device address is looked up once per device.
namespace {

constexpr size_t kStaticScratchBytes = (size_t)24 << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];  // per device: where that device holds its copy of `scratch`

// Device address of the current device's scratch array (looked up on the first call on that device).
int static_scratch(unsigned char** out, int* hip_code) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *hip_code = (int)e;
    return PQC_EHIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      *hip_code = (int)e;
      return PQC_EHIP;
    }
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return PQC_OK;
}

}  // namespace

extern "C" {

size_t pqc_static_scratch_bytes(void) { return kStaticScratchBytes; }

int pqc_decode_static(const pqc_config* cfg, const void* q, const float* centroids, const uint8_t* codes, const void* k_cache,
                      const void* v_cache, int32_t* out_idx, float* out_attn, void* stream) {
  pqc_ctx ctx;  // on the stack: nothing is allocated, on the host either
  const int rc = make_plan(cfg, &ctx.plan);
  if (rc != PQC_OK) return rc;
  if (ctx.plan.total > kStaticScratchBytes) return PQC_ESCRATCH;
  unsigned char* base = nullptr;
  int hip_code = 0;
  const int rs = static_scratch(&base, &hip_code);
  if (rs != PQC_OK) return rs;
  ctx.cfg = *cfg;
  ctx.cfg.n_capacity = ctx.plan.s.cap;
  ctx.workspace = reinterpret_cast<char*>(base);
  ctx.workspace_bytes = kStaticScratchBytes;
  bind_workspace(&ctx);
  ctx.next_phase = 0;
  ctx.hist_clean = false;  // the array keeps what the last call (of any shape) left: the step's counters are cleared first,
                           // by a fill kernel, so that the call can be recorded into a graph
  ctx.last_hip = 0;
  ctx.append = AppendArgs{nullptr, nullptr, nullptr, 0, nullptr};
  return decode_impl(&ctx, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, stream, 7u);
}

}  // extern "C"

/* ------------------------------------------------------------ PQ construction */
namespace {

struct BuildPlan {
  BuildShape s;
  size_t off_sums, off_counts, total;
};

int make_build_plan(const pqc_config* cfg, BuildPlan* bp) {
  Plan p;
  const int rc = make_plan(cfg, &p);
  if (rc != PQC_OK) return rc;
  bp->s.units = p.s.B * p.s.Hkv;
  bp->s.N = p.s.N; bp->s.M = p.s.M; bp->s.C = p.s.C; bp->s.Dm = p.s.Dm; bp->s.cap = p.s.cap;
  const size_t n = (size_t)bp->s.units * p.s.M * p.s.C;
  bp->off_sums = 0;
  bp->off_counts = align_up(sizeof(unsigned long long) * n * p.s.Dm);
  bp->total = align_up(bp->off_counts + sizeof(unsigned) * n);
  return PQC_OK;
}

template <typename T>
void launch_assign(const BuildShape& s, const T* keys, int64_t unit_stride, int n_tokens, int pos0, const float* cent,
                   uint8_t* codes, hipStream_t st) {
  if constexpr (sizeof(T) == 2) {
    if (s.Dm >= 32) {  // bf16 keys: the matrix-core kernel
      const dim3 mgrid((n_tokens + kAssignMfmaTok - 1) / kAssignMfmaTok, (unsigned)(s.units * s.M));
      const bf16_t* kb = reinterpret_cast<const bf16_t*>(keys);
      switch (s.Dm) {
        case 32: hipLaunchKernelGGL((pq_assign_mfma_kernel<32>), mgrid, dim3(256), 0, st, s, kb, unit_stride, n_tokens, pos0, cent, codes); break;
        case 64: hipLaunchKernelGGL((pq_assign_mfma_kernel<64>), mgrid, dim3(256), 0, st, s, kb, unit_stride, n_tokens, pos0, cent, codes); break;
        default: hipLaunchKernelGGL((pq_assign_mfma_kernel<128>), mgrid, dim3(256), 0, st, s, kb, unit_stride, n_tokens, pos0, cent, codes); break;
      }
      return;
    }
  }
  const dim3 grid((n_tokens + kAssignTok - 1) / kAssignTok, (unsigned)(s.units * s.M));
  switch (s.Dm) {
    case 16: hipLaunchKernelGGL((pq_assign_kernel<T, 16>), grid, dim3(256), 0, st, s, keys, unit_stride, n_tokens, pos0, cent, codes); break;
    case 32: hipLaunchKernelGGL((pq_assign_kernel<T, 32>), grid, dim3(256), 0, st, s, keys, unit_stride, n_tokens, pos0, cent, codes); break;
    case 64: hipLaunchKernelGGL((pq_assign_kernel<T, 64>), grid, dim3(256), 0, st, s, keys, unit_stride, n_tokens, pos0, cent, codes); break;
    default: hipLaunchKernelGGL((pq_assign_kernel<T, 128>), grid, dim3(256), 0, st, s, keys, unit_stride, n_tokens, pos0, cent, codes); break;
  }
}

template <typename T>
int pq_build_t(const BuildPlan& bp, const T* keys, const int32_t* init_idx, int iters, float* cent, uint8_t* codes,
               char* wsp, hipStream_t st) {
  const BuildShape& s = bp.s;
  unsigned long long* sums = reinterpret_cast<unsigned long long*>(wsp + bp.off_sums);
  unsigned* counts = reinterpret_cast<unsigned*>(wsp + bp.off_counts);
  const unsigned uj = (unsigned)(s.units * s.M);
  const size_t nacc = bp.total / sizeof(unsigned long long);  // sums and counts, zeroed together
  const size_t ncent = (size_t)uj * s.C * s.Dm;
  hipLaunchKernelGGL((pq_init_kernel<T>), dim3(1, uj), dim3(256), 0, st, s, keys, init_idx, cent);
  for (int it = 0; it < iters; ++it) {
    launch_assign<T>(s, keys, (int64_t)s.cap * kD, s.N, 0, cent, codes, st);
    hipLaunchKernelGGL(pq_zero_kernel, dim3((unsigned)((nacc + 255) / 256)), dim3(256), 0, st, sums, nacc);
    {
      const int tpw = accum_tokens_per_wg(s.C);
      const dim3 grid((s.N + tpw - 1) / tpw, uj);
      const size_t lds = (size_t)tpw * sizeof(unsigned short);
      switch (s.Dm) {
        case 16: hipLaunchKernelGGL((pq_accum_kernel<T, 16>), grid, dim3(256), lds, st, s, keys, codes, sums, counts); break;
        case 32: hipLaunchKernelGGL((pq_accum_kernel<T, 32>), grid, dim3(256), lds, st, s, keys, codes, sums, counts); break;
        case 64: hipLaunchKernelGGL((pq_accum_kernel<T, 64>), grid, dim3(256), lds, st, s, keys, codes, sums, counts); break;
        default: hipLaunchKernelGGL((pq_accum_kernel<T, 128>), grid, dim3(256), lds, st, s, keys, codes, sums, counts); break;
      }
    }
    hipLaunchKernelGGL(pq_mean_kernel, dim3((unsigned)((ncent + 255) / 256)), dim3(256), 0, st, s, sums, counts, cent);
  }
  launch_assign<T>(s, keys, (int64_t)s.cap * kD, s.N, 0, cent, codes, st);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

}  // namespace

extern "C" {

size_t pqc_pq_build_workspace_bytes(const pqc_config* cfg) {
  BuildPlan bp;
  if (make_build_plan(cfg, &bp) != PQC_OK) return 0;
  return bp.total;
}

int pqc_pq_build(const pqc_config* cfg, const void* keys, const int32_t* init_idx, int32_t iters, float* centroids,
                 uint8_t* codes, void* workspace, size_t workspace_bytes, void* stream) {
  BuildPlan bp;
  const int rc = make_build_plan(cfg, &bp);
  if (rc != PQC_OK) return rc;
  if (!keys || !init_idx || !centroids || !codes || iters < 0) return PQC_EINVAL;
  if (!aligned16(keys) || !aligned16(init_idx) || !aligned16(centroids) || !aligned16(codes)) return PQC_EINVAL;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) || workspace_bytes < bp.total) return PQC_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* wsp = static_cast<char*>(workspace);
  if (cfg->kv_dtype == PQC_F32) return pq_build_t<float>(bp, static_cast<const float*>(keys), init_idx, iters, centroids, codes, wsp, st);
  return pq_build_t<bf16_t>(bp, static_cast<const bf16_t*>(keys), init_idx, iters, centroids, codes, wsp, st);
}

int pqc_pq_assign(const pqc_config* cfg, const void* keys, const float* centroids, uint8_t* codes, void* stream) {
  BuildPlan bp;
  const int rc = make_build_plan(cfg, &bp);
  if (rc != PQC_OK) return rc;
  if (!keys || !centroids || !codes) return PQC_EINVAL;
  if (!aligned16(keys) || !aligned16(centroids) || !aligned16(codes)) return PQC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const BuildShape& s = bp.s;
  if (cfg->kv_dtype == PQC_F32)
    launch_assign<float>(s, static_cast<const float*>(keys), (int64_t)s.cap * kD, s.N, 0, centroids, codes, st);
  else
    launch_assign<bf16_t>(s, static_cast<const bf16_t*>(keys), (int64_t)s.cap * kD, s.N, 0, centroids, codes, st);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

int pqc_pq_encode_token(const pqc_config* cfg, const void* key, const float* centroids, uint8_t* codes, int32_t position,
                        void* stream) {
  BuildPlan bp;
  const int rc = make_build_plan(cfg, &bp);
  if (rc != PQC_OK) return rc;
  if (!key || !centroids || !codes || position < 0 || position >= bp.s.cap) return PQC_EINVAL;
  if (!aligned16(key) || !aligned16(centroids) || !aligned16(codes)) return PQC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const BuildShape& s = bp.s;
  const dim3 grid((unsigned)(s.units * s.M));
  if (cfg->kv_dtype == PQC_F32)
    hipLaunchKernelGGL(pq_encode_kernel<float>, grid, dim3(256), 0, st, s, static_cast<const float*>(key), (int)position, centroids,
                       codes);
  else
    hipLaunchKernelGGL(pq_encode_kernel<bf16_t>, grid, dim3(256), 0, st, s, static_cast<const bf16_t*>(key), (int)position,
                       centroids, codes);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

int pqc_block_stats(const pqc_config* cfg, const int32_t* idx, int64_t n_idx, int32_t block_tokens, int32_t k_cache,
                    int32_t* counts, int32_t* blocks, void* stream) {
  Plan p;
  int rc = make_plan(cfg, &p);
  if (rc != PQC_OK) return rc;
  if (!idx || !counts || n_idx < 0 || block_tokens < 1 || block_tokens >= kCountBins) return PQC_EINVAL;
  const int nb = (p.s.N + block_tokens - 1) / block_tokens;
  if (k_cache < 0 || k_cache > nb || (k_cache > 0 && !blocks)) return PQC_EINVAL;
  hipLaunchKernelGGL(block_stats_kernel, dim3((unsigned)(p.s.B * p.s.Hkv)), dim3(1024), 0, static_cast<hipStream_t>(stream),
                     idx, (long long)n_idx, p.s.N, (int)block_tokens, nb, (int)k_cache, counts, blocks);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

int pqc_block_cache_update(const pqc_config* cfg, int32_t block_tokens, int32_t n_slots, int32_t policy, int32_t step,
                           const int32_t* counts, const int32_t* blocks, int32_t k_cache, int32_t* slot_block,
                           int32_t* slot_stamp, int32_t* slot_uses, int32_t* stats, void* stream) {
  Plan p;
  const int rc = make_plan(cfg, &p);
  if (rc != PQC_OK) return rc;
  if (!counts || !slot_block || !slot_stamp || !slot_uses || !stats || block_tokens < 1) return PQC_EINVAL;
  if (n_slots < 1 || n_slots > kCacheSlots || k_cache < 0 || k_cache > kCacheSlots || (k_cache > 0 && !blocks)) return PQC_EINVAL;
  if (policy != PQC_CACHE_LRU && policy != PQC_CACHE_LFU) return PQC_EINVAL;
  const int nb = (p.s.N + block_tokens - 1) / block_tokens;
  hipLaunchKernelGGL(block_cache_kernel, dim3((unsigned)(p.s.B * p.s.Hkv)), dim3(256), 0, static_cast<hipStream_t>(stream), nb,
                     (int)n_slots, (int)k_cache, policy == PQC_CACHE_LFU ? 1 : 0, (int)step, counts, blocks, slot_block, slot_stamp,
                     slot_uses, stats);
  return hipGetLastError() == hipSuccess ? PQC_OK : PQC_EHIP;
}

}  // extern "C"
