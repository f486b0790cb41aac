// Host side of the C ABI declared in include/choco.h: argument checks, workspace
// layout, kernel launches.  No device memory is allocated here; everything lives
// in the caller's workspace.  No call synchronises unless the header says so.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "choco.h"
#include "choco_kernels.h"

using namespace choco;

struct choco_ctx {
  choco_config cfg;       // scalar fields as given (host CSR pointers are not kept)
  Args args;              // kernel arguments (device pointers into the workspace)
  hipStream_t stream;
  int32_t maxdeg;
  int32_t nnz;
  bool sparse;            // top_a / random_a
  int mix_form;           // resolved: CHOCO_MIX_INCREMENTAL_S or CHOCO_MIX_DIRECT
  int rpw;                // rows per wave of the tile kernels, 0 = tile does not fit
  uint64_t t;             // step counter
  double* metrics_part;   // device scratch of the metrics kernels
  double* metrics_out;
  int metrics_blocks;
  int last_hip_error;
  bool destroyed;
};

namespace {

constexpr size_t kAlign = 256;
constexpr int kMetricsBlocks = 1024;
constexpr int kMaxTileRows = 64;  // n * 1 KiB of LDS for the tile of all rows

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t xhat, s, row_ptr, col, w, ctl, partial, hist, cand, sel_idx, sel_val, bitmap, mpart, mout,
      total;
  uint32_t cand_cap;
  int64_t bitmap_words;
  int32_t nchunks;
};

bool is_sparse(int compressor) { return compressor == CHOCO_Q_TOPK || compressor == CHOCO_Q_RANDK; }

int resolve_mix_form(const choco_config& c) {
  if (c.mix_form == CHOCO_MIX_AUTO)
    return is_sparse(c.compressor) ? CHOCO_MIX_INCREMENTAL_S : CHOCO_MIX_DIRECT;
  return c.mix_form;
}

int64_t resolve_ld(const choco_config& c) { return c.ld == 0 ? (c.d + 3) / 4 * 4 : c.ld; }

// Scalar-field validation shared by choco_workspace_bytes and choco_init.
int check_scalars(const choco_config* c) {
  if (!c) return CHOCO_E_INVAL;
  if (c->n < 1 || c->d < 1 || c->d >= (int64_t)1 << 31) return CHOCO_E_INVAL;
  const int64_t ld = resolve_ld(*c);
  if (ld < c->d || (ld & 3) != 0) return CHOCO_E_INVAL;
  if (!(c->gamma > 0.0f) || !std::isfinite(c->gamma)) return CHOCO_E_INVAL;
  if (c->compressor < CHOCO_Q_IDENTITY || c->compressor > CHOCO_Q_QSGD) return CHOCO_E_INVAL;
  if (is_sparse(c->compressor) && (c->k < 1 || c->k > c->d)) return CHOCO_E_INVAL;
  if (c->compressor == CHOCO_Q_QSGD && c->levels < 1) return CHOCO_E_INVAL;
  if (c->order != CHOCO_ORDER_COMPRESS_THEN_MIX && c->order != CHOCO_ORDER_MIX_THEN_COMPRESS)
    return CHOCO_E_INVAL;
  if (c->mix_form < CHOCO_MIX_AUTO || c->mix_form > CHOCO_MIX_DIRECT) return CHOCO_E_INVAL;
  // combinations this build does not implement
  if (!is_sparse(c->compressor) && resolve_mix_form(*c) == CHOCO_MIX_INCREMENTAL_S)
    return CHOCO_E_UNSUPPORTED;
  return CHOCO_OK;
}

Layout make_layout(const choco_config& c, int32_t nnz) {
  Layout L{};
  const int64_t ld = resolve_ld(c);
  const size_t state = (size_t)c.n * (size_t)ld * sizeof(float);
  const bool sparse = is_sparse(c.compressor);
  size_t off = 0;
  auto take = [&off](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.xhat = take(state);
  L.s = take(resolve_mix_form(c) == CHOCO_MIX_INCREMENTAL_S ? state : 0);
  L.row_ptr = take((size_t)(c.n + 1) * sizeof(int32_t));
  L.col = take((size_t)nnz * sizeof(int32_t));
  L.w = take((size_t)nnz * sizeof(float));
  L.ctl = take((size_t)c.n * sizeof(WorkerCtl));
  L.nchunks = (int32_t)((c.d + kChunk - 1) / kChunk);
  L.partial = take(sparse ? 0 : (size_t)c.n * (size_t)L.nchunks * sizeof(double));
  int64_t cap = 0;
  if (sparse) {
    cap = 4 * c.k;
    if (cap < c.d / 128) cap = c.d / 128;
    if (cap < 8192) cap = 8192;
    if (cap > c.d) cap = c.d;
  }
  L.cand_cap = (uint32_t)cap;
  L.bitmap_words = sparse ? (c.d + 31) / 32 : 0;
  L.hist = take(sparse ? (size_t)c.n * kBins * sizeof(uint32_t) : 0);
  L.cand = take(sparse ? (size_t)c.n * (size_t)cap * sizeof(uint2) : 0);
  L.sel_idx = take(sparse ? (size_t)c.n * (size_t)c.k * sizeof(int32_t) : 0);
  L.sel_val = take(sparse ? (size_t)c.n * (size_t)c.k * sizeof(float) : 0);
  L.bitmap = take(sparse ? (size_t)c.n * (size_t)L.bitmap_words * sizeof(uint32_t) : 0);
  L.mpart = take((size_t)kMetricsBlocks * 3 * sizeof(double));
  L.mout = take(3 * sizeof(double));
  L.total = off;
  return L;
}

// Assumption 1: W symmetric, entries in [0,1], rows (hence columns) sum to one.
int check_csr(const choco_config* c, int32_t* nnz_out, int32_t* maxdeg_out) {
  if (!c->row_ptr_host || !c->col_idx_host || !c->w_host) return CHOCO_E_INVAL;
  const int32_t* rp = c->row_ptr_host;
  if (rp[0] != 0) return CHOCO_E_INVAL;
  int32_t maxdeg = 0;
  for (int i = 0; i < c->n; ++i) {
    if (rp[i + 1] <= rp[i]) return CHOCO_E_INVAL;  // the self-loop is mandatory
    if (rp[i + 1] - rp[i] > maxdeg) maxdeg = rp[i + 1] - rp[i];
  }
  const int32_t nnz = rp[c->n];
  for (int i = 0; i < c->n; ++i) {
    double sum = 0.0;
    bool self = false;
    for (int p = rp[i]; p < rp[i + 1]; ++p) {
      const int j = c->col_idx_host[p];
      const float wij = c->w_host[p];
      if (j < 0 || j >= c->n) return CHOCO_E_INVAL;
      if (p > rp[i] && j <= c->col_idx_host[p - 1]) return CHOCO_E_INVAL;
      if (!(wij >= 0.0f) || !(wij <= 1.0f + 1e-6f)) return CHOCO_E_INVAL;
      if (j == i) self = true;
      sum += (double)wij;
      // symmetric partner
      bool found = false;
      for (int p2 = rp[j]; p2 < rp[j + 1]; ++p2)
        if (c->col_idx_host[p2] == i) {
          found = std::fabs((double)c->w_host[p2] - (double)wij) <= 1e-6;
          break;
        }
      if (!found) return CHOCO_E_INVAL;
    }
    if (!self || std::fabs(sum - 1.0) > 1e-6 * (rp[i + 1] - rp[i])) return CHOCO_E_INVAL;
  }
  *nnz_out = nnz;
  *maxdeg_out = maxdeg;
  return CHOCO_OK;
}

int hip_fail(choco_ctx* ctx, hipError_t e) {
  if (ctx) ctx->last_hip_error = (int)e;
  return CHOCO_E_HIP;
}

#define HIP_TRY(ctx, expr)                        \
  do {                                            \
    hipError_t e_ = (expr);                       \
    if (e_ != hipSuccess) return hip_fail(ctx, e_); \
  } while (0)

#define LAUNCH_CHECK(ctx) HIP_TRY(ctx, hipGetLastError())

// grid for the streaming kernels: enough blocks to fill 256 CUs several times
// over, capped so that the grid-stride loops keep a few float4 per thread
dim3 stream_grid(int32_t nvec, int32_t n) {
  int64_t blocks = ((int64_t)nvec + 255) / 256;
  int64_t cap = 16384 / n;
  if (cap < 64) cap = 64;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return dim3((unsigned)blocks, (unsigned)n, 1);
}

int pick_rpw(int n) {
  if (n > kMaxTileRows) return 0;
  const int rows = (n + 3) / 4;
  if (rows <= 1) return 1;
  if (rows <= 2) return 2;
  if (rows <= 4) return 4;
  if (rows <= 8) return 8;
  return 16;
}

template <int COMP, bool CAPTURE>
void launch_apply_mix(choco_ctx* ctx, const Args& A) {
  const dim3 grid((unsigned)A.nchunks), block(kTileThreads);
  const size_t lds = (size_t)A.n * kChunk * sizeof(float);
  switch (ctx->rpw) {
    case 1: hipLaunchKernelGGL((k_dense_apply_mix<COMP, 1, CAPTURE>), grid, block, lds, ctx->stream, A); break;
    case 2: hipLaunchKernelGGL((k_dense_apply_mix<COMP, 2, CAPTURE>), grid, block, lds, ctx->stream, A); break;
    case 4: hipLaunchKernelGGL((k_dense_apply_mix<COMP, 4, CAPTURE>), grid, block, lds, ctx->stream, A); break;
    case 8: hipLaunchKernelGGL((k_dense_apply_mix<COMP, 8, CAPTURE>), grid, block, lds, ctx->stream, A); break;
    default: hipLaunchKernelGGL((k_dense_apply_mix<COMP, 16, CAPTURE>), grid, block, lds, ctx->stream, A); break;
  }
}

template <int STAT>
void launch_tile_mix(choco_ctx* ctx, const Args& A) {
  const dim3 grid((unsigned)A.nchunks), block(kTileThreads);
  const size_t lds = (size_t)A.n * kChunk * sizeof(float);
  switch (ctx->rpw) {
    case 1: hipLaunchKernelGGL((k_tile_mix<STAT, 1>), grid, block, lds, ctx->stream, A); break;
    case 2: hipLaunchKernelGGL((k_tile_mix<STAT, 2>), grid, block, lds, ctx->stream, A); break;
    case 4: hipLaunchKernelGGL((k_tile_mix<STAT, 4>), grid, block, lds, ctx->stream, A); break;
    case 8: hipLaunchKernelGGL((k_tile_mix<STAT, 8>), grid, block, lds, ctx->stream, A); break;
    default: hipLaunchKernelGGL((k_tile_mix<STAT, 16>), grid, block, lds, ctx->stream, A); break;
  }
}

template <int COMP>
void launch_dense_apply(choco_ctx* ctx, const Args& A, dim3 grid) {
  if (A.codes) hipLaunchKernelGGL((k_dense_apply<COMP, true>), grid, dim3(256), 0, ctx->stream, A);
  else hipLaunchKernelGGL((k_dense_apply<COMP, false>), grid, dim3(256), 0, ctx->stream, A);
}

template <int COMP>
void launch_apply_mix_cap(choco_ctx* ctx, const Args& A) {
  if (A.codes) launch_apply_mix<COMP, true>(ctx, A);
  else launch_apply_mix<COMP, false>(ctx, A);
}

// Dense operators (identity, sign, gsgd), direct mix form.
template <int COMP>
int gossip_dense(choco_ctx* ctx) {
  const Args& A = ctx->args;
  const int32_t nvec = (A.d + 3) >> 2;
  const dim3 sgrid = stream_grid(nvec, A.n);
  const bool needs_stat = (COMP == Q_SIGN || COMP == Q_QSGD);
  constexpr int STAT = (COMP == Q_SIGN || COMP == Q_QSGD) ? COMP : Q_NONE;
  if (ctx->cfg.order == CHOCO_ORDER_COMPRESS_THEN_MIX) {
    if (needs_stat) {
      int64_t blocks = ((int64_t)A.nchunks + 3) / 4;
      int64_t cap = 32768 / A.n;
      if (cap < 64) cap = 64;
      if (blocks > cap) blocks = cap;
      hipLaunchKernelGGL((k_dense_stat<STAT == Q_NONE ? Q_SIGN : STAT>), dim3((unsigned)blocks, (unsigned)A.n),
                         dim3(256), 0, ctx->stream, A);
      hipLaunchKernelGGL((k_dense_finalise<STAT == Q_NONE ? Q_SIGN : STAT>), dim3((unsigned)A.n), dim3(256), 0,
                         ctx->stream, A);
    }
    if (ctx->rpw) {
      launch_apply_mix_cap<COMP>(ctx, A);
    } else {
      launch_dense_apply<COMP>(ctx, A, sgrid);
      hipLaunchKernelGGL(k_mix_direct_global, sgrid, dim3(256), 0, ctx->stream, A);
    }
  } else {
    if (ctx->rpw) {
      launch_tile_mix<STAT>(ctx, A);
    } else {
      hipLaunchKernelGGL(k_mix_direct_global, sgrid, dim3(256), 0, ctx->stream, A);
      if (needs_stat) {
        int64_t blocks = ((int64_t)A.nchunks + 3) / 4;
        int64_t cap = 32768 / A.n;
        if (cap < 64) cap = 64;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL((k_dense_stat<STAT == Q_NONE ? Q_SIGN : STAT>), dim3((unsigned)blocks, (unsigned)A.n),
                           dim3(256), 0, ctx->stream, A);
      }
    }
    if (needs_stat)
      hipLaunchKernelGGL((k_dense_finalise<STAT == Q_NONE ? Q_SIGN : STAT>), dim3((unsigned)A.n), dim3(256), 0,
                         ctx->stream, A);
    launch_dense_apply<COMP>(ctx, A, sgrid);
  }
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

// Sparsifying operators (top_a, random_a).
template <int COMP>
int gossip_sparse(choco_ctx* ctx) {
  const Args& A = ctx->args;
  const int32_t nvec = (A.d + 3) >> 2;
  const dim3 sgrid = stream_grid(nvec, A.n);
  const bool incremental = ctx->mix_form == CHOCO_MIX_INCREMENTAL_S;
  const bool mix_first = ctx->cfg.order == CHOCO_ORDER_MIX_THEN_COMPRESS;
  bool mixed = false;
  if (mix_first) {
    if (incremental && COMP == Q_TOPK) {
      // fused below into the first select pass
    } else if (incremental) {
      hipLaunchKernelGGL(k_mix_incremental, sgrid, dim3(256), 0, ctx->stream, A);
      mixed = true;
    } else {
      if (ctx->rpw) launch_tile_mix<Q_NONE>(ctx, A);
      else hipLaunchKernelGGL(k_mix_direct_global, sgrid, dim3(256), 0, ctx->stream, A);
      mixed = true;
    }
  }
  // select: histogram pass, digit 0, rebuild pass (no-op unless the guess failed), refine + emit
  dim3 pgrid = sgrid;
  if (mix_first && !mixed)
    hipLaunchKernelGGL((k_sel_pass<COMP, true, COMP == Q_TOPK>), pgrid, dim3(256), 0, ctx->stream, A);
  else
    hipLaunchKernelGGL((k_sel_pass<COMP, true, false>), pgrid, dim3(256), 0, ctx->stream, A);
  hipLaunchKernelGGL(k_sel_final0, dim3((unsigned)A.n), dim3(256), 0, ctx->stream, A);
  hipLaunchKernelGGL((k_sel_pass<COMP, false, false>), pgrid, dim3(256), 0, ctx->stream, A);
  hipLaunchKernelGGL((k_sel_refine<COMP>), dim3((unsigned)A.n), dim3(1024), 0, ctx->stream, A);
  // messages: neighbour sums first (they recompute q from x - xhat), then xhat
  const unsigned kblocks = (unsigned)((A.k + 255) / 256);
  if (incremental)
    hipLaunchKernelGGL(k_scatter_s, dim3(kblocks, (unsigned)ctx->maxdeg, (unsigned)A.n), dim3(256), 0,
                       ctx->stream, A);
  hipLaunchKernelGGL(k_xhat_update, dim3(kblocks, (unsigned)A.n), dim3(256), 0, ctx->stream, A);
  if (!mix_first) {
    if (incremental) hipLaunchKernelGGL(k_mix_incremental, sgrid, dim3(256), 0, ctx->stream, A);
    else if (ctx->rpw) launch_tile_mix<Q_NONE>(ctx, A);
    else hipLaunchKernelGGL(k_mix_direct_global, sgrid, dim3(256), 0, ctx->stream, A);
  }
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

}  // namespace

extern "C" {

const char* choco_strerror(int code) {
  switch (code) {
    case CHOCO_OK: return "ok";
    case CHOCO_E_INVAL: return "invalid argument";
    case CHOCO_E_NOMEM: return "workspace too small or out of host memory";
    case CHOCO_E_HIP: return "HIP runtime error";
    case CHOCO_E_UNSUPPORTED: return "combination not implemented";
    default: return "unknown error";
  }
}

int choco_workspace_bytes(const choco_config* cfg, size_t* bytes_host) {
  if (!bytes_host) return CHOCO_E_INVAL;
  const int rc = check_scalars(cfg);
  if (rc != CHOCO_OK) return rc;
  if (!cfg->row_ptr_host) return CHOCO_E_INVAL;
  const int32_t nnz = cfg->row_ptr_host[cfg->n];
  if (nnz < cfg->n) return CHOCO_E_INVAL;
  *bytes_host = make_layout(*cfg, nnz).total;
  return CHOCO_OK;
}

int choco_init(const choco_config* cfg, float* x_dev, void* workspace_dev, size_t workspace_bytes,
               choco_ctx** out) {
  if (out) *out = nullptr;
  if (!out || !x_dev || !workspace_dev) return CHOCO_E_INVAL;
  int rc = check_scalars(cfg);
  if (rc != CHOCO_OK) return rc;
  if (((uintptr_t)x_dev & 15u) != 0 || ((uintptr_t)workspace_dev & (kAlign - 1)) != 0) return CHOCO_E_INVAL;
  int32_t nnz = 0, maxdeg = 0;
  rc = check_csr(cfg, &nnz, &maxdeg);
  if (rc != CHOCO_OK) return rc;
  const Layout L = make_layout(*cfg, nnz);
  if (workspace_bytes < L.total) return CHOCO_E_NOMEM;

  choco_ctx* ctx = new (std::nothrow) choco_ctx();
  if (!ctx) return CHOCO_E_NOMEM;
  ctx->cfg = *cfg;
  ctx->cfg.row_ptr_host = nullptr;
  ctx->cfg.col_idx_host = nullptr;
  ctx->cfg.w_host = nullptr;
  ctx->stream = (hipStream_t)cfg->stream;
  ctx->maxdeg = maxdeg;
  ctx->nnz = nnz;
  ctx->sparse = is_sparse(cfg->compressor);
  ctx->mix_form = resolve_mix_form(*cfg);
  ctx->rpw = pick_rpw(cfg->n);
  ctx->t = 0;
  ctx->last_hip_error = 0;
  ctx->destroyed = false;

  char* base = (char*)workspace_dev;
  Args& A = ctx->args;
  std::memset(&A, 0, sizeof(A));
  A.n = cfg->n;
  A.d = (int32_t)cfg->d;
  A.ld = resolve_ld(*cfg);
  A.X = x_dev;
  A.Xhat = (float*)(base + L.xhat);
  A.S = ctx->mix_form == CHOCO_MIX_INCREMENTAL_S ? (float*)(base + L.s) : nullptr;
  A.row_ptr = (const int32_t*)(base + L.row_ptr);
  A.col = (const int32_t*)(base + L.col);
  A.w = (const float*)(base + L.w);
  A.ctl = (WorkerCtl*)(base + L.ctl);
  A.gamma = cfg->gamma;
  A.partial = (double*)(base + L.partial);
  A.nchunks = L.nchunks;
  A.levels = cfg->levels;
  A.tau = 1.0;
  if (cfg->compressor == CHOCO_Q_QSGD && cfg->qsgd_biased) {
    const double s = (double)cfg->levels, dd = (double)cfg->d;
    A.tau = 1.0 + std::min(dd / (s * s), std::sqrt(dd) / s);
  }
  A.codes = nullptr;
  A.k = ctx->sparse ? cfg->k : 0;
  A.hist = (uint32_t*)(base + L.hist);
  A.cand = (uint2*)(base + L.cand);
  A.cand_cap = L.cand_cap;
  A.sel_idx = (int32_t*)(base + L.sel_idx);
  A.sel_val = (float*)(base + L.sel_val);
  A.bitmap = (uint32_t*)(base + L.bitmap);
  A.bitmap_words = L.bitmap_words;
  A.randk_rescale = cfg->randk_rescale ? 1 : 0;
  A.randk_scale = ctx->sparse ? (float)((double)cfg->d / (double)cfg->k) : 1.0f;
  A.seed_lo = (uint32_t)(cfg->seed & 0xFFFFFFFFu);
  A.seed_hi = (uint32_t)(cfg->seed >> 32);
  ctx->metrics_part = (double*)(base + L.mpart);
  ctx->metrics_out = (double*)(base + L.mout);
  ctx->metrics_blocks = kMetricsBlocks;

  // zero everything but the caller's X: xhat^(0) = 0, S = 0, counters, histograms, bitmap
  hipError_t e = hipMemsetAsync(workspace_dev, 0, L.total, ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(base + L.row_ptr, cfg->row_ptr_host, (size_t)(cfg->n + 1) * sizeof(int32_t),
                       hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(base + L.col, cfg->col_idx_host, (size_t)nnz * sizeof(int32_t),
                       hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(base + L.w, cfg->w_host, (size_t)nnz * sizeof(float), hipMemcpyHostToDevice,
                       ctx->stream);
  std::vector<WorkerCtl> ctl0;
  if (e == hipSuccess) {
    ctl0.resize((size_t)cfg->n);
    std::memset(ctl0.data(), 0, ctl0.size() * sizeof(WorkerCtl));
    for (auto& c : ctl0) c.guess_bin = c.guess_next = (uint32_t)kBins;  // no guess yet
    e = hipMemcpyAsync(base + L.ctl, ctl0.data(), ctl0.size() * sizeof(WorkerCtl), hipMemcpyHostToDevice,
                       ctx->stream);
  }
  // the host buffers above are pageable: wait until the copies have read them
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) {
    delete ctx;
    return CHOCO_E_HIP;
  }
  *out = ctx;
  return CHOCO_OK;
}

int choco_gossip_step(choco_ctx* ctx) {
  if (!ctx || ctx->destroyed) return CHOCO_E_INVAL;
  Args& A = ctx->args;
  A.t_lo = (uint32_t)(ctx->t & 0xFFFFFFFFu);
  A.t_hi = (uint32_t)(ctx->t >> 32);
  int rc;
  switch (ctx->cfg.compressor) {
    case CHOCO_Q_IDENTITY: rc = gossip_dense<Q_IDENTITY>(ctx); break;
    case CHOCO_Q_SIGN: rc = gossip_dense<Q_SIGN>(ctx); break;
    case CHOCO_Q_QSGD: rc = gossip_dense<Q_QSGD>(ctx); break;
    case CHOCO_Q_TOPK: rc = gossip_sparse<Q_TOPK>(ctx); break;
    case CHOCO_Q_RANDK: rc = gossip_sparse<Q_RANDK>(ctx); break;
    default: rc = CHOCO_E_INVAL;
  }
  if (rc == CHOCO_OK) ctx->t += 1;
  return rc;
}

int choco_sgd_step(choco_ctx* ctx, const float* g_dev, float lr) {
  if (!ctx || ctx->destroyed || !g_dev || ((uintptr_t)g_dev & 15u) != 0) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  const int32_t nvec = (A.d + 3) >> 2;
  hipLaunchKernelGGL(k_sgd, stream_grid(nvec, A.n), dim3(256), 0, ctx->stream, A.X, g_dev, A.ld, nvec, lr);
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

int choco_momentum_step(choco_ctx* ctx, const float* g_dev, float* m_dev, float lr, float beta,
                        float lambda) {
  if (!ctx || ctx->destroyed || !g_dev || !m_dev) return CHOCO_E_INVAL;
  if (((uintptr_t)g_dev & 15u) != 0 || ((uintptr_t)m_dev & 15u) != 0) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  const int32_t nvec = (A.d + 3) >> 2;
  hipLaunchKernelGGL(k_momentum, stream_grid(nvec, A.n), dim3(256), 0, ctx->stream, A.X, g_dev, m_dev,
                     A.ld, nvec, lr, beta, lambda);
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

int choco_metrics(choco_ctx* ctx, double* consensus_host, double* mean_norm_host, double* psi_host) {
  if (!ctx || ctx->destroyed) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  int blocks = (A.d + 255) / 256;
  if (blocks > ctx->metrics_blocks) blocks = ctx->metrics_blocks;
  hipLaunchKernelGGL(k_metrics_partial, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, A,
                     ctx->metrics_part);
  hipLaunchKernelGGL(k_metrics_final, dim3(1), dim3(64), 0, ctx->stream, ctx->metrics_part, blocks,
                     ctx->metrics_out);
  LAUNCH_CHECK(ctx);
  double out[3];
  HIP_TRY(ctx, hipMemcpyAsync(out, ctx->metrics_out, sizeof(out), hipMemcpyDeviceToHost, ctx->stream));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  if (consensus_host) *consensus_host = out[0] / (double)A.n;
  if (mean_norm_host) *mean_norm_host = std::sqrt(out[1]);
  if (psi_host) *psi_host = out[0] + out[2];
  return CHOCO_OK;
}

int choco_xhat(choco_ctx* ctx, float** xhat_dev) {
  if (!ctx || ctx->destroyed || !xhat_dev) return CHOCO_E_INVAL;
  *xhat_dev = ctx->args.Xhat;
  return CHOCO_OK;
}

int choco_nsum(choco_ctx* ctx, float** s_dev) {
  if (!ctx || ctx->destroyed || !s_dev) return CHOCO_E_INVAL;
  *s_dev = ctx->args.S;
  return CHOCO_OK;
}

int choco_last_selection(choco_ctx* ctx, int32_t* idx_dev, float* val_dev) {
  if (!ctx || ctx->destroyed || !ctx->sparse) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  const size_t count = (size_t)A.n * (size_t)A.k;
  if (idx_dev)
    HIP_TRY(ctx, hipMemcpyAsync(idx_dev, A.sel_idx, count * sizeof(int32_t), hipMemcpyDeviceToDevice,
                                ctx->stream));
  if (val_dev)
    HIP_TRY(ctx, hipMemcpyAsync(val_dev, A.sel_val, count * sizeof(float), hipMemcpyDeviceToDevice,
                                ctx->stream));
  return CHOCO_OK;
}

int choco_set_capture(choco_ctx* ctx, int32_t* codes_dev) {
  if (!ctx || ctx->destroyed) return CHOCO_E_INVAL;
  if (ctx->cfg.compressor != CHOCO_Q_SIGN && ctx->cfg.compressor != CHOCO_Q_QSGD) return CHOCO_E_INVAL;
  if (((uintptr_t)codes_dev & 15u) != 0) return CHOCO_E_INVAL;
  ctx->args.codes = codes_dev;
  return CHOCO_OK;
}

int choco_last_scalars(choco_ctx* ctx, double* scalars_host) {
  if (!ctx || ctx->destroyed || !scalars_host) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  std::vector<WorkerCtl> ctl((size_t)A.n);
  HIP_TRY(ctx, hipMemcpyAsync(ctl.data(), A.ctl, ctl.size() * sizeof(WorkerCtl), hipMemcpyDeviceToHost,
                              ctx->stream));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  for (int i = 0; i < A.n; ++i) {
    double* o = scalars_host + 4 * i;
    const WorkerCtl& c = ctl[(size_t)i];
    o[0] = o[1] = o[2] = o[3] = 0.0;
    switch (ctx->cfg.compressor) {
      case CHOCO_Q_SIGN: o[0] = c.stat; o[1] = (double)c.scale_c; break;
      case CHOCO_Q_QSGD: o[0] = c.stat; o[1] = c.nrm; o[2] = (double)c.scale_r; o[3] = (double)c.scale_step; break;
      case CHOCO_Q_TOPK:
      case CHOCO_Q_RANDK:
        o[0] = (double)(uint32_t)(c.kstar >> 32);
        o[1] = (double)(uint32_t)(~(uint32_t)(c.kstar & 0xFFFFFFFFu));
        o[2] = (double)c.kept;
        o[3] = (double)c.mode;
        break;
      default: break;
    }
  }
  return CHOCO_OK;
}

int choco_get_step(choco_ctx* ctx, uint64_t* t_host) {
  if (!ctx || ctx->destroyed || !t_host) return CHOCO_E_INVAL;
  *t_host = ctx->t;
  return CHOCO_OK;
}

int choco_set_step(choco_ctx* ctx, uint64_t t) {
  if (!ctx || ctx->destroyed) return CHOCO_E_INVAL;
  ctx->t = t;
  return CHOCO_OK;
}

int choco_sync(choco_ctx* ctx) {
  if (!ctx || ctx->destroyed) return CHOCO_E_INVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  return CHOCO_OK;
}

int choco_destroy(choco_ctx* ctx) {
  if (!ctx) return CHOCO_OK;
  ctx->destroyed = true;
  delete ctx;
  return CHOCO_OK;
}

int choco_last_hip_error(choco_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

}  // extern "C"
