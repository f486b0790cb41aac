// Host side of the C ABI declared in include/choco.h: argument checks, workspace
// layout, kernel launches.  No device memory is allocated here; everything lives
// in the caller's workspace.  No call synchronises unless the header says so.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "choco.h"
#include "choco_kernels.h"
#include "choco_layers.h"
#include "choco_wire.h"

using namespace choco;

// How the guessed-threshold select (Appendix C: top_a, random_a) is run on one "row" of d
// entries of which k are kept: the whole vector, or one long layer of it.
struct SelectPlan {
  int64_t d, k;
  uint32_t cand_cap, seg_cap;          // candidate list: aimed-at total and capacity of a sub-list
  uint32_t extra, want, delta0;        // see Args
  uint32_t guess0, shift0;             // first guess and bin width (all ones: none, the first step falls back)
  uint32_t sample_stride, sample_need; // fallback histogram
  bool multipart;                      // long candidate lists: three multi-block launches instead of one block
  bool fallback_chain;                 // long rows: histogram passes repair a failed guess (else a row scan)
};

// A layer too long for the register-resident layer kernel: it takes the select chain of the
// whole-vector path on its own piece of the rows.
struct LongLayer {
  int32_t start, len, k, sel_base, id;
  SelectPlan plan;
  LongSel sel;      // what the kernels need of it (filled by choco_init)
  bool batched;     // its pass and its select share a launch with those of the other such layers
};

// random_a selects ahead in batches of up to this many steps (two event operations on the
// caller's stream per batch instead of per step: they cost 11 us of idle queue each time, n = 64,
// d = 270 k).  Rows above 2^21 entries take batches of one step: there the event operations do
// not show, and four candidate passes in a row (0.25 ms of Philox arithmetic each) beside the
// first step of a batch slow its bandwidth-bound pass more than they save (n = 8, 31.8 M
// entries in 14 layers: 0.877 against 0.927 ms per step).
constexpr int kAheadSteps = 4;
constexpr int kAheadBufs = 2 * kAheadSteps;
struct AheadBatch {
  uint64_t base;   // selections of steps base .. base + (batch length) - 1
  bool valid;
};

// Partial sums of choco_metrics_noalloc: the same three doubles per block that choco_metrics
// keeps in the caller's workspace, here in device memory that belongs to the loaded library
// (24 KiB on every GPU the library runs on, until the process ends).  In host code this name
// is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr int kNoAllocBlocks = 1024;
static __device__ __align__(256) double scratch[kNoAllocBlocks * 3];
static_assert(sizeof(double) * kNoAllocBlocks * 3 == CHOCO_NOALLOC_SCRATCH_BYTES, "header states the size of the array");

struct choco_ctx {
  choco_config cfg;       // scalar fields as given (host CSR pointers are not kept)
  Args args;              // kernel arguments (device pointers into the workspace)
  hipStream_t stream;
  // random_a: the mask of a step depends on (seed, step, worker) only, so while the steps of one
  // batch (ahead_steps of them) run on the caller's stream the selections of the NEXT batch
  // already run on this one.  2 * ahead_steps copies of the kept-index lists and of the bitmap
  // take turns: step t uses copy t mod (2 * ahead_steps).
  hipStream_t aux_stream;
  hipStream_t launch_stream;   // where LAUNCH puts kernels: the caller's stream, or aux_stream while selecting ahead
  hipEvent_t ev_fork, ev_ahead;
  // layer tables: a selection made ahead is several short chains of launches that do not depend
  // on one another (the layers that share launches, those with launches of their own, the layer
  // kernel); on one stream they wait for each other and the whole takes longer than the step
  // beside it, so half of them goes to a third stream, forked from and joined to aux_stream
  hipStream_t aux_stream2;
  hipEvent_t ev_fork2, ev_join2;
  bool split_ahead;       // between that fork and join
  bool lookahead;         // the configuration allows it and it has not been switched off
  bool can_lookahead;     // the configuration allows it (random_a)
  bool ahead_pending;     // the batch `nxt` is in flight (or done) on aux_stream and not yet joined
  AheadBatch cur, nxt;    // the batch whose selections the steps are using / the one selected beside them
  int ahead_steps;        // steps per batch: kAheadSteps, or 1 for long rows; step t uses copy t mod (2 * ahead_steps)
  int32_t* sel_idx_buf[kAheadBufs];
  uint32_t* bitmap_buf[kAheadBufs];
  uint32_t* keptmap_buf[kAheadBufs];
  double* layer_scal_buf[kAheadBufs];
  uint32_t dirty_maps;    // rows without an LDS bitmap: the bit-map copies that hold a selection made ahead and not yet used
  int last_buf;           // which copy the last finished step used
  int32_t maxdeg;
  int32_t nnz;
  bool sparse;            // top_a / random_a
  bool fused_sparse_apply;   // ... whose update of xhat rides on the tile mix pass (direct form, compress-then-mix)
  bool values_in_qv;      // random_a after such a step: the kept values are in Qv, not yet in the list
  int mix_form;           // resolved: CHOCO_MIX_INCREMENTAL_S or CHOCO_MIX_DIRECT
  int rpw;                // rows per wave of the tile kernels, 0 = tile does not fit
  bool fused;             // the step being enqueued carries the local update in its first pass
  bool multipart;         // long candidate lists: the select runs as three multi-block launches
  bool fallback_chain;    // long rows: a failed guess is repaired by the histogram passes, not a row scan
  bool nt;                // non-temporal loads/stores: the state does not fit in cache anyway
  int nlayers;            // > 0: the operator is applied layer by layer
  bool layers_generic;    // ... on a table that is not aligned (see layers_aligned): no pass carries the local update
  int nmid, nsmall;       // layers (by falling length, after the long ones) that take a 1024- / a 256-thread workgroup
  SelectPlan plan;        // whole-vector top_a / random_a
  std::vector<LongLayer> long_layers;   // top_a / random_a layer by layer: layers above CHOCO_MAX_LAYER_LEN
  const LongSel* long_tab;   // device copy of the batched ones' LongSel, in the order of long_layers
  int nbatched;           // how many those are, and the 4-vectors of the longest of them
  int32_t batched_nvec;
  bool long_silent;       // one of them keeps nothing (its pass cannot carry the local update)
  bool overlap_long;      // top_a, several long layers with launches of their own: a layer's select runs on the second stream beside the next layer's pass
  size_t set_hist16, set_cand, set_hist_parts, set_small_list;   // bytes from one long layer's select scratch to the next
  bool long_rows;         // d > 2^21: four 4-vectors per thread in the streaming kernels
  uint64_t t;             // step counter
  uint32_t* wire_rank;    // random_a without a bitmap: n x ceil(ld / 1024) chunk ranks of the message encoder
  uint64_t last_t;        // step counter the last finished gossip step ran with (tags what it remembered)
  const int64_t* wire_word_off;   // layer by layer: where each layer's message starts / prefix of plane lengths
  const int64_t* wire_plane_off;
  int64_t wire_words, wire_plane_words;
  int device;             // the GPU that was current in choco_init
  double* noalloc_scratch;   // address of `scratch` on that GPU (null: more GPUs than the table holds)
  double* metrics_part;   // device scratch of the metrics kernels
  double* metrics_out;
  int metrics_blocks;
  int last_hip_error;
  // optional per-kernel timing with HIP events on the context's stream
  bool profiling;
  std::vector<hipEvent_t> ev_begin, ev_end;
  std::vector<int> ev_kernel;
  size_t ev_used;
};

namespace {

constexpr size_t kAlign = 256;
constexpr int kMetricsBlocks = 1024;
constexpr int kMaxTileRows = 64;  // n * 1 KiB of LDS for the tile of all rows

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t xhat, s, row_ptr, col, w, ctl, chunk_sums, group_sums, hist16, cand, hist_parts, small_list, sel_idx, sel_val, keptmap, bitmap,
      layers, layer_work, long_tab, layer_guess, layer_scal, layer_groups, layer_group_first, layer_group_sums, layer_scale,
      chunk_layer, planes, ovf_ring, ovf_pos, wire_rank, wire_word_off, wire_plane_off, sel_idx2, bitmap2, keptmap2, layer_scal2, qv, mpart, mout, total;
  int64_t wire_words, wire_plane_words;   // layer by layer: words of a worker's message / of one bit plane
  int32_t ngroup_items;
  uint32_t cand_cap, seg_cap;
  int64_t bitmap_words;
  bool multipart;
  int32_t select_sets;   // copies of the select scratch (candidate lists, histograms, short list)
  size_t hist16_bytes, cand_bytes, hist_parts_bytes, small_list_bytes;   // size of one copy
  size_t sel_idx_bytes, bitmap_bytes, keptmap_bytes, layer_scal_bytes;   // ... of what a selection made ahead writes
  int32_t nchunks, ngroups;
};

bool is_sparse(int compressor) { return compressor == CHOCO_Q_TOPK || compressor == CHOCO_Q_RANDK; }

// CHOCO_MIX_AUTO.  Dense operators: the direct form (the tile kernels, or rows read from global
// memory).  top_a / random_a: the direct form too wherever the LDS tile of all n rows exists
// (n <= kMaxTileRows) - one fused pass then applies the sparse update of xhat and the mix, no S
// array, no scatter: measured faster at every size (n = 64, d = 270 k: 0.101 against 0.118 ms
// before the passes were fused; n = 8, d = 28 M: 1.09 against 1.27 ms).  The incremental
// neighbour sums remain for more workers than the tile holds, for top_a in the printed order,
// where mix and candidate pass are one 20 B/entry pass over S, and for layer tables in the
// printed order (layer by layer only the fused pass is built for the direct form).
int resolve_mix_form(const choco_config& c) {
  if (c.mix_form != CHOCO_MIX_AUTO) return c.mix_form;
  if (!is_sparse(c.compressor)) return CHOCO_MIX_DIRECT;
  if (c.n > kMaxTileRows) return CHOCO_MIX_INCREMENTAL_S;
  if (c.nlayers > 0 && c.order == CHOCO_ORDER_MIX_THEN_COMPRESS) return CHOCO_MIX_INCREMENTAL_S;
  if (c.compressor == CHOCO_Q_TOPK && c.order == CHOCO_ORDER_MIX_THEN_COMPRESS) return CHOCO_MIX_INCREMENTAL_S;
  return CHOCO_MIX_DIRECT;
}

int64_t resolve_ld(const choco_config& c) { return c.ld == 0 ? (c.d + 3) / 4 * 4 : c.ld; }

// top_a / random_a, compress-then-mix order, direct form with the LDS tile: xhat += q is applied
// by the mix pass itself (k_tile_mix<.., SPARSE>), off the kept-entry bits.
bool fused_sparse_apply(const choco_config& c) {
  return is_sparse(c.compressor) && c.order == CHOCO_ORDER_COMPRESS_THEN_MIX &&
         resolve_mix_form(c) == CHOCO_MIX_DIRECT && c.n <= kMaxTileRows;
}

// Kept entries per worker and step: k, or the sum over the layers.
int64_t kept_per_worker(const choco_config& c) {
  if (!is_sparse(c.compressor)) return 0;
  if (c.nlayers <= 0) return c.k;
  int64_t sum = 0;
  for (int32_t l = 0; l < c.nlayers; ++l) sum += c.layer_k_host[l];
  return sum;
}

int check_layers(const choco_config* c) {
  if (c->nlayers < 0) return CHOCO_E_INVAL;
  if (c->nlayers == 0) return CHOCO_OK;
  if (!c->layer_start_host || !c->layer_len_host) return CHOCO_E_INVAL;
  const bool sparse = is_sparse(c->compressor);
  if (sparse && !c->layer_k_host) return CHOCO_E_INVAL;
  int64_t end = 0, ktot = 0;
  for (int32_t l = 0; l < c->nlayers; ++l) {
    const int64_t start = c->layer_start_host[l], len = c->layer_len_host[l];
    if (start < end || len < 1) return CHOCO_E_INVAL;   // disjoint, ascending, not empty
    end = start + len;
    if (end > c->d) return CHOCO_E_INVAL;
    if (sparse) {
      const int64_t k = c->layer_k_host[l];
      if (k < 0 || k > len) return CHOCO_E_INVAL;
      ktot += k;
    }
  }
  if (sparse && ktot < 1) return CHOCO_E_INVAL;
  if (c->compressor == CHOCO_Q_IDENTITY) return CHOCO_E_UNSUPPORTED;
  // sign / gsgd layer by layer: the direct form only (what AUTO gives them); top_a / random_a:
  // incremental sums, or the direct form where its fused pass exists
  if (!sparse && c->mix_form != CHOCO_MIX_AUTO) return CHOCO_E_UNSUPPORTED;
  if (sparse && c->mix_form == CHOCO_MIX_DIRECT && !fused_sparse_apply(*c)) return CHOCO_E_UNSUPPORTED;
  return CHOCO_OK;
}

// A layer table is "aligned" if every layer starts on a multiple of 4, the layers follow one
// another with only the padding to the next multiple of 4 between them, and they cover the
// vector: a 16-byte 4-vector then never spans two layers and the layer passes can carry the
// local update.  Any other table (layers that start anywhere, gaps, a vector that goes on
// after the last layer) takes the generic paths: per-entry layer look-ups, entry-wise loads
// where a layer's norm tree starts off a 16-byte boundary, the local update as its own pass.
bool layers_aligned(const choco_config& c) {
  int64_t expect = 0, end = 0;
  for (int32_t l = 0; l < c.nlayers; ++l) {
    if (c.layer_start_host[l] != expect) return false;
    end = expect + c.layer_len_host[l];
    expect = (end + 3) / 4 * 4;
  }
  return end == c.d;
}

// Scalar-field validation shared by choco_workspace_bytes and choco_init.
int check_scalars(const choco_config* c) {
  if (!c) return CHOCO_E_INVAL;
  // (the kernels index entries and 4-vectors of a row in int32 and step by up to 2^18 entries)
  if (c->n < 1 || c->d < 1 || c->d > CHOCO_MAX_D) return CHOCO_E_INVAL;
  if (c->n > 65535) return CHOCO_E_UNSUPPORTED;   // workers are a grid dimension of the launches
  const int64_t ld = resolve_ld(*c);
  if (ld < c->d || (ld & 3) != 0) return CHOCO_E_INVAL;
  if (!(c->gamma > 0.0f) || !std::isfinite(c->gamma)) return CHOCO_E_INVAL;
  if (c->compressor < CHOCO_Q_IDENTITY || c->compressor > CHOCO_Q_QSGD) return CHOCO_E_INVAL;
  if (is_sparse(c->compressor) && c->nlayers == 0 && (c->k < 1 || c->k > c->d)) return CHOCO_E_INVAL;
  if (c->compressor == CHOCO_Q_QSGD && c->levels < 1) return CHOCO_E_INVAL;
  if (c->order != CHOCO_ORDER_COMPRESS_THEN_MIX && c->order != CHOCO_ORDER_MIX_THEN_COMPRESS)
    return CHOCO_E_INVAL;
  if (c->mix_form < CHOCO_MIX_AUTO || c->mix_form > CHOCO_MIX_DIRECT) return CHOCO_E_INVAL;
  // combinations this build does not implement
  if (!is_sparse(c->compressor) && resolve_mix_form(*c) == CHOCO_MIX_INCREMENTAL_S)
    return CHOCO_E_UNSUPPORTED;
  return check_layers(c);
}

// Candidates wanted beyond k so that the guess survives the step-to-step drift of the
// threshold (top_a) or the binomial spread of the count (random_a).
double extra_candidates(int64_t k) {
  const double kk = (double)k;
  return std::min(std::max(0.5 * kk, 6.0 * std::sqrt(kk) + 32.0), 2147483647.0);
}

// Entries the guess aims to leave above it beyond the k kept ones.  top_a: the k entries
// kept in a step are absorbed by xhat and drop out, so the next step's k largest are (about)
// this step's ranks k+1..2k; random_a draws afresh every step.
double want_candidates(int compressor, int64_t k) {
  return extra_candidates(k) + (compressor == CHOCO_Q_TOPK ? (double)k : 0.0);
}

double expected_candidates(int compressor, int64_t k) { return (double)k + want_candidates(compressor, k); }

SelectPlan plan_select(int compressor, int64_t d, int64_t k) {
  SelectPlan P{};
  P.d = d;
  P.k = k;
  int64_t cap = 4 * k;
  if (cap < d / 128) cap = d / 128;
  if (cap < 8192) cap = 8192;
  if (cap > d) cap = d;
  P.cand_cap = (uint32_t)cap;
  // sub-lists: block b of a worker appends to sub-list b % kSegs; each gets twice its even
  // share of the capacity, but never more than the blocks feeding it can produce
  const int64_t per_block = 256 * kCompactVecs * 4;   // (short rows use half-size blocks: the bound below still holds)
  const int64_t nblocks = (d + per_block - 1) / per_block;
  const int64_t feeders = (nblocks + kSegs - 1) / kSegs;
  int64_t seg_cap = std::max<int64_t>((2 * cap + kSegs - 1) / kSegs, 1024);
  seg_cap = std::min<int64_t>(seg_cap, feeders * per_block);
  P.seg_cap = (uint32_t)seg_cap;
  P.multipart = expected_candidates(compressor, k) > 16384.0;
  // A failed guess (first step, or the distribution moved) is repaired by three extra passes
  // (sampled histogram, new guess, rebuild) that are launched every step and normally exit at
  // once.  For short rows even those idle launches show, and the select kernel's own row scan
  // (one block per worker) is quick enough, so they are left out.
  P.fallback_chain = d > ((int64_t)1 << 21);
  const double kk = (double)k, dd = (double)d;
  const double extra = extra_candidates(k);
  P.extra = (uint32_t)extra;
  P.want = (uint32_t)std::min(want_candidates(compressor, k), 4294967295.0);
  P.guess0 = 0xFFFFFFFFu;   // top_a: no guess yet, the first step takes the fallback
  P.shift0 = 0;
  if (compressor == CHOCO_Q_RANDK) {
    // keys are uniform on [0, 2^32): the k + extra largest start near (1 - (k+extra)/d) 2^32
    const double frac = std::min(1.0, (kk + extra) / dd);
    const double g = (1.0 - frac) * 4294967296.0;
    P.guess0 = g <= 0.0 ? 0u : (uint32_t)std::min(g, 4294967295.0);
    // 2048 candidate bins over the keys above the guess
    const uint64_t range = 4294967296ull - (uint64_t)P.guess0;
    while ((range >> P.shift0) > (uint64_t)kBins) ++P.shift0;
    const double d0 = std::min(extra / dd, 1.0) * 4294967296.0;
    P.delta0 = (uint32_t)std::min(std::max(d0, 1.0), 4294967295.0);
  } else {
    P.delta0 = 1u << 19;   // about 6 % in magnitude
  }
  // fallback histogram: aim the rebuilt list at max(2k + extra, capacity / 4), at most
  // half the capacity, and sample the row so that the aim is still >= ~2000 samples
  double aim = std::max(2.0 * kk + extra, 0.25 * (double)P.cand_cap);
  aim = std::min(aim, std::max(0.5 * (double)P.cand_cap, kk));
  uint32_t stride = 1;
  if (d > (1 << 21)) {
    stride = 16;
    while (stride > 1 && aim / stride < 2048.0) stride >>= 1;
  }
  P.sample_stride = stride;
  P.sample_need = (uint32_t)std::max(1.0, std::ceil(aim / stride));
  return P;
}

// The layers of a top_a / random_a configuration that are too long for the layer kernel.
std::vector<LongLayer> long_layers_of(const choco_config& c) {
  std::vector<LongLayer> out;
  if (c.nlayers <= 0 || !is_sparse(c.compressor)) return out;
  int64_t sel_base = 0;
  for (int32_t l = 0; l < c.nlayers; ++l) {
    const int64_t len = c.layer_len_host[l], k = c.layer_k_host[l];
    if (len + (c.layer_start_host[l] & 3) > kMidLayerLen) {   // (with the entries before it in its first 4-vector)
      LongLayer B{};
      B.start = (int32_t)c.layer_start_host[l];
      B.len = (int32_t)len;
      B.k = (int32_t)k;
      B.sel_base = (int32_t)sel_base;
      B.id = l;
      B.plan = plan_select(c.compressor, len, std::max<int64_t>(k, 1));
      // one block per worker finishes the select, no histogram passes: such layers share launches
      B.batched = k > 0 && !B.plan.multipart && !B.plan.fallback_chain;
      out.push_back(B);
    }
    sel_base += k;
  }
  return out;
}

// Put the plan's numbers into a kernel argument block.
void apply_plan(Args& A, const SelectPlan& P) {
  A.cand_cap = P.cand_cap;
  A.seg_cap = P.seg_cap;
  A.extra = P.extra;
  A.want = P.want;
  A.delta0 = P.delta0;
  A.sample_stride = P.sample_stride;
  A.sample_need = P.sample_need;
}

int magnitude_bits(int levels) {
  int mb = 0;
  for (int x = levels - 1; x > 0; x >>= 1) ++mb;
  return mb < 1 ? 1 : mb;
}

// 32-bit words of one worker's message in the layout of choco_wire.h.
int64_t message_words(int compressor, int64_t d, int64_t k, int levels) {
  const int64_t W = (d + 31) / 32;
  switch (compressor) {
    case CHOCO_Q_TOPK: return 2 * k;
    case CHOCO_Q_RANDK: return k;
    case CHOCO_Q_SIGN: return 1 + W;
    case CHOCO_Q_QSGD: return 1 + kOverflowSlots + (int64_t)(1 + magnitude_bits(levels)) * W;
    default: return -1;
  }
}

Layout make_layout(const choco_config& c, int32_t nnz) {
  Layout L{};
  const int64_t ld = resolve_ld(c);
  const size_t state = (size_t)c.n * (size_t)ld * sizeof(float);
  const bool sparse = is_sparse(c.compressor);
  const bool layered = c.nlayers > 0;
  // selects by guessed threshold: the whole row, or every long layer in turn (they share the
  // candidate lists and histograms, each has control blocks of its own)
  const std::vector<LongLayer> longs = long_layers_of(c);
  const bool guessed = sparse && (!layered || !longs.empty());
  std::vector<SelectPlan> plans;
  if (sparse && !layered) plans.push_back(plan_select(c.compressor, c.d, c.k));
  for (const LongLayer& B : longs) plans.push_back(B.plan);
  const int64_t kept = kept_per_worker(c);
  size_t off = 0;
  auto take = [&off](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.xhat = take(state);
  L.s = take(resolve_mix_form(c) == CHOCO_MIX_INCREMENTAL_S ? state : 0);
  L.row_ptr = take((size_t)(c.n + 1) * sizeof(int32_t));
  L.col = take((size_t)nnz * sizeof(int32_t));
  L.w = take((size_t)nnz * sizeof(float));
  L.ctl = take((size_t)c.n * std::max<size_t>(1, longs.size()) * sizeof(WorkerCtl));
  L.nchunks = (int32_t)((c.d + kChunk - 1) / kChunk);
  L.ngroups = (L.nchunks + kGroup - 1) / kGroup;
  const bool dense_stat = c.compressor == CHOCO_Q_SIGN || c.compressor == CHOCO_Q_QSGD;
  // chunk sums are only materialised by the tile kernel of the printed order
  L.chunk_sums = take(dense_stat && c.order == CHOCO_ORDER_MIX_THEN_COMPRESS
                          ? (size_t)c.n * (size_t)L.nchunks * sizeof(double) : 0);
  L.group_sums = take(dense_stat ? (size_t)c.n * (size_t)L.ngroups * sizeof(double) : 0);
  int64_t cap = 0, seg_cap = 0;
  bool multipart = false;
  for (const SelectPlan& P : plans) {
    cap = std::max<int64_t>(cap, P.cand_cap);
    seg_cap = std::max<int64_t>(seg_cap, P.seg_cap);
    multipart = multipart || P.multipart;
  }
  L.cand_cap = (uint32_t)cap;
  L.seg_cap = (uint32_t)seg_cap;
  // a set of select scratch per long layer: the layers that share launches are selected at the
  // same time, and the select of one that has launches of its own can run (top_a, on the
  // library's second stream) beside the next layer's pass over the rows
  L.select_sets = std::max<int32_t>(1, (int32_t)longs.size());
  bool chain = !layered;   // the histogram passes: long rows, whole-vector rows of any length
  for (const SelectPlan& P : plans) chain = chain || P.fallback_chain;
  L.hist16_bytes = align_up(guessed && chain ? (size_t)c.n * kBins16 * sizeof(uint32_t) : 0);
  L.cand_bytes = align_up(guessed ? (size_t)c.n * kSegs * (size_t)seg_cap * sizeof(uint2) : 0);
  L.hist16 = take(L.hist16_bytes * (size_t)L.select_sets);
  L.cand = take(L.cand_bytes * (size_t)L.select_sets);
  L.sel_idx = take(sparse ? (size_t)c.n * (size_t)kept * sizeof(int32_t) : 0);
  L.sel_val = take(sparse ? (size_t)c.n * (size_t)kept * sizeof(float) : 0);
  L.multipart = guessed && multipart;
  L.hist_parts_bytes = align_up(L.multipart ? (size_t)c.n * kRefineParts * kBins * sizeof(uint32_t) : 0);
  L.small_list_bytes = align_up(L.multipart ? (size_t)c.n * kSmallCap * sizeof(uint2) : 0);
  L.hist_parts = take(L.hist_parts_bytes * (size_t)L.select_sets);
  L.small_list = take(L.small_list_bytes * (size_t)L.select_sets);
  // kept entries: a bitmap per worker if it fits in the (single-block) select's LDS (40 KiB
  // beside its other arrays), else a bit per entry in global memory
  L.bitmap_words = (guessed && !layered && !L.multipart && c.d <= 40 * 1024 * 8) ? (c.d + 31) / 32 : 0;
  const size_t map_bytes = (size_t)c.n * (size_t)((ld + 31) / 32) * sizeof(uint32_t);   // a bit per entry
  L.keptmap = take(sparse && !L.bitmap_words ? map_bytes : 0);
  L.bitmap = take((size_t)c.n * (size_t)L.bitmap_words * sizeof(uint32_t));
  // further copies for the selections random_a makes ahead: the kept-index lists, the bitmap
  // (short rows in whole-vector mode) or the bit map in global memory, the per-layer scalars
  const bool ahead = c.compressor == CHOCO_Q_RANDK;
  const size_t more = c.d > ((int64_t)1 << 21) ? 1 : kAheadBufs - 1;   // (long rows select one step ahead)
  L.sel_idx_bytes = align_up((size_t)c.n * (size_t)kept * sizeof(int32_t));
  L.bitmap_bytes = align_up((size_t)c.n * (size_t)L.bitmap_words * sizeof(uint32_t));
  L.keptmap_bytes = align_up(map_bytes);
  L.layer_scal_bytes = align_up((size_t)c.n * (size_t)c.nlayers * 4 * sizeof(double));
  L.sel_idx2 = take(ahead ? more * L.sel_idx_bytes : 0);
  L.bitmap2 = take(ahead ? more * L.bitmap_bytes : 0);
  L.keptmap2 = take(ahead && !L.bitmap_words ? more * L.keptmap_bytes : 0);
  L.layer_scal2 = take(ahead && layered ? more * L.layer_scal_bytes : 0);
  L.layers = take((size_t)c.nlayers * sizeof(LayerDesc));
  L.layer_work = take((size_t)c.nlayers * sizeof(LayerDesc));
  L.long_tab = take(longs.size() * sizeof(LongSel));
  L.layer_guess = take((size_t)c.n * (size_t)c.nlayers * sizeof(uint32_t));
  L.layer_scal = take((size_t)c.n * (size_t)c.nlayers * 4 * sizeof(double));
  // sign / gsgd layer by layer: work items of the norm pass (groups of 16 chunks of one layer)
  const bool dense_layers = layered && dense_stat;
  int64_t items = 0;
  if (dense_layers)
    for (int32_t l = 0; l < c.nlayers; ++l) items += (c.layer_len_host[l] + kGroup * kChunk - 1) / (kGroup * kChunk);
  L.ngroup_items = (int32_t)items;
  L.layer_groups = take((size_t)items * sizeof(LayerGroup));
  L.layer_group_first = take(dense_layers ? (size_t)(c.nlayers + 1) * sizeof(int32_t) : 0);
  L.layer_group_sums = take((size_t)c.n * (size_t)items * sizeof(double));
  L.layer_scale = take(dense_layers ? (size_t)c.n * (size_t)c.nlayers * sizeof(LayerScale) : 0);
  L.chunk_layer = take(dense_layers ? (size_t)L.nchunks * sizeof(int4) : 0);
  // the message of a dense operator: bit planes written by the compress pass (sign: one plane;
  // gsgd: the sign plane and mb magnitude planes) and, for gsgd, the ring of entries at level s
  const size_t wire_units = (size_t)c.n * (size_t)(layered ? c.nlayers : 1);
  const int nplanes = c.compressor == CHOCO_Q_SIGN ? 1 : c.compressor == CHOCO_Q_QSGD ? 1 + magnitude_bits(c.levels) : 0;
  L.planes = take((size_t)c.n * (size_t)nplanes * (size_t)((ld + 31) / 32) * sizeof(uint32_t));
  L.ovf_ring = take(c.compressor == CHOCO_Q_QSGD ? wire_units * kOvfRing * sizeof(uint4) : 0);
  L.ovf_pos = take(c.compressor == CHOCO_Q_QSGD ? wire_units * sizeof(uint32_t) : 0);
  L.wire_rank = take(c.compressor == CHOCO_Q_RANDK && !L.bitmap_words
                         ? (size_t)c.n * (size_t)((ld + 1023) / 1024) * sizeof(uint32_t) : 0);
  L.wire_word_off = take(dense_layers ? (size_t)(c.nlayers + 1) * sizeof(int64_t) : 0);
  L.wire_plane_off = take(dense_layers ? (size_t)(c.nlayers + 1) * sizeof(int64_t) : 0);
  L.wire_words = L.wire_plane_words = 0;
  if (dense_layers)
    for (int32_t l = 0; l < c.nlayers; ++l) {
      L.wire_words += message_words(c.compressor, c.layer_len_host[l], 0, c.levels);
      L.wire_plane_words += (c.layer_len_host[l] + 31) / 32;
    }
  // random_a whose update of xhat rides on the fused mix pass: the kept values by entry
  L.qv = take(fused_sparse_apply(c) && c.compressor == CHOCO_Q_RANDK ? state : 0);
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
  if (ctx) {
    ctx->last_hip_error = (int)e;
    // an error between a fork and its join: later calls launch on the caller's stream again
    ctx->launch_stream = ctx->stream;
    ctx->split_ahead = false;
  }
  return CHOCO_E_HIP;
}

#define HIP_TRY(ctx, expr)                        \
  do {                                            \
    hipError_t e_ = (expr);                       \
    if (e_ != hipSuccess) return hip_fail(ctx, e_); \
  } while (0)

#define LAUNCH_CHECK(ctx) HIP_TRY(ctx, hipGetLastError())

// Every GPU holds its own copy of `scratch` at its own address: resolved once per device, with
// that device current, and kept.
constexpr int kMaxGpus = 64;
std::mutex g_scratch_mutex;
double* g_scratch_addr[kMaxGpus] = {nullptr};

hipError_t resolve_scratch(int* device_out, double** addr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  *device_out = dev;
  *addr_out = nullptr;
  if (dev < 0 || dev >= kMaxGpus) return hipSuccess;   // no table slot: the no-alloc call reports it
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_addr[dev] = (double*)p;
  }
  *addr_out = g_scratch_addr[dev];
  return hipSuccess;
}

// Frees the host-side objects of a context (its own stream and events; never device memory).
void release_ctx(choco_ctx* ctx) {
  if (ctx->aux_stream) {
    (void)hipStreamSynchronize(ctx->aux_stream);
    (void)hipStreamDestroy(ctx->aux_stream);
  }
  if (ctx->aux_stream2) {
    (void)hipStreamSynchronize(ctx->aux_stream2);
    (void)hipStreamDestroy(ctx->aux_stream2);
  }
  if (ctx->ev_fork2) (void)hipEventDestroy(ctx->ev_fork2);
  if (ctx->ev_join2) (void)hipEventDestroy(ctx->ev_join2);
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_ahead) (void)hipEventDestroy(ctx->ev_ahead);
  for (hipEvent_t e : ctx->ev_begin) (void)hipEventDestroy(e);
  for (hipEvent_t e : ctx->ev_end) (void)hipEventDestroy(e);
  delete ctx;
}

// The caller's stream waits for a look-ahead selection that is still in flight.
int join_lookahead(choco_ctx* ctx) {
  if (ctx->ahead_pending) {
    HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_ahead, 0));
    ctx->ahead_pending = false;
  }
  return CHOCO_OK;
}


enum KernelId {
  KID_SGD, KID_MOMENTUM, KID_DENSE_STAT, KID_GROUP_REDUCE, KID_DENSE_FINALISE, KID_DENSE_APPLY_MIX, KID_TILE_MIX,
  KID_DENSE_APPLY, KID_MIX_DIRECT_GLOBAL, KID_MIX_INCREMENTAL, KID_SEL_COMPACT, KID_SEL_FALLBACK,
  KID_SEL_REFINE, KID_SCATTER_S, KID_XHAT_UPDATE, KID_GATHER_VALUES, KID_SEL_VALUES, KID_SEL_HIST_PARTS, KID_SEL_EMIT_PARTS, KID_SEL_FINISH, KID_DENSE_STAT_SGD, KID_SEL_COMPACT_SGD, KID_TILE_MIX_SGD, KID_MIX_INCREMENTAL_SGD, KID_LAYER_COMPRESS, KID_LAYER_COMPRESS_SGD, KID_LAYER_STAT, KID_LAYER_STAT_SGD, KID_LAYER_FINALISE, KID_WIRE, KID_ZERO_WORDS, KID_COUNT
};
const char* const kKernelNames[KID_COUNT] = {
  "k_sgd", "k_momentum", "k_dense_stat", "k_group_reduce", "k_dense_finalise", "k_dense_apply_mix", "k_tile_mix",
  "k_dense_apply", "k_mix_direct_global", "k_mix_incremental", "k_sel_compact", "k_sel_fallback",
  "k_sel_refine", "k_scatter_s", "k_xhat_update", "k_gather_values", "k_sel_values", "k_sel_hist_parts", "k_sel_emit_parts", "k_sel_finish",
  "k_dense_stat_sgd", "k_sel_compact_sgd", "k_tile_mix_sgd", "k_mix_incremental_sgd",
  "k_layer_compress", "k_layer_compress_sgd", "k_layer_stat", "k_layer_stat_sgd", "k_layer_finalise", "k_wire",
  "k_zero_words"};
constexpr size_t kMaxProfiledLaunches = 16384;

// Brackets one launch with two events when profiling is on (no-op otherwise).
struct Timed {
  choco_ctx* ctx;
  size_t slot;
  bool on;
  Timed(choco_ctx* c, int kid) : ctx(c), slot(0), on(false) {
    if (!c->profiling || c->launch_stream != c->stream || c->ev_used >= kMaxProfiledLaunches) return;
    if (c->ev_used == c->ev_begin.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return;
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
      c->ev_begin.push_back(a);
      c->ev_end.push_back(b);
      c->ev_kernel.push_back(kid);
    }
    slot = c->ev_used++;
    c->ev_kernel[slot] = kid;
    on = hipEventRecord(c->ev_begin[slot], c->stream) == hipSuccess;
  }
  ~Timed() {
    if (on) (void)hipEventRecord(ctx->ev_end[slot], ctx->stream);
  }
};
// LAUNCH(ctx, kernel id, kernel, grid, block, dynamic LDS bytes, kernel arguments...)
#define LAUNCH(ctx, kid, kernel, grid, block, lds, ...)                              \
  do {                                                                               \
    Timed timed_(ctx, kid);                                                          \
    hipLaunchKernelGGL(kernel, grid, block, lds, (ctx)->launch_stream, __VA_ARGS__); \
  } while (0)

// One block per 256 * vecs consecutive 4-vectors of a row, one grid row per worker.
dim3 chunk_grid(int32_t nvec, int32_t n, int vecs) {
  const int64_t per_block = 256 * (int64_t)vecs;
  return dim3((unsigned)(((int64_t)nvec + per_block - 1) / per_block), (unsigned)n, 1);
}

// Tile kernels: waves per block (8 up to 8 workers - a row per wave measured 4 % faster than
// two -, 4 up to 16, else 16) and rows per wave.  (n = 64 with 8-wave workgroups of 8 rows per
// wave, which leave half of a compute unit's wave slots free: the mix pass 55 against 43 us.)
int pick_rpw(int n) {
  if (n > kMaxTileRows) return 0;
  const int nw = n <= 8 ? 8 : n <= 16 ? 4 : 16;
  const int rows = (n + nw - 1) / nw;
  return rows <= 1 ? 1 : rows <= 2 ? 2 : 4;
}

#define TILE_SWITCH(n, rpw, CALL)                      \
  if ((n) <= 8) {                                      \
    CALL(1, 8);                                        \
  } else if ((n) <= 16) {                                     \
    switch (rpw) {                                     \
      case 1: CALL(1, 4); break;                       \
      case 2: CALL(2, 4); break;                       \
      default: CALL(4, 4); break;                      \
    }                                                  \
  } else {                                             \
    switch (rpw) {                                     \
      case 1: CALL(1, 16); break;                      \
      case 2: CALL(2, 16); break;                      \
      default: CALL(4, 16); break;                     \
    }                                                  \
  }

template <int COMP, bool CAPTURE, bool NT, bool LAYERED = false>
void launch_apply_mix(choco_ctx* ctx, const Args& A) {
  const dim3 grid((unsigned)A.nchunks), block(A.n <= 8 ? 512 : A.n <= 16 ? 256 : 1024);
  const size_t lds = (size_t)A.n * kChunk * sizeof(float);
#define CALL(R, W) \
  LAUNCH(ctx, KID_DENSE_APPLY_MIX, (k_dense_apply_mix<COMP, R, W, CAPTURE, NT, LAYERED>), grid, block, lds, A)
  TILE_SWITCH(A.n, ctx->rpw, CALL)
#undef CALL
}

template <int STAT, bool NT, bool SPARSE = false>
void launch_tile_mix(choco_ctx* ctx, const Args& A, bool fused) {
  const size_t lds = (size_t)A.n * kChunk * sizeof(float);
  const int kid = fused ? KID_TILE_MIX_SGD : KID_TILE_MIX;
  const dim3 grid((unsigned)A.nchunks), block(A.n <= 8 ? 512 : A.n <= 16 ? 256 : 1024);
#define CALL(R, W) LAUNCH(ctx, kid, (k_tile_mix<STAT, R, W, NT, SPARSE>), grid, block, lds, A)
  TILE_SWITCH(A.n, ctx->rpw, CALL)
#undef CALL
}

template <int COMP, bool NT, bool LAYERED = false>
void launch_dense_apply(choco_ctx* ctx, const Args& A) {
  const dim3 grid = chunk_grid((A.d + 3) >> 2, A.n, kStreamVecs);
  if (A.codes) LAUNCH(ctx, KID_DENSE_APPLY, (k_dense_apply<COMP, true, NT, LAYERED>), grid, dim3(256), 0, A);
  else LAUNCH(ctx, KID_DENSE_APPLY, (k_dense_apply<COMP, false, NT, LAYERED>), grid, dim3(256), 0, A);
}

// x += gamma (S - xhat), 4 four-vectors per thread for long rows and 2 for short ones.
template <bool NT>
void launch_mix_incremental(choco_ctx* ctx, const Args& A, bool carries_update) {
  const int kid = carries_update ? KID_MIX_INCREMENTAL_SGD : KID_MIX_INCREMENTAL;
  const int32_t nvec = (A.d + 3) >> 2;
  if (ctx->long_rows)   // (1024 threads with one 4-vector each: 573 against 582 us for 256 with four, d = 28 M)
    LAUNCH(ctx, kid, (k_mix_incremental<NT, 1, 1024>), chunk_grid(nvec, A.n, 4), dim3(1024), 0, A);
  else
    LAUNCH(ctx, kid, (k_mix_incremental<NT, 2>), chunk_grid(nvec, A.n, 2), dim3(256), 0, A);
}

void launch_mix_direct_global(choco_ctx* ctx, const Args& A) {
  LAUNCH(ctx, KID_MIX_DIRECT_GLOBAL, k_mix_direct_global, chunk_grid((A.d + 3) >> 2, A.n, 1), dim3(256), 0, A);
}

// In the two functions below `F` is the argument block for the FIRST kernel that reads X
// in the step (it may carry the fused local update, F.G != nullptr) and `A` the block for
// every later kernel (A.G == nullptr).

// Dense operators (identity, sign, gsgd), direct mix form.
template <int COMP, bool NT>
int gossip_dense(choco_ctx* ctx, const Args& F) {
  Args A = F;
  A.G = nullptr;
  const bool fused = F.G != nullptr;
  constexpr bool needs_stat = (COMP == Q_SIGN || COMP == Q_QSGD);
  constexpr int STAT = needs_stat ? COMP : Q_NONE;
  constexpr int STATK = needs_stat ? COMP : Q_SIGN;   // any valid instantiation where unused
  const dim3 stat_grid((unsigned)A.ngroups, (unsigned)A.n);
  if (ctx->cfg.order == CHOCO_ORDER_COMPRESS_THEN_MIX) {
    if (needs_stat) {
      LAUNCH(ctx, fused ? KID_DENSE_STAT_SGD : KID_DENSE_STAT, (k_dense_stat<STATK, NT>), stat_grid,
             dim3(stat_threads(NT)), 0, F);
      if (!A.fold_finalise)
        LAUNCH(ctx, KID_DENSE_FINALISE, (k_dense_finalise<STATK>), dim3((unsigned)A.n), dim3(256), 0, A);
    }
    if (ctx->rpw) {
      if (A.codes) launch_apply_mix<COMP, true, NT>(ctx, A);
      else launch_apply_mix<COMP, false, NT>(ctx, A);
    } else {
      launch_dense_apply<COMP, NT>(ctx, A);
      launch_mix_direct_global(ctx, A);
    }
  } else {
    if (ctx->rpw) {
      launch_tile_mix<STAT, NT>(ctx, F, fused);
      if (needs_stat)
        LAUNCH(ctx, KID_GROUP_REDUCE, k_group_reduce, dim3((unsigned)((A.ngroups + 15) / 16), (unsigned)A.n),
               dim3(256), 0, A);
    } else {
      launch_mix_direct_global(ctx, A);
      if (needs_stat)
        LAUNCH(ctx, KID_DENSE_STAT, (k_dense_stat<STATK, NT>), stat_grid, dim3(stat_threads(NT)), 0, A);
    }
    if (needs_stat)
      LAUNCH(ctx, KID_DENSE_FINALISE, (k_dense_finalise<STATK>), dim3((unsigned)A.n), dim3(256), 0, A);
    launch_dense_apply<COMP, NT>(ctx, A);
  }
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

// Workgroups of the fallback launch: kFallbackBlocks per worker while all of them fit the chip
// together (those of a worker wait for each other inside the kernel), one per worker beyond.
dim3 fallback_grid(int n) {
  const int per = (int64_t)kFallbackBlocks * n <= 1024 ? kFallbackBlocks : std::max(1, 1024 / n);
  return dim3((unsigned)per, (unsigned)n);
}

// A long pass that selects ahead generates Philox words (ALU work) while the caller's stream
// runs the bandwidth-bound mix.  Left alone its workgroups fill every wave slot first and the
// mix waits behind them; 48 KiB of LDS that it does not use hold it to two workgroups per
// compute unit, so that both make progress (n = 8, 31.8 M entries in 14 layers, ms per step by
// pad: 0 KiB 1.296, 16 KiB 1.267, 28 KiB 1.223, 48 KiB 1.189; a single workgroup per unit is
// too slow to finish behind the mix: 1.316).
size_t ahead_lds_pad(const choco_ctx* ctx, int64_t row_len) {
  return (ctx->launch_stream != ctx->stream && row_len > ((int64_t)1 << 21)) ? (size_t)48 << 10 : 0;
}

// The select of the whole-vector path: one pass over the rows appends the candidates, the
// histogram fallback and the rebuild are no-ops unless a guess failed, then the exact select
// on the lists.  C is the argument block for the pass over the rows (it may carry the local
// update and, with fuse_mix, the mix), A the one without.
template <int COMP, bool NT>
void launch_select(choco_ctx* ctx, const Args& C, const Args& A, int kid_compact, bool fuse_mix) {
  const int32_t nvec = (A.d + 3) >> 2;
  // long rows: 4 four-vectors per thread, short ones 2; random_a 4 at any length (its pass draws
  // Philox words beside the step's bandwidth-bound pass: half as many workgroups get in that pass's
  // way less, n = 64, d = 270 k: 79.4 -> 75.3 us per step; 8 per thread: 76.3; one per thread of a
  // 1024-thread workgroup, the shape top_a's long rows take: 73.7 against 66.4 us as the step stands now)
  const int cvecs = (ctx->fallback_chain || COMP == Q_RANDK) ? kCompactVecs : 2;
  const dim3 cgrid = chunk_grid(nvec, A.n, cvecs);
  const size_t pad = ahead_lds_pad(ctx, A.d);
  // top_a on long rows: the same 4096-entry chunks as one 4-vector per thread of a 1024-thread
  // workgroup (measured against four per thread of 256 threads: 580 against 597 us at d = 28 M;
  // two per thread of 512: 603; short rows gain nothing from wider workgroups: 47.9 against 46.2 us)
  constexpr bool kWide = COMP == Q_TOPK;
  if (fuse_mix) {
    if (cvecs == 2) LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, COMP == Q_TOPK, NT, 2>), cgrid, dim3(256), 0, C);
    else if (kWide) LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, COMP == Q_TOPK, NT, 1, false, 1024>), cgrid, dim3(1024), 0, C);
    else LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, COMP == Q_TOPK, NT, kCompactVecs>), cgrid, dim3(256), 0, C);
  } else {
    if (cvecs == 2) LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, false, NT, 2>), cgrid, dim3(256), pad, C);
    else if (kWide) LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, false, NT, 1, false, 1024>), cgrid, dim3(1024), pad, C);
    else LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, false, NT, kCompactVecs>), cgrid, dim3(256), pad, C);
  }
  if (ctx->fallback_chain) {
    LAUNCH(ctx, KID_SEL_FALLBACK, (k_sel_fallback<COMP>), fallback_grid(A.n), dim3(256), 0, A);
  }
  if (ctx->multipart) {
    const dim3 pgrid((unsigned)kRefineParts, (unsigned)A.n);
    LAUNCH(ctx, KID_SEL_HIST_PARTS, (k_sel_hist_parts<COMP>), pgrid, dim3(1024), 0, A);
    LAUNCH(ctx, KID_SEL_EMIT_PARTS, (k_sel_emit_parts<COMP>), pgrid, dim3(1024), 0, A);
    LAUNCH(ctx, KID_SEL_FINISH, (k_sel_finish<COMP>), dim3((unsigned)A.n), dim3(1024), 0, A);
  } else {
    LAUNCH(ctx, KID_SEL_REFINE, (k_sel_refine<COMP>), dim3((unsigned)A.n), dim3(1024),
           (size_t)A.bitmap_words * sizeof(uint32_t), A);
  }
}

// random_a selects ahead: the mask of a step depends on (seed, step, worker) only, so the
// selection of step t + 1 runs on the library's second stream beside the rest of step t.
// look_ahead_begin: was this step's selection made ahead?  It joins the second stream and, if a
// selection made ahead is being dropped (counter set, look-ahead or timing switched), clears
// the marks it left in its copy of the bit map (no xhat update ever would).
bool in_batch(const choco_ctx* ctx, const AheadBatch& b, uint64_t t) {
  return b.valid && t >= b.base && t - b.base < (uint64_t)ctx->ahead_steps;
}
int ahead_buf(const choco_ctx* ctx, uint64_t t) { return (int)(t % (uint64_t)(2 * ctx->ahead_steps)); }

int look_ahead_begin(choco_ctx* ctx, const Args& A, bool ahead, bool* selected) {
  const uint64_t t = ctx->t;
  if (ahead && in_batch(ctx, ctx->nxt, t)) {   // the first step of a batch: wait for its selections, once
    const int rc = join_lookahead(ctx);
    if (rc != CHOCO_OK) return rc;
    ctx->cur = ctx->nxt;
    ctx->nxt.valid = false;
  }
  *selected = ahead && in_batch(ctx, ctx->cur, t);
  if (!*selected) {
    // this step selects in line (with the same control blocks and candidate lists): nothing may
    // be under way, and what was selected ahead for other steps is dropped
    const int rc = join_lookahead(ctx);
    if (rc != CHOCO_OK) return rc;
    for (int b = 0; b < kAheadBufs; ++b)
      if ((ctx->dirty_maps >> b) & 1u) {
        const int64_t words = (int64_t)A.n * A.map_words;
        LAUNCH(ctx, KID_ZERO_WORDS, k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0,
               ctx->keptmap_buf[b], words);
      }
    ctx->dirty_maps = 0;
    ctx->cur.valid = ctx->nxt.valid = false;
  } else {
    ctx->dirty_maps &= ~(1u << (unsigned)ahead_buf(ctx, t));   // this step's own pass clears the marks it uses
  }
  return CHOCO_OK;
}

// Will this step start the selections of the next batch?  At the first step of a batch whose
// own selections were made ahead (the steps after it then select nothing in line), or at the
// last step before a batch boundary (the start of a run: one step of head start).
bool look_ahead_due(const choco_ctx* ctx, bool ahead) {
  if (!ahead || ctx->nxt.valid) return false;
  const uint64_t B = (uint64_t)ctx->ahead_steps, t = ctx->t, nb = (t / B + 1) * B;
  return in_batch(ctx, ctx->cur, t) || t == nb - 1;
}

// The argument block of the selection of a later step tn: no local update (the keys are Philox
// words, no state is read), that step's copy of the lists, maps and scalars.
Args look_ahead_args(const choco_ctx* ctx, const Args& A, uint64_t tn) {
  Args P = A;
  P.G = nullptr;
  P.M = nullptr;
  P.deferred_sgd = 0;
  P.t_lo = (uint32_t)(tn & 0xFFFFFFFFu);
  P.t_hi = (uint32_t)(tn >> 32);
  const int buf = ahead_buf(ctx, tn);
  P.sel_idx = ctx->sel_idx_buf[buf];
  P.bitmap = ctx->bitmap_buf[buf];
  P.keptmap = ctx->keptmap_buf[buf];
  if (ctx->nlayers > 0) P.layer_scal = ctx->layer_scal_buf[buf];
  return P;
}

// Bracket of the launches that select ahead: between fork and join LAUNCH goes to the second
// stream, which first waits for everything enqueued on the caller's stream so far.
// The point on the caller's stream from which the selection ahead may run; the kernels of this
// step that follow are enqueued BEFORE the selection's (look_ahead_fork comes after them), so
// that they get the compute units first and the selection fills in beside them: enqueued the
// other way round, the selection's many small workgroups take every wave slot and the step's
// own bandwidth-bound pass waits behind them.
int look_ahead_mark(choco_ctx* ctx) {
  HIP_TRY(ctx, hipEventRecord(ctx->ev_fork, ctx->stream));
  return CHOCO_OK;
}

int look_ahead_fork(choco_ctx* ctx) {
  HIP_TRY(ctx, hipStreamWaitEvent(ctx->aux_stream, ctx->ev_fork, 0));
  ctx->launch_stream = ctx->aux_stream;
  return CHOCO_OK;
}

int look_ahead_end(choco_ctx* ctx, const Args& A, uint64_t base) {
  ctx->launch_stream = ctx->stream;
  HIP_TRY(ctx, hipGetLastError());
  HIP_TRY(ctx, hipEventRecord(ctx->ev_ahead, ctx->aux_stream));
  ctx->ahead_pending = true;
  ctx->nxt.base = base;
  ctx->nxt.valid = true;
  if (!A.bitmap_words)
    for (int u = 0; u < ctx->ahead_steps; ++u) ctx->dirty_maps |= 1u << (unsigned)ahead_buf(ctx, base + (uint64_t)u);
  return CHOCO_OK;
}

// Sparsifying operators (top_a, random_a).
template <int COMP, bool NT>
int gossip_sparse(choco_ctx* ctx, const Args& F) {
  Args A = F;
  // a deferred local update (random_a) keeps G visible to the kernels that gather single
  // entries of x; otherwise only the first pass may see it
  if (!F.deferred_sgd) A.G = nullptr;
  const bool fused = F.G != nullptr && !F.deferred_sgd;
  const bool incremental = ctx->mix_form == CHOCO_MIX_INCREMENTAL_S;
  const bool mix_first = ctx->cfg.order == CHOCO_ORDER_MIX_THEN_COMPRESS;
  bool fuse_mix = false;     // the mix rides on the select pass (top_a, printed order, incremental sums)
  bool x_touched = false;    // has a kernel of this step already read X (and taken the fused update)?
  if (mix_first) {
    if (incremental && COMP == Q_TOPK) {
      fuse_mix = true;
    } else {
      if (incremental) launch_mix_incremental<NT>(ctx, F, fused);
      else if (ctx->rpw) launch_tile_mix<Q_NONE, NT>(ctx, F, fused);
      else launch_mix_direct_global(ctx, A);
      x_touched = true;
    }
  }
  // select: one pass over the rows; histogram fallback and rebuild are no-ops unless a guess failed
  const Args& C = x_touched ? A : F;
  const int kid_compact = (!x_touched && fused) ? KID_SEL_COMPACT_SGD : KID_SEL_COMPACT;
  // random_a: this step's selection may already have been made (or be under way) on the second
  // stream; then it is only waited for
  const bool ahead = COMP == Q_RANDK && ctx->lookahead && !ctx->profiling;
  bool selected = false;
  {
    const int rc = look_ahead_begin(ctx, A, ahead, &selected);
    if (rc != CHOCO_OK) return rc;
  }
  if (!selected) launch_select<COMP, NT>(ctx, C, A, kid_compact, fuse_mix);
  const bool due = look_ahead_due(ctx, ahead);
  if (due) {
    const int rc = look_ahead_mark(ctx);
    if (rc != CHOCO_OK) return rc;
  }
  // messages: neighbour sums first (they recompute q from x - xhat), then xhat.  random_a's
  // selection knows no values: gathered for the scatter, else listed by the kernel that forms q
  const unsigned kblocks = (unsigned)((A.k + 255) / 256);
  A.update_values = (COMP == Q_RANDK && !incremental) ? 1 : 0;
  if (COMP == Q_RANDK && incremental)
    LAUNCH(ctx, KID_SEL_VALUES, k_sel_values, dim3(kblocks, (unsigned)A.n), dim3(256), 0, A);
  if (incremental)
    LAUNCH(ctx, KID_SCATTER_S, k_scatter_s, dim3(kblocks, (unsigned)ctx->maxdeg, (unsigned)A.n), dim3(256),
           0, A);
  // short rows: the final mix reads the bitmap and applies xhat += q itself; direct form with
  // the tile kernel: the mix pass applies it off the kept-entry bits whatever the row length
  const bool fused_apply = ctx->fused_sparse_apply;
  const bool fold_xhat = !mix_first && incremental && A.bitmap_words > 0;
  if (!fold_xhat && !fused_apply)
    LAUNCH(ctx, KID_XHAT_UPDATE, k_xhat_update, dim3(kblocks, (unsigned)A.n), dim3(256), 0, A);
  if (!mix_first) {
    // random_a under choco_step: the deferred local update rides on this last pass
    const bool last_carries = F.deferred_sgd != 0;
    Args L = A;
    if (last_carries) L.G = F.G;
    L.fold_xhat = fold_xhat ? 1 : 0;
    if (incremental) launch_mix_incremental<NT>(ctx, L, last_carries);
    else if (fused_apply) launch_tile_mix<Q_NONE, NT, true>(ctx, L, last_carries);
    else if (ctx->rpw) launch_tile_mix<Q_NONE, NT>(ctx, L, last_carries);
    else launch_mix_direct_global(ctx, A);
  }
  ctx->values_in_qv = fused_apply && COMP == Q_RANDK;
  LAUNCH_CHECK(ctx);
  if (due) {
    // the selections of the next batch of steps, into those steps' copies of the lists and of the
    // map, side by side with this step and the ones after it (from the mark set above)
    const uint64_t base = (ctx->t / (uint64_t)ctx->ahead_steps + 1) * (uint64_t)ctx->ahead_steps;
    int rc = look_ahead_fork(ctx);
    if (rc != CHOCO_OK) return rc;
    for (int u = 0; u < ctx->ahead_steps; ++u) {
      const Args P = look_ahead_args(ctx, A, base + (uint64_t)u);
      launch_select<COMP, NT>(ctx, P, P, KID_SEL_COMPACT, false);
    }
    rc = look_ahead_end(ctx, A, base);
    if (rc != CHOCO_OK) return rc;
  }
  return CHOCO_OK;
}

// Layer-wise sign / gsgd: the whole-row pipeline with per-layer norms (norm pass over
// (layer, group) work items, per-layer scales, apply kernels that look the scale up by layer).
template <int COMP, bool NT>
int gossip_layers_dense(choco_ctx* ctx, const Args& F) {
  Args A = F;
  A.G = nullptr;
  const bool fused = F.G != nullptr;
  const bool mix_first = ctx->cfg.order == CHOCO_ORDER_MIX_THEN_COMPRESS;
  bool x_touched = false;
  if (mix_first) {
    if (ctx->rpw) launch_tile_mix<Q_NONE, NT>(ctx, F, fused);   // carries the local update if there is one
    else launch_mix_direct_global(ctx, A);                     // (never handed one: see first_pass_can_carry_sgd)
    x_touched = true;
  }
  const Args& C = x_touched ? A : F;
  LAUNCH(ctx, C.G ? KID_LAYER_STAT_SGD : KID_LAYER_STAT, (k_layer_stat<COMP, NT>),
         dim3((unsigned)A.ngroup_items, (unsigned)A.n), dim3(stat_threads(NT)), 0, C);
  LAUNCH(ctx, KID_LAYER_FINALISE, (k_layer_finalise<COMP>), dim3((unsigned)A.nlayers, (unsigned)A.n), dim3(256), 0, A);
  if (!mix_first && ctx->rpw) {
    if (A.codes) launch_apply_mix<COMP, true, NT, true>(ctx, A);
    else launch_apply_mix<COMP, false, NT, true>(ctx, A);
  } else {
    launch_dense_apply<COMP, NT, true>(ctx, A);
    if (!mix_first) launch_mix_direct_global(ctx, A);
  }
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

// The guessed-threshold select of one long layer (number `which` of ctx->long_layers): the
// launches of the whole-vector path on an argument block that points at the layer's piece of
// the rows (and, where the layers' selects overlap, at the layer's own select scratch).
Args long_layer_args(const choco_ctx* ctx, const Args& src, int which) {
  // the piece of the rows from the 4-vector boundary at or below the layer's first entry (the
  // entries before the layer in that 4-vector do not take part), the layer's own select scratch
  Args R = long_view(src, ctx->long_layers[(size_t)which].sel);
  R.hist16 = (uint32_t*)((char*)src.hist16 + (size_t)which * ctx->set_hist16);
  R.hist_parts = (uint32_t*)((char*)src.hist_parts + (size_t)which * ctx->set_hist_parts);
  R.small_list = (uint2*)((char*)src.small_list + (size_t)which * ctx->set_small_list);
  return R;
}

// ... its pass over the rows (C may carry the local update) ...
template <int COMP, bool NT>
void long_layer_pass(choco_ctx* ctx, const Args& C, int which) {
  const LongLayer& B = ctx->long_layers[(size_t)which];
  if (B.k == 0 || B.batched) return;
  const Args Cl = long_layer_args(ctx, C, which);
  const int kid_compact = Cl.G ? KID_SEL_COMPACT_SGD : KID_SEL_COMPACT;
  const int32_t nvec = (B.sel.d + 3) >> 2;   // (with the entries before the layer in its first 4-vector)
  if (B.plan.fallback_chain && COMP == Q_TOPK)   // (the shape of the whole-row pass on long rows)
    LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, false, NT, 1, false, 1024>), chunk_grid(nvec, C.n, kCompactVecs),
           dim3(1024), 0, Cl);
  else if (B.plan.fallback_chain)
    LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, false, NT, kCompactVecs>), chunk_grid(nvec, C.n, kCompactVecs),
           dim3(256), ahead_lds_pad(ctx, B.len), Cl);
  else
    LAUNCH(ctx, kid_compact, (k_sel_compact<COMP, false, NT, 2>), chunk_grid(nvec, C.n, 2), dim3(256), 0, Cl);
}

// ... and the exact select on its candidates (A: no local update).
template <int COMP, bool NT>
void long_layer_select(choco_ctx* ctx, const Args& A, int which) {
  const LongLayer& B = ctx->long_layers[(size_t)which];
  if (B.k == 0 || B.batched) return;
  const Args Al = long_layer_args(ctx, A, which);
  if (B.plan.fallback_chain) {
    LAUNCH(ctx, KID_SEL_FALLBACK, (k_sel_fallback<COMP>), fallback_grid(A.n), dim3(256), 0, Al);
  }
  if (B.plan.multipart) {
    const dim3 pgrid((unsigned)kRefineParts, (unsigned)A.n);
    LAUNCH(ctx, KID_SEL_HIST_PARTS, (k_sel_hist_parts<COMP>), pgrid, dim3(1024), 0, Al);
    LAUNCH(ctx, KID_SEL_EMIT_PARTS, (k_sel_emit_parts<COMP>), pgrid, dim3(1024), 0, Al);
    LAUNCH(ctx, KID_SEL_FINISH, (k_sel_finish<COMP>), dim3((unsigned)A.n), dim3(1024), 0, Al);
  } else {
    LAUNCH(ctx, KID_SEL_REFINE, (k_sel_refine<COMP>), dim3((unsigned)A.n), dim3(1024), 0, Al);
  }
}

// Layer-wise top_a / random_a: one workgroup or wave per (worker, layer) selects the layer's
// kept entries (layers above CHOCO_MAX_LAYER_LEN: the select chain of the whole-vector path, layer
// after layer); the message kernels and the mix are those of the whole-row path.
template <int COMP, bool NT>
int gossip_layers_sparse(choco_ctx* ctx, const Args& F) {
  Args A = F;
  if (!F.deferred_sgd) A.G = nullptr;
  const bool fused = F.G != nullptr && !F.deferred_sgd;
  const bool mix_first = ctx->cfg.order == CHOCO_ORDER_MIX_THEN_COMPRESS;
  bool x_touched = false;
  if (mix_first) {
    launch_mix_incremental<NT>(ctx, fused ? F : A, fused);
    x_touched = true;
  }
  // random_a never reads X in the layer kernel, so it cannot carry the local update
  Args C = (x_touched || COMP == Q_RANDK) ? A : F;
  if (COMP == Q_RANDK) C.G = nullptr;
  const int nlong = (int)ctx->long_layers.size();   // first in the work list, not for the layer kernel
  const int nmid = ctx->nmid, nsmall = ctx->nsmall, ntiny = A.nlayers - nlong - nmid - nsmall;
  const int wide_blocks = nmid + nsmall + (ntiny + 15) / 16;
  // few workers: with a 1024-thread workgroup for every layer above a wave's reach (and sixteen
  // waves' worth of smaller layers in each of the others) the chip still is not full, and one
  // launch does
  const bool wide = (int64_t)wide_blocks * A.n <= 256;
  // the long layers (those that share launches first, then the others one after the other), then
  // the layer kernel for the layers within its reach
  auto select_layers = [&](const Args& S) -> int {
    Args Q = S;
    Q.G = nullptr;
    Q.M = nullptr;
    // a selection made ahead: the chains that do not depend on one another on two streams - the
    // layers with launches of their own on the one, everything else on the other; without such
    // layers the ones that share launches on the one, the layer kernel on the other
    // (forked and joined once for all the steps of a batch: a chain of one step follows the same
    // chain of the step before on its stream, which is all the order the steps need - they share
    // the control blocks and candidate lists of a chain, and nothing across chains)
    const bool split = ctx->split_ahead;
    const bool solo = nlong > ctx->nbatched;
    auto second = [&](bool yes) {
      if (split) ctx->launch_stream = yes ? ctx->aux_stream2 : ctx->aux_stream;
    };
    second(solo);
    if (ctx->nbatched > 0 && NT && COMP == Q_TOPK) {
      // (large states, streamed past the caches: the workgroup shape of the whole-row pass on long rows)
      const dim3 cgrid((unsigned)((ctx->batched_nvec + 1023) / 1024), (unsigned)A.n, (unsigned)ctx->nbatched);
      LAUNCH(ctx, S.G ? KID_SEL_COMPACT_SGD : KID_SEL_COMPACT, (k_sel_compact<COMP, false, NT, 1, true, 1024>), cgrid,
             dim3(1024), 0, S);
    } else if (ctx->nbatched > 0) {
      const dim3 cgrid((unsigned)((ctx->batched_nvec + 511) / 512), (unsigned)A.n, (unsigned)ctx->nbatched);
      LAUNCH(ctx, S.G ? KID_SEL_COMPACT_SGD : KID_SEL_COMPACT, (k_sel_compact<COMP, false, NT, 2, true>), cgrid,
             dim3(256), 0, S);
    }
    if (ctx->nbatched > 0) {
      LAUNCH(ctx, KID_SEL_REFINE, (k_sel_refine<COMP, true>), dim3((unsigned)A.n, (unsigned)ctx->nbatched), dim3(1024),
             0, Q);
    }
    // top_a with several long layers: a layer's select (a few small launches that wait on
    // memory) goes to the second stream and runs beside the next layer's pass over the rows
    const bool overlap = COMP == Q_TOPK && ctx->overlap_long && !ctx->profiling && ctx->launch_stream == ctx->stream;
    second(false);
    for (int b = 0; b < nlong; ++b) {
      long_layer_pass<COMP, NT>(ctx, S, b);
      if (overlap) {
        HIP_TRY(ctx, hipEventRecord(ctx->ev_fork, ctx->stream));
        HIP_TRY(ctx, hipStreamWaitEvent(ctx->aux_stream, ctx->ev_fork, 0));
        ctx->launch_stream = ctx->aux_stream;
      }
      long_layer_select<COMP, NT>(ctx, Q, b);
      ctx->launch_stream = overlap ? ctx->stream : ctx->launch_stream;
    }
    const int kid = S.G ? KID_LAYER_COMPRESS_SGD : KID_LAYER_COMPRESS;
    second(true);
    if (wide) {
      if (wide_blocks > 0)
        LAUNCH(ctx, kid, (k_layer_compress<COMP, 1024, NT>), dim3((unsigned)wide_blocks, (unsigned)A.n), dim3(1024), 0,
               S, nlong, nmid + nsmall);
    } else {
      if (nmid > 0)
        LAUNCH(ctx, kid, (k_layer_compress<COMP, 1024, NT>), dim3((unsigned)nmid, (unsigned)A.n), dim3(1024), 0, S,
               nlong, nmid);
      if (nsmall + ntiny > 0)
        LAUNCH(ctx, kid, (k_layer_compress<COMP, 256, NT>), dim3((unsigned)(nsmall + (ntiny + 3) / 4), (unsigned)A.n),
               dim3(256), 0, S, nlong + nmid, nsmall);
    }
    if (overlap && nlong > 0) {   // the caller's stream goes on when the last select is done
      HIP_TRY(ctx, hipEventRecord(ctx->ev_ahead, ctx->aux_stream));
      HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_ahead, 0));
    }
    second(false);
    return CHOCO_OK;
  };
  // random_a: this step's masks may already have been drawn on the second stream
  const bool ahead = COMP == Q_RANDK && ctx->lookahead && !ctx->profiling;
  bool selected = false;
  {
    const int rc = look_ahead_begin(ctx, A, ahead, &selected);
    if (rc != CHOCO_OK) return rc;
  }
  if (!selected) {
    const int rc = select_layers(C);
    if (rc != CHOCO_OK) return rc;
  }
  const bool due = look_ahead_due(ctx, ahead);
  if (due) {
    const int rc = look_ahead_mark(ctx);
    if (rc != CHOCO_OK) return rc;
  }
  // direct form (compress-then-mix only): one pass applies xhat += q off the kept-entry bits and
  // mixes; else the messages go into the neighbour sums, then into xhat, and the mix reads S
  const bool fused_apply = ctx->fused_sparse_apply;
  const unsigned kblocks = (unsigned)((A.k + 255) / 256);
  if (!fused_apply) {
    if (COMP == Q_RANDK)
      LAUNCH(ctx, KID_SEL_VALUES, k_sel_values, dim3(kblocks, (unsigned)A.n), dim3(256), 0, A);
    LAUNCH(ctx, KID_SCATTER_S, k_scatter_s, dim3(kblocks, (unsigned)ctx->maxdeg, (unsigned)A.n), dim3(256), 0, A);
    LAUNCH(ctx, KID_XHAT_UPDATE, k_xhat_update, dim3(kblocks, (unsigned)A.n), dim3(256), 0, A);
  }
  if (!mix_first) {
    const bool last_carries = F.deferred_sgd != 0;
    Args L = A;
    if (last_carries) L.G = F.G;
    if (fused_apply) launch_tile_mix<Q_NONE, NT, true>(ctx, L, last_carries);
    else launch_mix_incremental<NT>(ctx, L, last_carries);
  }
  ctx->values_in_qv = fused_apply && COMP == Q_RANDK;
  LAUNCH_CHECK(ctx);
  if (due) {   // the next batch's masks, enqueued after this step's own kernels (see look_ahead_mark)
    const uint64_t base = (ctx->t / (uint64_t)ctx->ahead_steps + 1) * (uint64_t)ctx->ahead_steps;
    int rc = look_ahead_fork(ctx);
    if (rc != CHOCO_OK) return rc;
    if (ctx->aux_stream2 != nullptr) {
      HIP_TRY(ctx, hipEventRecord(ctx->ev_fork2, ctx->aux_stream));
      HIP_TRY(ctx, hipStreamWaitEvent(ctx->aux_stream2, ctx->ev_fork2, 0));
      ctx->split_ahead = true;
    }
    for (int u = 0; u < ctx->ahead_steps; ++u) (void)select_layers(look_ahead_args(ctx, A, base + (uint64_t)u));
    if (ctx->split_ahead) {
      ctx->split_ahead = false;
      HIP_TRY(ctx, hipEventRecord(ctx->ev_join2, ctx->aux_stream2));
      HIP_TRY(ctx, hipStreamWaitEvent(ctx->aux_stream, ctx->ev_join2, 0));
    }
    rc = look_ahead_end(ctx, A, base);
    if (rc != CHOCO_OK) return rc;
  }
  return CHOCO_OK;
}

template <bool NT>
int gossip_any(choco_ctx* ctx, const Args& A) {
  if (ctx->nlayers > 0) {
    switch (ctx->cfg.compressor) {
      case CHOCO_Q_SIGN: return gossip_layers_dense<Q_SIGN, NT>(ctx, A);
      case CHOCO_Q_QSGD: return gossip_layers_dense<Q_QSGD, NT>(ctx, A);
      case CHOCO_Q_TOPK: return gossip_layers_sparse<Q_TOPK, NT>(ctx, A);
      case CHOCO_Q_RANDK: return gossip_layers_sparse<Q_RANDK, NT>(ctx, A);
      default: return CHOCO_E_UNSUPPORTED;
    }
  }
  switch (ctx->cfg.compressor) {
    case CHOCO_Q_IDENTITY: return gossip_dense<Q_IDENTITY, NT>(ctx, A);
    case CHOCO_Q_SIGN: return gossip_dense<Q_SIGN, NT>(ctx, A);
    case CHOCO_Q_QSGD: return gossip_dense<Q_QSGD, NT>(ctx, A);
    case CHOCO_Q_TOPK: return gossip_sparse<Q_TOPK, NT>(ctx, A);
    case CHOCO_Q_RANDK: return gossip_sparse<Q_RANDK, NT>(ctx, A);
    default: return CHOCO_E_INVAL;
  }
}

// Does the first kernel of a gossip step in this configuration read and write X densely,
// so that the local update can ride on it?
bool first_pass_can_carry_sgd(const choco_ctx* ctx) {
  const int comp = ctx->cfg.compressor;
  if (ctx->long_silent) return false;   // the select pass skips a long layer that keeps nothing
  if (ctx->layers_generic) return false;   // layer passes off 16-byte boundaries load entry by entry and store nothing
  const bool incremental = ctx->mix_form == CHOCO_MIX_INCREMENTAL_S;
  if (ctx->cfg.order == CHOCO_ORDER_COMPRESS_THEN_MIX)
    return comp == CHOCO_Q_SIGN || comp == CHOCO_Q_QSGD || comp == CHOCO_Q_TOPK;
  // printed order: the first kernel is the mix
  if (ctx->sparse) return incremental || ctx->rpw != 0;   // k_sel_compact(+mix) / k_mix_incremental / k_tile_mix
  return ctx->rpw != 0;                                    // k_tile_mix
}

int launch_sgd(choco_ctx* ctx, const float* g_dev, float lr) {
  const Args& A = ctx->args;
  const int32_t nvec = (A.d + 3) >> 2;
  const dim3 grid = chunk_grid(nvec, A.n, kStreamVecs);
  if (ctx->nt) LAUNCH(ctx, KID_SGD, k_sgd<true>, grid, dim3(256), 0, A.X, g_dev, A.ld, nvec, lr);
  else LAUNCH(ctx, KID_SGD, k_sgd<false>, grid, dim3(256), 0, A.X, g_dev, A.ld, nvec, lr);
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

// Under choco_step with random_a in the compress-then-mix order nothing reads X densely
// before the final mix, so the local update is deferred into that mix.
bool last_pass_carries_sgd(const choco_ctx* ctx) {
  return !ctx->layers_generic && ctx->cfg.compressor == CHOCO_Q_RANDK && ctx->cfg.order == CHOCO_ORDER_COMPRESS_THEN_MIX &&
         (ctx->mix_form == CHOCO_MIX_INCREMENTAL_S || ctx->rpw != 0);
}

struct LocalUpdate {      // the local update a fused step carries (g == nullptr: none)
  const float* g = nullptr;
  float lr = 0.0f;
  float* m = nullptr;     // momentum memory, or nullptr for plain SGD
  float beta = 0.0f, lambda = 0.0f;
};

int run_gossip(choco_ctx* ctx, const LocalUpdate& u, bool deferred = false) {
  Args A = ctx->args;
  A.t_lo = (uint32_t)(ctx->t & 0xFFFFFFFFu);
  A.t_hi = (uint32_t)(ctx->t >> 32);
  A.G = u.g;
  A.lr = u.lr;
  A.M = u.g ? u.m : nullptr;
  A.beta = u.beta;
  A.lambda = u.lambda;
  A.deferred_sgd = deferred ? 1 : 0;
  const int buf = ahead_buf(ctx, ctx->t);       // the copies take turns (they are one and the same
  A.sel_idx = ctx->sel_idx_buf[buf];       // unless the configuration selects ahead)
  A.bitmap = ctx->bitmap_buf[buf];
  A.keptmap = ctx->keptmap_buf[buf];
  if (ctx->nlayers > 0) A.layer_scal = ctx->layer_scal_buf[buf];
  ctx->fused = u.g != nullptr;
  const int rc = ctx->nt ? gossip_any<true>(ctx, A) : gossip_any<false>(ctx, A);
  ctx->fused = false;
  if (rc == CHOCO_OK) {
    ctx->last_buf = buf;
    ctx->last_t = ctx->t;
    ctx->t += 1;
  }
  return rc;
}

int launch_momentum(choco_ctx* ctx, const float* g_dev, float* m_dev, float lr, float beta, float lambda) {
  const Args& A = ctx->args;
  const int32_t nvec = (A.d + 3) >> 2;
  const dim3 grid = chunk_grid(nvec, A.n, kStreamVecs);
  if (ctx->nt)
    LAUNCH(ctx, KID_MOMENTUM, k_momentum<true>, grid, dim3(256), 0, A.X, g_dev, m_dev, A.ld, nvec, lr, beta, lambda);
  else
    LAUNCH(ctx, KID_MOMENTUM, k_momentum<false>, grid, dim3(256), 0, A.X, g_dev, m_dev, A.ld, nvec, lr, beta, lambda);
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

// One whole iteration: the local update (plain or momentum), then the gossip step; fused
// into the first (or, for random_a, the last) dense pass where the configuration has one.
int fused_iteration(choco_ctx* ctx, const LocalUpdate& u) {
  if (first_pass_can_carry_sgd(ctx)) return run_gossip(ctx, u);
  if (last_pass_carries_sgd(ctx)) return run_gossip(ctx, u, true);
  const int rc = u.m ? launch_momentum(ctx, u.g, u.m, u.lr, u.beta, u.lambda) : launch_sgd(ctx, u.g, u.lr);
  if (rc != CHOCO_OK) return rc;
  return run_gossip(ctx, LocalUpdate());
}

// Which configurations the message kernels cover.
int wire_supported(const choco_ctx* ctx) {
  if (ctx->cfg.compressor == CHOCO_Q_IDENTITY) return CHOCO_E_UNSUPPORTED;
  return CHOCO_OK;
}

WireArgs wire_args(const choco_ctx* ctx) {
  const Args& A = ctx->args;
  WireArgs Wa;
  std::memset(&Wa, 0, sizeof(Wa));
  Wa.n = A.n;
  Wa.d = A.d;
  Wa.ld = A.ld;
  const bool dense_layers = ctx->nlayers > 0 && !ctx->sparse;
  Wa.words = dense_layers ? ctx->wire_words : message_words(ctx->cfg.compressor, A.d, A.k, ctx->cfg.levels);
  Wa.W = ((int64_t)A.d + 31) / 32;
  Wa.mb = magnitude_bits(ctx->cfg.levels);
  Wa.levels = ctx->cfg.levels;
  Wa.planes = A.planes;
  Wa.plane_words = A.plane_words;
  Wa.nplanes = A.nplanes;
  Wa.ovf_ring = A.ovf_ring;
  Wa.t_lo = (uint32_t)(ctx->last_t & 0xFFFFFFFFu);
  Wa.t_hi = (uint32_t)(ctx->last_t >> 32);
  Wa.ctl = A.ctl;
  Wa.layers = A.layers;
  Wa.nlayers = dense_layers ? ctx->nlayers : 0;
  Wa.layer_word_off = ctx->wire_word_off;
  Wa.layer_plane_off = ctx->wire_plane_off;
  Wa.layer_scale = A.layer_scale;
  Wa.k = A.k;
  Wa.sel_idx = ctx->sel_idx_buf[ctx->last_buf];   // of the last finished step
  Wa.sel_val = A.sel_val;
  Wa.bitmap = ctx->bitmap_buf[ctx->last_buf];
  Wa.bitmap_words = A.bitmap_words;
  Wa.keptmap = ctx->keptmap_buf[ctx->last_buf];
  Wa.map_words = A.map_words;
  Wa.chunk_rank = ctx->wire_rank;
  Wa.nchunk = (A.ld + 1023) / 1024;
  return Wa;
}

// random_a without a bitmap: mark the kept entries of the last step in the (otherwise zero) bit
// map and count them chunk by chunk, so that a kept entry's rank is a table look-up plus a
// count inside its own chunk.  The caller clears the marks again.
void launch_rank_tables(choco_ctx* ctx, const WireArgs& Wa) {
  LAUNCH(ctx, KID_WIRE, k_wire_mark, dim3((unsigned)((Wa.k + 255) / 256), (unsigned)Wa.n), dim3(256), 0, Wa, 1);
  LAUNCH(ctx, KID_WIRE, k_wire_chunk_counts, dim3((unsigned)((Wa.nchunk + 7) / 8), (unsigned)Wa.n), dim3(256), 0, Wa);
  LAUNCH(ctx, KID_WIRE, k_wire_chunk_scan, dim3((unsigned)Wa.n), dim3(1024), 0, Wa);
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
  ctx->cfg.layer_start_host = nullptr;
  ctx->cfg.layer_len_host = nullptr;
  ctx->cfg.layer_k_host = nullptr;
  ctx->stream = (hipStream_t)cfg->stream;
  ctx->aux_stream = nullptr;
  ctx->launch_stream = ctx->stream;
  ctx->ev_fork = ctx->ev_ahead = nullptr;
  ctx->aux_stream2 = nullptr;
  ctx->ev_fork2 = ctx->ev_join2 = nullptr;
  ctx->split_ahead = false;
  ctx->lookahead = ctx->can_lookahead = ctx->ahead_pending = false;
  ctx->cur = ctx->nxt = AheadBatch{0, false};
  ctx->ahead_steps = cfg->d > ((int64_t)1 << 21) ? 1 : kAheadSteps;
  ctx->last_buf = 0;
  ctx->dirty_maps = 0;
  ctx->maxdeg = maxdeg;
  ctx->nnz = nnz;
  ctx->sparse = is_sparse(cfg->compressor);
  ctx->mix_form = resolve_mix_form(*cfg);
  ctx->fused_sparse_apply = fused_sparse_apply(*cfg);
  ctx->values_in_qv = false;
  ctx->rpw = pick_rpw(cfg->n);
  ctx->plan = SelectPlan{};
  ctx->plan.guess0 = 0xFFFFFFFFu;
  if (ctx->sparse && cfg->nlayers == 0) ctx->plan = plan_select(cfg->compressor, cfg->d, cfg->k);
  ctx->fallback_chain = ctx->plan.fallback_chain;
  ctx->long_rows = cfg->d > ((int64_t)1 << 21);
  ctx->long_layers = long_layers_of(*cfg);
  ctx->long_silent = false;
  for (const LongLayer& B : ctx->long_layers) ctx->long_silent = ctx->long_silent || B.k == 0;
  ctx->nlayers = cfg->nlayers;
  ctx->layers_generic = cfg->nlayers > 0 && !layers_aligned(*cfg);
  // Non-temporal (streaming) or ordinary cached accesses, by the size of one state array;
  // measured on MI355X with 64 workers on a ring unless said otherwise (ms per step, NT / cached):
  //   8.6 MB (n = 8) sign 0.0189 / 0.0216;  16 MB sign 0.0326 / 0.0319;  33 MB sign 0.0567 / 0.0536,
  //   top-k 0.0772 / 0.0676;  69 MB top-k 0.131 / 0.124, sign per layer 0.117 / 0.101;
  //   132 MB top-k 0.258 / 0.316;  264 MB top-k 0.542 / 0.685.
  // The three or four arrays of a step stay in the 256 MB last-level cache between kernels when
  // they fit, and ordinary accesses then beat the streaming ones; small states lose more at
  // the kernel boundaries (dirty lines are written back there), large ones only thrash.
  const size_t state_bytes = (size_t)cfg->n * (size_t)resolve_ld(*cfg) * sizeof(float);
  const bool cache_resident = state_bytes >= ((size_t)12 << 20) && state_bytes <= ((size_t)96 << 20);
  ctx->nt = state_bytes >= ((size_t)4 << 20) && !cache_resident;
  ctx->t = 0;
  ctx->last_hip_error = 0;
  ctx->profiling = false;
  ctx->fused = false;
  ctx->ev_used = 0;

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
  // polls of about 2 us each: a tenth of a second before a workgroup of the fallback stops waiting
  // for its worker's others (CHOCO_FALLBACK_SPIN_LIMIT: for tests of that path, which scans the row)
  A.spin_limit = 1u << 16;
  if (const char* sl = std::getenv("CHOCO_FALLBACK_SPIN_LIMIT")) A.spin_limit = (uint32_t)std::strtoul(sl, nullptr, 10);
  A.gamma = cfg->gamma;
  A.chunk_sums = (double*)(base + L.chunk_sums);
  A.group_sums = (double*)(base + L.group_sums);
  A.nchunks = L.nchunks;
  A.ngroups = L.ngroups;
  A.levels = cfg->levels;
  A.tau = 1.0;
  if (cfg->compressor == CHOCO_Q_QSGD && cfg->qsgd_biased) {
    const double s = (double)cfg->levels, dd = (double)cfg->d;
    A.tau = 1.0 + std::min(dd / (s * s), std::sqrt(dd) / s);
  }
  A.codes = nullptr;
  // with few group sums the fused apply kernel finishes the norm tree itself (one launch less)
  A.fold_finalise = (ctx->rpw != 0 && cfg->order == CHOCO_ORDER_COMPRESS_THEN_MIX && L.ngroups <= 256) ? 1 : 0;
  A.k = kept_per_worker(*cfg);
  A.hist16 = (uint32_t*)(base + L.hist16);
  A.cand = (uint2*)(base + L.cand);
  A.hist_parts = (uint32_t*)(base + L.hist_parts);
  A.small_list = (uint2*)(base + L.small_list);
  ctx->multipart = ctx->plan.multipart;
  apply_plan(A, ctx->plan);
  const uint32_t guess0 = ctx->plan.guess0, shift0 = ctx->plan.shift0;
  A.sel_stride = A.k;
  A.idx_base = 0;
  A.vec_base = 0;
  A.sel_idx = (int32_t*)(base + L.sel_idx);
  A.sel_val = (float*)(base + L.sel_val);
  A.keptmap = (uint32_t*)(base + L.keptmap);
  A.Qv = (ctx->fused_sparse_apply && cfg->compressor == CHOCO_Q_RANDK) ? (float*)(base + L.qv) : nullptr;
  A.map_words = (A.ld + 31) / 32;
  A.bitmap = (uint32_t*)(base + L.bitmap);
  A.bitmap_words = L.bitmap_words;
  for (int b = 0; b < kAheadBufs; ++b) {
    ctx->sel_idx_buf[b] = A.sel_idx;
    ctx->bitmap_buf[b] = A.bitmap;
    ctx->keptmap_buf[b] = A.keptmap;
  }
  // what the kernels need of each long layer; those that share launches go into a device table
  std::vector<LongSel> long_tab;
  ctx->nbatched = 0;
  ctx->batched_nvec = 0;
  int nsolo = 0;
  for (size_t b = 0; b < ctx->long_layers.size(); ++b) {
    LongLayer& B = ctx->long_layers[b];
    LongSel& Z = B.sel;
    Z.e_lo = B.start & 3;
    Z.base = B.start - Z.e_lo;
    Z.d = B.len + Z.e_lo;
    Z.k = B.k;
    Z.sel_base = B.sel_base;
    Z.set = (int32_t)b;
    Z.cand_cap = B.plan.cand_cap;
    Z.seg_cap = B.plan.seg_cap;
    Z.extra = B.plan.extra;
    Z.want = B.plan.want;
    Z.delta0 = B.plan.delta0;
    Z.sample_stride = B.plan.sample_stride;
    Z.sample_need = B.plan.sample_need;
    Z.set_cand = (int64_t)(L.cand_bytes / sizeof(uint2));
    if (B.batched && long_tab.size() < 65535) {   // (a grid has that many layers at most)
      long_tab.push_back(Z);
      ctx->batched_nvec = std::max(ctx->batched_nvec, (Z.d + 3) >> 2);
    } else {
      B.batched = false;
      nsolo += B.k > 0 ? 1 : 0;
    }
  }
  ctx->nbatched = (int)long_tab.size();
  ctx->long_tab = (const LongSel*)(base + L.long_tab);
  A.long_tab = ctx->long_tab;
  ctx->overlap_long = cfg->compressor == CHOCO_Q_TOPK && nsolo >= 2;
  ctx->set_hist16 = L.hist16_bytes;
  ctx->set_cand = L.cand_bytes;
  ctx->set_hist_parts = L.hist_parts_bytes;
  ctx->set_small_list = L.small_list_bytes;
  if (ctx->overlap_long) {
    hipError_t se = hipStreamCreateWithFlags(&ctx->aux_stream, hipStreamNonBlocking);
    if (se == hipSuccess) se = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
    if (se == hipSuccess) se = hipEventCreateWithFlags(&ctx->ev_ahead, hipEventDisableTiming);
    if (se != hipSuccess) {
      release_ctx(ctx);
      return CHOCO_E_HIP;
    }
  }
  if (cfg->compressor == CHOCO_Q_RANDK) {
    for (int b = 1; b < 2 * ctx->ahead_steps; ++b) {
      ctx->sel_idx_buf[b] = (int32_t*)(base + L.sel_idx2 + (size_t)(b - 1) * L.sel_idx_bytes);
      if (L.bitmap_words > 0) ctx->bitmap_buf[b] = (uint32_t*)(base + L.bitmap2 + (size_t)(b - 1) * L.bitmap_bytes);
      else ctx->keptmap_buf[b] = (uint32_t*)(base + L.keptmap2 + (size_t)(b - 1) * L.keptmap_bytes);
    }
    hipError_t se = hipStreamCreateWithFlags(&ctx->aux_stream, hipStreamNonBlocking);
    if (se == hipSuccess) se = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
    if (se == hipSuccess) se = hipEventCreateWithFlags(&ctx->ev_ahead, hipEventDisableTiming);
    if (cfg->nlayers > 0) {
      if (se == hipSuccess) se = hipStreamCreateWithFlags(&ctx->aux_stream2, hipStreamNonBlocking);
      if (se == hipSuccess) se = hipEventCreateWithFlags(&ctx->ev_fork2, hipEventDisableTiming);
      if (se == hipSuccess) se = hipEventCreateWithFlags(&ctx->ev_join2, hipEventDisableTiming);
    }
    if (se != hipSuccess) {
      release_ctx(ctx);
      return CHOCO_E_HIP;
    }
    ctx->lookahead = ctx->can_lookahead = true;
  }
  A.randk_rescale = cfg->randk_rescale ? 1 : 0;
  A.randk_scale = (ctx->sparse && cfg->nlayers == 0) ? (float)((double)cfg->d / (double)cfg->k) : 1.0f;
  A.qsgd_biased = cfg->qsgd_biased ? 1 : 0;
  // layer tables: descriptors in layer order, and again by falling length (the work list)
  std::vector<LayerDesc> layers((size_t)cfg->nlayers), work;
  A.nlayers = cfg->nlayers;
  A.layers_generic = ctx->layers_generic ? 1 : 0;
  A.layers = (const LayerDesc*)(base + L.layers);
  A.layer_work = (const LayerDesc*)(base + L.layer_work);
  A.layer_guess = (uint32_t*)(base + L.layer_guess);
  A.layer_scal = (double*)(base + L.layer_scal);
  for (int b = 0; b < kAheadBufs; ++b) {
    ctx->layer_scal_buf[b] = A.layer_scal;
    if (b > 0 && b < 2 * ctx->ahead_steps && ctx->can_lookahead && cfg->nlayers > 0)
      ctx->layer_scal_buf[b] = (double*)(base + L.layer_scal2 + (size_t)(b - 1) * L.layer_scal_bytes);
  }
  if (cfg->nlayers > 0) {
    int64_t sel_base = 0;
    for (int32_t l = 0; l < cfg->nlayers; ++l) {
      LayerDesc& D = layers[(size_t)l];
      D.start = (int32_t)cfg->layer_start_host[l];
      D.len = (int32_t)cfg->layer_len_host[l];
      D.k = ctx->sparse ? (int32_t)cfg->layer_k_host[l] : 0;
      D.sel_base = (int32_t)sel_base;
      D.id = l;
      D.head = D.start & 3;
      D.pad[0] = D.pad[1] = 0;
      sel_base += D.k;
    }
    work = layers;
    std::stable_sort(work.begin(), work.end(),
                     [](const LayerDesc& a, const LayerDesc& b) { return a.len + a.head > b.len + b.head; });
    ctx->nmid = ctx->nsmall = 0;
    for (const LayerDesc& D : work) {
      const int32_t span = D.len + D.head;   // what the layer kernel holds in registers
      // (long layers: first in the list, skipped by the layer kernel)
      if (span <= kMidLayerLen && span > kSmallLayerLen) ctx->nmid += 1;
      else if (span <= kSmallLayerLen && span > kWaveLayerLen) ctx->nsmall += 1;
    }
  }
  std::vector<LayerGroup> groups;
  std::vector<int32_t> group_first;
  std::vector<int4> chunk_layer;
  A.layer_groups = (const LayerGroup*)(base + L.layer_groups);
  A.layer_group_first = (const int32_t*)(base + L.layer_group_first);
  A.ngroup_items = L.ngroup_items;
  A.layer_group_sums = (double*)(base + L.layer_group_sums);
  A.layer_scale = (LayerScale*)(base + L.layer_scale);
  A.chunk_layer = (const int4*)(base + L.chunk_layer);
  if (cfg->nlayers > 0 && !ctx->sparse) {
    const int32_t span = kGroup * kChunk;
    for (const LayerDesc& D : layers) {
      group_first.push_back((int32_t)groups.size());
      for (int32_t off = 0; off < D.len; off += span) groups.push_back(LayerGroup{D.start + off, D.len - off, D.id, 0});
    }
    group_first.push_back((int32_t)groups.size());
    chunk_layer.resize((size_t)L.nchunks);
    int32_t lay = 0;
    for (int32_t ch = 0; ch < L.nchunks && !ctx->layers_generic; ++ch) {
      while (lay + 1 < cfg->nlayers && layers[(size_t)lay + 1].start <= ch * kChunk) ++lay;
      const LayerDesc& D = layers[(size_t)lay];
      const int32_t next = lay + 1 < cfg->nlayers ? layers[(size_t)lay + 1].start : INT32_MAX;
      chunk_layer[(size_t)ch] = make_int4(lay, D.start + D.len, next, 0);
    }
  }
  A.seed_lo = (uint32_t)(cfg->seed & 0xFFFFFFFFu);
  A.seed_hi = (uint32_t)(cfg->seed >> 32);
  A.nplanes = cfg->compressor == CHOCO_Q_SIGN ? 1 : cfg->compressor == CHOCO_Q_QSGD ? 1 + magnitude_bits(cfg->levels) : 0;
  A.mb = magnitude_bits(cfg->levels);
  A.plane_words = (A.ld + 31) / 32;
  A.planes = A.nplanes ? (uint32_t*)(base + L.planes) : nullptr;
  A.ovf_ring = (uint4*)(base + L.ovf_ring);
  A.ovf_pos = (uint32_t*)(base + L.ovf_pos);
  ctx->last_t = 0;
  ctx->wire_rank = (uint32_t*)(base + L.wire_rank);
  ctx->wire_word_off = (const int64_t*)(base + L.wire_word_off);
  ctx->wire_plane_off = (const int64_t*)(base + L.wire_plane_off);
  ctx->wire_words = L.wire_words;
  ctx->wire_plane_words = L.wire_plane_words;
  std::vector<int64_t> word_off, plane_off;
  if (cfg->nlayers > 0 && !ctx->sparse) {
    int64_t wo = 0, po = 0;
    for (int32_t l = 0; l < cfg->nlayers; ++l) {
      word_off.push_back(wo);
      plane_off.push_back(po);
      wo += message_words(cfg->compressor, cfg->layer_len_host[l], 0, cfg->levels);
      po += (cfg->layer_len_host[l] + 31) / 32;
    }
    word_off.push_back(wo);
    plane_off.push_back(po);
  }
  ctx->metrics_part = (double*)(base + L.mpart);
  ctx->metrics_out = (double*)(base + L.mout);
  ctx->metrics_blocks = kMetricsBlocks;

  // the library's own scratch array on this GPU (used by choco_metrics_noalloc only)
  ctx->device = -1;
  ctx->noalloc_scratch = nullptr;
  {
    const hipError_t se = resolve_scratch(&ctx->device, &ctx->noalloc_scratch);
    if (se != hipSuccess) {
      release_ctx(ctx);
      return CHOCO_E_HIP;
    }
  }

  // zero everything but the caller's X: xhat^(0) = 0, S = 0, counters, histograms, kept-entry map
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
  if (e == hipSuccess && cfg->nlayers > 0)
    e = hipMemcpyAsync(base + L.layers, layers.data(), layers.size() * sizeof(LayerDesc), hipMemcpyHostToDevice,
                       ctx->stream);
  if (e == hipSuccess && cfg->nlayers > 0)
    e = hipMemcpyAsync(base + L.layer_work, work.data(), work.size() * sizeof(LayerDesc), hipMemcpyHostToDevice,
                       ctx->stream);
  if (e == hipSuccess && !long_tab.empty())
    e = hipMemcpyAsync(base + L.long_tab, long_tab.data(), long_tab.size() * sizeof(LongSel), hipMemcpyHostToDevice,
                       ctx->stream);
  if (e == hipSuccess && cfg->nlayers > 0)   // no threshold guesses yet
    e = hipMemsetAsync(base + L.layer_guess, 0xFF, (size_t)cfg->n * (size_t)cfg->nlayers * sizeof(uint32_t),
                       ctx->stream);
  if (e == hipSuccess && !groups.empty())
    e = hipMemcpyAsync(base + L.layer_groups, groups.data(), groups.size() * sizeof(LayerGroup), hipMemcpyHostToDevice,
                       ctx->stream);
  if (e == hipSuccess && !groups.empty())
    e = hipMemcpyAsync(base + L.layer_group_first, group_first.data(), group_first.size() * sizeof(int32_t),
                       hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess && !groups.empty())
    e = hipMemcpyAsync(base + L.chunk_layer, chunk_layer.data(), chunk_layer.size() * sizeof(int4),
                       hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess && !word_off.empty())
    e = hipMemcpyAsync(base + L.wire_word_off, word_off.data(), word_off.size() * sizeof(int64_t),
                       hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess && !plane_off.empty())
    e = hipMemcpyAsync(base + L.wire_plane_off, plane_off.data(), plane_off.size() * sizeof(int64_t),
                       hipMemcpyHostToDevice, ctx->stream);
  std::vector<WorkerCtl> ctl0;
  if (e == hipSuccess) {
    const size_t nlong = ctx->long_layers.size();
    ctl0.resize((size_t)cfg->n * std::max<size_t>(1, nlong));
    std::memset(ctl0.data(), 0, ctl0.size() * sizeof(WorkerCtl));
    for (size_t j = 0; j < ctl0.size(); ++j) {
      const SelectPlan& P = nlong ? ctx->long_layers[j / (size_t)cfg->n].plan : ctx->plan;
      ctl0[j].guess_key = nlong ? P.guess0 : guess0;
      ctl0[j].bin_shift = nlong ? P.shift0 : shift0;
    }
    e = hipMemcpyAsync(base + L.ctl, ctl0.data(), ctl0.size() * sizeof(WorkerCtl), hipMemcpyHostToDevice,
                       ctx->stream);
  }
  // the host buffers above are pageable: wait until the copies have read them
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) {
    release_ctx(ctx);
    return CHOCO_E_HIP;
  }
  *out = ctx;
  return CHOCO_OK;
}

int choco_gossip_step(choco_ctx* ctx) {
  if (!ctx) return CHOCO_E_INVAL;
  return run_gossip(ctx, LocalUpdate());
}

int choco_sgd_step(choco_ctx* ctx, const float* g_dev, float lr) {
  if (!ctx || !g_dev || ((uintptr_t)g_dev & 15u) != 0) return CHOCO_E_INVAL;
  return launch_sgd(ctx, g_dev, lr);
}

int choco_step(choco_ctx* ctx, const float* g_dev, float lr) {
  if (!ctx || !g_dev || ((uintptr_t)g_dev & 15u) != 0) return CHOCO_E_INVAL;
  LocalUpdate u;
  u.g = g_dev;
  u.lr = lr;
  return fused_iteration(ctx, u);
}

int choco_momentum_step(choco_ctx* ctx, const float* g_dev, float* m_dev, float lr, float beta,
                        float lambda) {
  if (!ctx || !g_dev || !m_dev) return CHOCO_E_INVAL;
  if (((uintptr_t)g_dev & 15u) != 0 || ((uintptr_t)m_dev & 15u) != 0) return CHOCO_E_INVAL;
  return launch_momentum(ctx, g_dev, m_dev, lr, beta, lambda);
}

int choco_step_momentum(choco_ctx* ctx, const float* g_dev, float* m_dev, float lr, float beta,
                        float lambda) {
  if (!ctx || !g_dev || !m_dev) return CHOCO_E_INVAL;
  if (((uintptr_t)g_dev & 15u) != 0 || ((uintptr_t)m_dev & 15u) != 0) return CHOCO_E_INVAL;
  LocalUpdate u;
  u.g = g_dev;
  u.lr = lr;
  u.m = m_dev;
  u.beta = beta;
  u.lambda = lambda;
  return fused_iteration(ctx, u);
}

int choco_metrics(choco_ctx* ctx, double* consensus_host, double* mean_norm_host, double* psi_host) {
  if (!ctx) return CHOCO_E_INVAL;
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

int choco_metrics_noalloc(choco_ctx* ctx, double* out_dev) {
  if (!ctx || !out_dev || ((uintptr_t)out_dev & 7u) != 0) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  if ((int64_t)A.d > (int64_t)CHOCO_NOALLOC_MAX_D) return CHOCO_E_UNSUPPORTED;
  if (!ctx->noalloc_scratch) return CHOCO_E_UNSUPPORTED;   // GPU number beyond the table of scratch addresses
  int dev = -1;
  HIP_TRY(ctx, hipGetDevice(&dev));
  if (dev != ctx->device) return CHOCO_E_INVAL;            // the address kept is that GPU's
  int blocks = (A.d + 255) / 256;
  if (blocks > kNoAllocBlocks) blocks = kNoAllocBlocks;
  // every block writes its three partial sums and the last kernel reads exactly `blocks` of them,
  // so what an earlier (larger) call left behind in the array is never read: nothing to clear
  hipLaunchKernelGGL(k_metrics_partial, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, A,
                     ctx->noalloc_scratch);
  hipLaunchKernelGGL(k_metrics_final_dev, dim3(1), dim3(64), 0, ctx->stream, ctx->noalloc_scratch, blocks,
                     A.n, out_dev);
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

int choco_xhat(choco_ctx* ctx, float** xhat_dev) {
  if (!ctx || !xhat_dev) return CHOCO_E_INVAL;
  *xhat_dev = ctx->args.Xhat;
  return CHOCO_OK;
}

int choco_nsum(choco_ctx* ctx, float** s_dev) {
  if (!ctx || !s_dev) return CHOCO_E_INVAL;
  *s_dev = ctx->args.S;
  return CHOCO_OK;
}

}  // extern "C"

namespace {

// random_a after a fused update-and-mix pass: collect the kept values of the last step from Qv
// into the list (idempotent; read-back and message encoding call it, a step never does).
int gather_values(choco_ctx* ctx) {
  if (!ctx->values_in_qv) return CHOCO_OK;
  Args A = ctx->args;
  A.sel_idx = ctx->sel_idx_buf[ctx->last_buf];
  LAUNCH(ctx, KID_GATHER_VALUES, k_gather_values, dim3((unsigned)((A.k + 255) / 256), (unsigned)A.n), dim3(256), 0, A);
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

}  // namespace

extern "C" {

int choco_last_selection(choco_ctx* ctx, int32_t* idx_dev, float* val_dev) {
  if (!ctx || !ctx->sparse) return CHOCO_E_INVAL;
  {
    const int rc = gather_values(ctx);
    if (rc != CHOCO_OK) return rc;
  }
  const Args& A = ctx->args;
  const size_t count = (size_t)A.n * (size_t)A.k;
  if (idx_dev)
    HIP_TRY(ctx, hipMemcpyAsync(idx_dev, ctx->sel_idx_buf[ctx->last_buf], count * sizeof(int32_t),
                                hipMemcpyDeviceToDevice, ctx->stream));
  if (val_dev)
    HIP_TRY(ctx, hipMemcpyAsync(val_dev, A.sel_val, count * sizeof(float), hipMemcpyDeviceToDevice,
                                ctx->stream));
  return CHOCO_OK;
}

int choco_last_message(choco_ctx* ctx, int32_t worker, int32_t* idx_dev, float* val_dev, uint32_t* bits_dev,
                       float* scale_host) {
  if (!ctx || worker < 0 || worker >= ctx->args.n || ctx->cfg.compressor == CHOCO_Q_IDENTITY) return CHOCO_E_INVAL;
  const Args& A = ctx->args;
  if (scale_host) *scale_host = 0.0f;
  if (ctx->sparse) {
    const int rc = gather_values(ctx);
    if (rc != CHOCO_OK) return rc;
    const size_t off = (size_t)worker * (size_t)A.k, count = (size_t)A.k;
    if (idx_dev)
      HIP_TRY(ctx, hipMemcpyAsync(idx_dev, ctx->sel_idx_buf[ctx->last_buf] + off, count * sizeof(int32_t),
                                  hipMemcpyDeviceToDevice, ctx->stream));
    if (val_dev)
      HIP_TRY(ctx, hipMemcpyAsync(val_dev, A.sel_val + off, count * sizeof(float), hipMemcpyDeviceToDevice,
                                  ctx->stream));
    return CHOCO_OK;
  }
  if (scale_host && ctx->nlayers > 0) return CHOCO_E_INVAL;
  if (bits_dev) {
    const size_t W = ((size_t)A.d + 31) / 32;
    HIP_TRY(ctx, hipMemcpy2DAsync(bits_dev, W * sizeof(uint32_t),
                                  A.planes + (size_t)worker * (size_t)A.nplanes * (size_t)A.plane_words,
                                  (size_t)A.plane_words * sizeof(uint32_t), W * sizeof(uint32_t), (size_t)A.nplanes,
                                  hipMemcpyDeviceToDevice, ctx->stream));
  }
  if (scale_host) {
    WorkerCtl c;
    HIP_TRY(ctx, hipMemcpyAsync(&c, A.ctl + worker, sizeof(c), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    *scale_host = ctx->cfg.compressor == CHOCO_Q_SIGN ? c.scale_c : c.scale_step;
  }
  return CHOCO_OK;
}

int choco_paper_message_bits(int32_t compressor, int64_t d, int64_t k, int32_t levels, int64_t* bits_host) {
  if (!bits_host || d < 1) return CHOCO_E_INVAL;
  switch (compressor) {
    case CHOCO_Q_IDENTITY: *bits_host = 32 * d; return CHOCO_OK;
    case CHOCO_Q_TOPK:
    case CHOCO_Q_RANDK:
      if (k < 1 || k > d) return CHOCO_E_INVAL;
      *bits_host = (compressor == CHOCO_Q_TOPK ? 64 : 32) * k;
      return CHOCO_OK;
    case CHOCO_Q_SIGN: *bits_host = d + 32; return CHOCO_OK;
    case CHOCO_Q_QSGD: {
      if (levels < 1) return CHOCO_E_INVAL;
      int b = 1;
      for (int x = levels; x > 1; x >>= 1) ++b;
      *bits_host = (int64_t)b * d + 32;
      return CHOCO_OK;
    }
    default: return CHOCO_E_INVAL;
  }
}

int choco_message_bytes(choco_ctx* ctx, size_t* bytes_host) {
  if (!ctx || !bytes_host) return CHOCO_E_INVAL;
  const int rc = wire_supported(ctx);
  if (rc != CHOCO_OK) return rc;
  *bytes_host = (size_t)wire_args(ctx).words * 4;
  return CHOCO_OK;
}

int choco_pack_messages(choco_ctx* ctx, void* msgs_dev) {
  if (!ctx || !msgs_dev || ((uintptr_t)msgs_dev & 3u) != 0) return CHOCO_E_INVAL;
  int rc = wire_supported(ctx);
  if (rc != CHOCO_OK) return rc;
  rc = gather_values(ctx);   // random_a after a fused update-and-mix pass: the value list is made now
  if (rc != CHOCO_OK) return rc;
  const WireArgs Wa = wire_args(ctx);
  uint32_t* msg = (uint32_t*)msgs_dev;
  const dim3 kgrid((unsigned)((Wa.k + 255) / 256), (unsigned)Wa.n);
  const dim3 lgrid((unsigned)((ctx->wire_plane_words + 255) / 256), (unsigned)Wa.n);
  const dim3 pgrid((unsigned)((Wa.W + 255) / 256), (unsigned)(Wa.nplanes > 0 ? Wa.nplanes : 1), (unsigned)Wa.n);
  switch (ctx->cfg.compressor) {
    case CHOCO_Q_SIGN:
      if (Wa.nlayers) LAUNCH(ctx, KID_WIRE, k_pack_dense_layers<false>, lgrid, dim3(256), 0, Wa, msg);
      else LAUNCH(ctx, KID_WIRE, k_pack_planes<false>, pgrid, dim3(256), 0, Wa, msg);
      break;
    case CHOCO_Q_QSGD:
      if (Wa.nlayers) LAUNCH(ctx, KID_WIRE, k_pack_dense_layers<true>, lgrid, dim3(256), 0, Wa, msg);
      else LAUNCH(ctx, KID_WIRE, k_pack_planes<true>, pgrid, dim3(256), 0, Wa, msg);
      break;
    case CHOCO_Q_TOPK:
      LAUNCH(ctx, KID_WIRE, k_pack_topk, kgrid, dim3(256), 0, Wa, msg);
      break;
    case CHOCO_Q_RANDK:
      if (Wa.bitmap_words) {
        LAUNCH(ctx, KID_WIRE, k_pack_randk, dim3((unsigned)Wa.n), dim3(1024),
               (size_t)Wa.bitmap_words * sizeof(uint32_t), Wa, msg);
      } else {
        launch_rank_tables(ctx, Wa);
        LAUNCH(ctx, KID_WIRE, k_pack_randk_ranked, dim3((unsigned)((Wa.k + 3) / 4), (unsigned)Wa.n), dim3(256), 0, Wa,
               msg);
        LAUNCH(ctx, KID_WIRE, k_wire_mark, kgrid, dim3(256), 0, Wa, 0);
      }
      break;
    default: return CHOCO_E_UNSUPPORTED;
  }
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

int choco_unpack_messages(choco_ctx* ctx, const void* msgs_dev, float* q_dev) {
  if (!ctx || !msgs_dev || !q_dev) return CHOCO_E_INVAL;
  if (((uintptr_t)msgs_dev & 3u) != 0 || ((uintptr_t)q_dev & 15u) != 0) return CHOCO_E_INVAL;
  const int rc = wire_supported(ctx);
  if (rc != CHOCO_OK) return rc;
  const WireArgs Wa = wire_args(ctx);
  const uint32_t* msg = (const uint32_t*)msgs_dev;
  const dim3 wgrid((unsigned)((Wa.W + 255) / 256), (unsigned)Wa.n);
  const dim3 kgrid((unsigned)((Wa.k + 255) / 256), (unsigned)Wa.n);
  const dim3 lgrid((unsigned)((ctx->wire_plane_words + 255) / 256), (unsigned)Wa.n);
  // every entry of q is written: pad columns and entries not sent are zero (the dense decoders
  // write whole 4-vectors up to d themselves, so they need the fill only for a wider ld)
  if (ctx->sparse || Wa.nlayers || Wa.ld > ((int64_t)Wa.d + 3) / 4 * 4)
    LAUNCH(ctx, KID_WIRE, k_wire_zero, dim3((unsigned)((Wa.ld + 1023) / 1024), (unsigned)Wa.n), dim3(256), 0, q_dev,
           Wa.ld);
  switch (ctx->cfg.compressor) {
    case CHOCO_Q_SIGN:
      if (Wa.nlayers) LAUNCH(ctx, KID_WIRE, k_unpack_dense_layers<false>, lgrid, dim3(256), 0, Wa, msg, q_dev);
      else LAUNCH(ctx, KID_WIRE, k_unpack_sign, wgrid, dim3(256), 0, Wa, msg, q_dev);
      break;
    case CHOCO_Q_QSGD:
      if (Wa.nlayers) LAUNCH(ctx, KID_WIRE, k_unpack_dense_layers<true>, lgrid, dim3(256), 0, Wa, msg, q_dev);
      else if (Wa.levels < 256)
        LAUNCH(ctx, KID_WIRE, k_unpack_gsgd<true>, wgrid, dim3(256), (size_t)(1 + Wa.mb) * 1024, Wa, msg, q_dev);
      else
        LAUNCH(ctx, KID_WIRE, k_unpack_gsgd<false>, wgrid, dim3(256), (size_t)(1 + Wa.mb) * 1024, Wa, msg, q_dev);
      break;
    case CHOCO_Q_TOPK: LAUNCH(ctx, KID_WIRE, k_unpack_topk, kgrid, dim3(256), 0, Wa, msg, q_dev); break;
    case CHOCO_Q_RANDK:
      if (Wa.bitmap_words) {
        LAUNCH(ctx, KID_WIRE, k_unpack_randk, dim3((unsigned)Wa.n), dim3(1024),
               (size_t)Wa.bitmap_words * sizeof(uint32_t), Wa, msg, q_dev);
      } else {
        launch_rank_tables(ctx, Wa);
        LAUNCH(ctx, KID_WIRE, k_unpack_randk_ranked, dim3((unsigned)((Wa.k + 3) / 4), (unsigned)Wa.n), dim3(256), 0,
               Wa, msg, q_dev);
        LAUNCH(ctx, KID_WIRE, k_wire_mark, kgrid, dim3(256), 0, Wa, 0);
      }
      break;
    default: return CHOCO_E_UNSUPPORTED;
  }
  LAUNCH_CHECK(ctx);
  return CHOCO_OK;
}

int choco_set_capture(choco_ctx* ctx, int32_t* codes_dev) {
  if (!ctx) return CHOCO_E_INVAL;
  if (ctx->cfg.compressor != CHOCO_Q_SIGN && ctx->cfg.compressor != CHOCO_Q_QSGD) return CHOCO_E_INVAL;
  if (((uintptr_t)codes_dev & 15u) != 0) return CHOCO_E_INVAL;
  ctx->args.codes = codes_dev;
  return CHOCO_OK;
}

int choco_layer_scalars(choco_ctx* ctx, double* scalars_host) {
  if (!ctx || !scalars_host || ctx->nlayers == 0) return CHOCO_E_INVAL;

  const Args& A = ctx->args;
  HIP_TRY(ctx, hipMemcpyAsync(scalars_host, ctx->layer_scal_buf[ctx->last_buf], (size_t)A.n * (size_t)A.nlayers * 4 * sizeof(double),
                              hipMemcpyDeviceToHost, ctx->stream));
  const size_t nlong = ctx->long_layers.size();
  std::vector<WorkerCtl> ctl((size_t)A.n * nlong);
  if (nlong) {
    const int rc = join_lookahead(ctx);   // the control blocks may be under the next step's selection
    if (rc != CHOCO_OK) return rc;
  }
  if (nlong)
    HIP_TRY(ctx, hipMemcpyAsync(ctl.data(), A.ctl, ctl.size() * sizeof(WorkerCtl), hipMemcpyDeviceToHost, ctx->stream));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  for (size_t b = 0; b < nlong; ++b)
    for (int i = 0; i < A.n; ++i) {
      const WorkerCtl& c = ctl[b * (size_t)A.n + (size_t)i];
      double* o = scalars_host + ((size_t)i * (size_t)A.nlayers + (size_t)ctx->long_layers[b].id) * 4;
      o[0] = (double)(uint32_t)(c.kstar >> 32);
      o[1] = o[2] = 0.0;
      o[3] = c.mode == 0u ? 1.0 : 0.0;
    }
  return CHOCO_OK;
}

int choco_last_scalars(choco_ctx* ctx, double* scalars_host) {
  if (!ctx || !scalars_host) return CHOCO_E_INVAL;
  if (ctx->nlayers > 0) return CHOCO_E_UNSUPPORTED;
  {
    const int rc = join_lookahead(ctx);   // the control blocks may be under the next step's selection
    if (rc != CHOCO_OK) return rc;
  }
  const Args& A = ctx->args;
  std::vector<WorkerCtl> ctl((size_t)A.n);
  HIP_TRY(ctx, hipMemcpyAsync(ctl.data(), A.ctl, ctl.size() * sizeof(WorkerCtl), hipMemcpyDeviceToHost,
                              ctx->stream));
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  for (int i = 0; i < A.n; ++i) {
    double* o = scalars_host + 6 * i;
    const WorkerCtl& c = ctl[(size_t)i];
    o[0] = o[1] = o[2] = o[3] = o[4] = o[5] = 0.0;
    switch (ctx->cfg.compressor) {
      case CHOCO_Q_SIGN: o[0] = c.stat; o[1] = (double)c.scale_c; break;
      case CHOCO_Q_QSGD: o[0] = c.stat; o[1] = c.nrm; o[2] = (double)c.scale_r; o[3] = (double)c.scale_step; break;
      case CHOCO_Q_TOPK:
      case CHOCO_Q_RANDK:
        o[0] = (double)(uint32_t)(c.kstar >> 32);
        o[1] = (double)(uint32_t)(~(uint32_t)(c.kstar & 0xFFFFFFFFu));
        o[2] = (double)c.kept;
        o[3] = (double)c.mode;
        o[4] = (double)c.fallbacks;
        o[5] = (double)c.last_candidates;
        break;
      default: break;
    }
  }
  return CHOCO_OK;
}

int choco_get_mix_form(choco_ctx* ctx, int32_t* mix_form_host) {
  if (!ctx || !mix_form_host) return CHOCO_E_INVAL;
  *mix_form_host = ctx->mix_form;
  return CHOCO_OK;
}

int choco_get_step(choco_ctx* ctx, uint64_t* t_host) {
  if (!ctx || !t_host) return CHOCO_E_INVAL;
  *t_host = ctx->t;
  return CHOCO_OK;
}

int choco_set_step(choco_ctx* ctx, uint64_t t) {
  if (!ctx) return CHOCO_E_INVAL;
  if (t != ctx->t) ctx->cur.valid = ctx->nxt.valid = false;   // selections made ahead were for the old counter
  ctx->t = t;
  return CHOCO_OK;
}

int choco_set_lookahead(choco_ctx* ctx, int enable) {
  if (!ctx) return CHOCO_E_INVAL;
  ctx->lookahead = ctx->can_lookahead && enable != 0;
  if (!ctx->lookahead) ctx->cur.valid = ctx->nxt.valid = false;   // selections already under way are joined and made again
  return CHOCO_OK;
}

int choco_sync(choco_ctx* ctx) {
  if (!ctx) return CHOCO_E_INVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  if (ctx->aux_stream) HIP_TRY(ctx, hipStreamSynchronize(ctx->aux_stream));   // a selection made ahead writes the workspace
  return CHOCO_OK;
}

int choco_set_profiling(choco_ctx* ctx, int enable) {
  if (!ctx) return CHOCO_E_INVAL;
  ctx->profiling = enable != 0;
  if (enable) ctx->ev_used = 0;
  return CHOCO_OK;
}

int choco_profile_report(choco_ctx* ctx, char* buf_host, size_t buf_bytes) {
  if (!ctx || !buf_host || buf_bytes == 0) return CHOCO_E_INVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  double total_ms[KID_COUNT] = {0};
  long count[KID_COUNT] = {0};
  for (size_t e = 0; e < ctx->ev_used; ++e) {
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, ctx->ev_begin[e], ctx->ev_end[e]) != hipSuccess) continue;
    total_ms[ctx->ev_kernel[e]] += (double)ms;
    count[ctx->ev_kernel[e]] += 1;
  }
  size_t used = 0;
  buf_host[0] = 0;
  for (int k = 0; k < KID_COUNT; ++k) {
    if (!count[k]) continue;
    const int w = snprintf(buf_host + used, buf_bytes - used, "%s %ld %.6f\n", kKernelNames[k], count[k],
                           total_ms[k]);
    if (w < 0 || (size_t)w >= buf_bytes - used) return CHOCO_E_NOMEM;
    used += (size_t)w;
  }
  ctx->ev_used = 0;
  return CHOCO_OK;
}

int choco_destroy(choco_ctx* ctx) {
  if (!ctx) return CHOCO_OK;
  release_ctx(ctx);
  return CHOCO_OK;
}

int choco_last_hip_error(choco_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

}  // extern "C"
