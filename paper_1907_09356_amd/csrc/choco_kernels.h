// Device code of the CHOCO-Gossip / CHOCO-SGD step for gfx950 (wave64).
//
// Layout: all arrays are n x ld fp32, row-major, one row per worker, ld a
// multiple of 4 so every row starts 16-byte aligned and a lane can always load
// a whole 4-vector (the pad columns d..ld-1 are read but never take part in a
// norm, a histogram or a selection).
//
// Launch shape: the streaming kernels use one block per contiguous chunk (no
// grid-stride loops) and, for states that do not fit in cache, non-temporal
// loads and stores; on MI355X that shape measured 6.4 TB/s on a 3-read/1-write
// stream against 4.9-5.3 TB/s for persistent grid-stride loops.
//
// Arithmetic rules shared with no other code: every fp32 product and sum is
// rounded on its own (compiled with -ffp-contract=off), neighbour
// contributions are added in CSR order, norms are accumulated in fp64 over a
// fixed three-level tree (chunks of 256 consecutive entries, 4 per lane and a
// 64-lane butterfly; groups of 16 chunk sums, butterfly; 256 strided lanes over
// the group sums and a halving tree).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace choco {

enum { Q_IDENTITY = 0, Q_TOPK = 1, Q_RANDK = 2, Q_SIGN = 3, Q_QSGD = 4, Q_NONE = 5 };
enum { STREAM_RANDK = 1, STREAM_DITHER = 2 };

typedef float vf4 __attribute__((ext_vector_type(4)));
typedef int vi4 __attribute__((ext_vector_type(4)));

constexpr int kBins = 2048;       // radix-select digits are at most 11 bits wide
constexpr int kBins16 = 65536;    // first digit of the fallback histogram (16 bits)
constexpr int kChunk = 256;       // entries per first-level norm chunk / tile width
constexpr int kGroup = 16;        // chunks per second-level group (4096 entries)
constexpr int kStreamVecs = 2;    // 4-vectors per thread in the streaming kernels
constexpr int kCompactVecs = 4;   // 4-vectors per thread in the select pass (long rows; short rows take 2)
constexpr int kStageCap = 1024;   // candidates one block stages in LDS before its single append
constexpr int kSmallCap = 1024;   // entries of the threshold bin the select ranks directly in LDS
// Chunks per wave in the norm passes (a workgroup takes a group of 16 chunks): one, in
// 1024-thread workgroups, where the state is streamed past the caches (large states, and the
// small ones that are latency-bound), two, in 512-thread workgroups, where it is read through
// them (n = 64, d = 270 k, layer by layer: 47 against 52 us; the other way round the large
// and the small states lose 3-4 %).
constexpr int stat_cpw(bool nt) { return nt ? 1 : 2; }
constexpr int stat_threads(bool nt) { return 64 * (16 / stat_cpw(nt)); }
constexpr int kFallbackBlocks = 64; // blocks per worker of the (normally idle) fallback passes
constexpr int kRefineParts = 16;    // blocks per worker of the select when the candidate lists are long
constexpr int kSegs = 32;         // candidate sub-lists per worker (spreads the append counter)
constexpr int kOvfRing = 8;       // gsgd: remembered entries at the top level per worker (and layer); a step adds at most 4

// Per-worker control block in device memory (written by small "finalise" code,
// read by the streaming kernels; the host never reads it on the hot path).
struct WorkerCtl {
  // norms and scales of the dense operators (Appendix C: sign, gsgd_b)
  double stat;        // ||v||_1 (sign) or sum v^2 (gsgd)
  double nrm;         // ||v||_2 (gsgd)
  float scale_c;      // sign: ||v||_1 / d
  float scale_r;      // gsgd: s / ||v||_2
  float scale_step;   // gsgd: ||v||_2 / (tau s)
  int32_t nonzero;    // gsgd: ||v||_2 > 0
  // radix select of the sparsifying operators (Appendix C: top_a, random_a)
  uint32_t guess_key;   // entries with key32 >= this are appended to the candidate list
  uint32_t bin_shift;   // the select bins candidates by min((key32 - guess_key) >> bin_shift, 2047)
  uint32_t mode;        // 0: candidate list is complete, 1: rebuild it, 2: scan the row
  uint32_t seg_count[kSegs];  // entries with key32 >= guess_key appended per sub-list (may exceed seg_cap)
  uint32_t kept;        // number of entries emitted by the last selection
  uint32_t fallbacks;   // how many steps needed a fallback (histogram rebuild or row scan)
  uint32_t last_candidates;  // length of the candidate list the last select worked on
  uint32_t emit_count;  // multi-block select: kept entries emitted so far
  uint32_t small_count; // multi-block select: entries of the threshold bin collected so far
  // the fallback's workgroups of this worker: how many have histogrammed their share so far (never
  // reset: 'the last one in' is by remainder), the number of the round whose guess is placed, and
  // 'a workgroup gave up waiting: do not trust the list' (cleared when the next guess is placed)
  uint32_t fb_arrive, fb_go, fb_abort;
  uint64_t kstar;       // composite key of the k-th largest entry: kept <=> key >= kstar
};

// One layer of a worker's vector when the operator is applied layer by layer.
struct LayerDesc {
  int32_t start;     // first entry
  int32_t len;       // entries
  int32_t k;         // top_a / random_a: entries kept of this layer
  int32_t sel_base;  // where the layer's kept entries start in the worker's selection list
  int32_t id;        // number of the layer in the caller's table
  int32_t head;      // start mod 4: the kernels that hold a layer in registers load whole 4-vectors
                     // from start - head and ignore the first `head` entries (0 in an aligned table)
  int32_t pad[2];
};

// Scales of one layer of one worker (dense operators applied layer by layer).
struct LayerScale {
  float c, r, step;
  int32_t nonzero;
};

// One work item of the layer-wise norm pass: a group of up to 16 chunks of one layer.
struct LayerGroup {
  int32_t off;   // first entry of the group in the row (a multiple of 4)
  int32_t rem;   // entries of the layer from there to its end
  int32_t id;    // the layer
  int32_t pad;
};

// One long layer of a layer-wise top_a / random_a configuration (it takes the guessed-threshold
// select of the whole-row path on its own piece of the rows).
struct LongSel {
  int32_t base;        // the 4-vector boundary at or below the layer's first entry
  int32_t d;           // entries from there to the layer's end
  int32_t e_lo;        // ... of which the first e_lo lie before the layer
  int32_t k;           // kept entries
  int32_t sel_base;    // the layer's first slot in a worker's kept lists
  int32_t set;         // which control blocks (n per layer) and which set of select scratch
  uint32_t cand_cap, seg_cap, extra, want, delta0, sample_stride, sample_need;   // see Args
  int64_t set_cand;    // candidate entries from one set of lists to the next
};

struct Args {
  int32_t n;
  int32_t d;
  int64_t ld;
  float* X;
  float* Xhat;
  float* S;
  const int32_t* row_ptr;
  const int32_t* col;
  const float* w;
  WorkerCtl* ctl;
  float gamma;
  // fused local update (choco_step): when G is non-null the first pass over X of the step
  // also does x <- x - lr * g (Algorithm 1, local gradient step) before using x
  const float* G;
  float lr;
  float* M;              // momentum memory (Algorithm 2) or null for plain SGD
  float beta, lambda;    // momentum factor and weight decay of Algorithm 2
  int32_t deferred_sgd;  // the local update is applied by the LAST kernel of the step (random_a)
  // dense operators
  double* chunk_sums;  // n x nchunks first-level sums (only the printed-order tile kernel writes them)
  double* group_sums;  // n x ngroups second-level sums
  int32_t nchunks;
  int32_t ngroups;
  int32_t levels;      // gsgd: s
  double tau;          // gsgd: 1 + min(d/s^2, sqrt(d)/s) or 1
  int32_t* codes;      // optional capture of the transmitted codes (n x ld)
  // The message of a dense operator as it goes on the wire, written by the pass that encodes q
  // (Appendix C: one sign bit per entry for sign; b bits per entry for gsgd_b): bit e%32 of
  // word e/32 of plane p of row i.  Plane 0: the entry is negative (and, for gsgd, its level
  // is not zero); planes 1..mb (gsgd): bit p-1 of min(level, 2^mb - 1).
  uint32_t* planes;    // n x nplanes x plane_words (null: identity, top_a, random_a)
  int64_t plane_words; // ceil(ld / 32)
  int32_t nplanes;     // 1 (sign) or 1 + mb (gsgd)
  int32_t mb;          // gsgd: magnitude bits = bit length of s - 1 (at least 1)
  // gsgd: an entry at level s when s does not fit the magnitude bits is remembered by index in a
  // small ring per worker (and layer), tagged with the step: {t_lo, t_hi + 1, index, 0}
  uint4* ovf_ring;     // n x max(nlayers, 1) x kOvfRing
  uint32_t* ovf_pos;   // n x max(nlayers, 1): entries appended so far (never reset)
  int32_t fold_finalise;  // ngroups <= 256: the apply kernel does level 3 of the norm tree itself
  // sparse operators
  int64_t k;
  uint32_t* hist16;    // n x kBins16 (fallback histogram)
  uint2* cand;         // n x kSegs x seg_cap  (a, index)
  uint32_t* hist_parts; // n x kRefineParts x kBins: per-block candidate histograms (multi-block select)
  uint2* small_list;   // n x kSmallCap: entries of the threshold bin (multi-block select)
  uint32_t seg_cap;    // capacity of one sub-list
  uint32_t cand_cap;   // largest total the fallback aims to stay under
  uint32_t sample_stride;  // the fallback histogram looks at every sample_stride-th 4-vector
  uint32_t sample_need;    // rank (within the sample) at which the fallback puts the guess
  uint32_t spin_limit;     // polls after which a waiting workgroup of the fallback gives up
  uint32_t want;       // entries the next guess should leave above it now: extra (+ k for top_a)
  uint32_t extra;      // candidates wanted beyond k: max(k/2, 6 sqrt(k) + 32)
  uint32_t delta0;     // default distance of the guess below the threshold key
  int32_t* sel_idx;    // n x sel_stride: kept indices (slot m of worker i at i * sel_stride + m)
  float* sel_val;      // n x sel_stride: their values
  // The select kernels see one "row" of d entries per worker of which k are kept.  That is the
  // whole vector, or one long layer of it: then X, Xhat, G, M and the kept-entry map point at the
  // layer's first entry, sel_idx / sel_val at the layer's first slot, and
  int64_t sel_stride;  // slots per worker in sel_idx / sel_val (k for the whole vector)
  int32_t idx_base;    // is added to the kept indices (the layer's first entry; 0 for the whole vector)
  uint32_t vec_base;   // is added to the 4-vector number that keys the random words (idx_base / 4)
  uint32_t* keptmap;   // n x map_words: bit e of row j set <=> worker j kept entry e this step (rows without a
                       // bitmap built in LDS: set with atomics by the select, cleared by the xhat update; a bit
                       // per entry keeps the scatter's look-ups in the caches, bytes did not)
  int64_t map_words;   // ceil(ld / 32)
  uint32_t* bitmap;    // n x bitmap_words: the same as bits, used instead when a row's bitmap fits in LDS
  int64_t bitmap_words;  // 0: use the bit map in global memory (keptmap)
  int32_t fold_xhat;     // the final mix also applies xhat += q (bitmap rows, compress-then-mix)
  // random_a: nobody knows the kept values when the selection is made (it reads no state).  With
  // incremental sums k_sel_values gathers them for the scatter; otherwise they are listed by the
  // kernel that forms q anyway:
  int32_t update_values;   // k_xhat_update computes q_j[e] = x_j[e] - xhat_j[e] itself and stores it (direct mix)
  float* Qv;               // or, where one fused pass applies the update and the mix (direct form), to entry
                           // (j, e) of this n x ld array, from which the list is gathered on request; else null
  int32_t randk_rescale;
  float randk_scale;   // (float)(d / k)
  // layer-wise compression (nlayers = 0: the whole row is compressed as one vector)
  const LayerDesc* layers;   // sorted by start, disjoint
  int32_t nlayers;
  int32_t layers_generic;    // 0: every layer starts on a multiple of 4 and the layers tile the row up to that
                             // padding (a 4-vector then lies in one layer); 1: any disjoint ascending slices
  int32_t e_lo;              // select kernels: entries of the row below this index do not take part (the head
                             // of a long layer that does not start on a multiple of 4; else 0)
  const LongSel* long_tab;   // batched select launches: the long layers that one launch covers (grid.z / grid.y)
  const LayerDesc* layer_work;  // the same by falling length: the order the layer kernel takes them in
  uint32_t* layer_guess;     // n x nlayers: top_a threshold key of the last step (all ones: none yet)
  const LayerGroup* layer_groups;   // ngroup_items work items of the layer-wise norm pass, layer after layer
  const int32_t* layer_group_first; // nlayers + 1: where each layer's items start
  int32_t ngroup_items;
  double* layer_group_sums;  // n x ngroup_items second-level norm sums
  LayerScale* layer_scale;   // n x nlayers: scales of the last step (sign, gsgd)
  const int4* chunk_layer;   // per 256-entry chunk of a row: layer of its first entry, that layer's end, next layer's start
  double* layer_scal;        // n x nlayers x 4: norms and scales / threshold of the last step
  int32_t qsgd_biased;
  // randomness
  uint32_t seed_lo, seed_hi, t_lo, t_hi;
};

// The select kernels' view of one long layer: the argument block of the whole-row select made
// to point at the layer's piece of the rows, its slots of the kept lists, its control blocks
// and its candidate lists.  The host builds the view for a launch that covers one layer; a
// launch that covers several builds it per workgroup from the table.
__host__ __device__ __forceinline__ Args long_view(const Args& src, const LongSel& L) {
  Args R = src;
  R.X += L.base;
  R.Xhat += L.base;
  if (R.G) R.G += L.base;
  if (R.M) R.M += L.base;
  R.d = L.d;
  R.e_lo = L.e_lo;
  R.k = L.k;
  R.ctl = src.ctl + (int64_t)L.set * src.n;
  R.sel_idx += L.sel_base;     // sel_stride stays the worker's whole list
  R.sel_val += L.sel_base;
  R.idx_base = L.base;
  R.vec_base = (uint32_t)L.base >> 2;
  R.cand_cap = L.cand_cap;
  R.seg_cap = L.seg_cap;
  R.extra = L.extra;
  R.want = L.want;
  R.delta0 = L.delta0;
  R.sample_stride = L.sample_stride;
  R.sample_need = L.sample_need;
  R.cand = src.cand + (int64_t)L.set * L.set_cand;
  return R;
}

// The layer that holds entry e of a row.
__device__ __forceinline__ int layer_of(const Args& A, int e) {
  int lo = 0, hi = A.nlayers - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (A.layers[mid].start <= e) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

// Generic tables: the layer that holds entry e, or -1 if e lies in no layer.
__device__ __forceinline__ int layer_holding(const Args& A, int e) {
  if (e < A.layers[0].start) return -1;
  const int lay = layer_of(A, e);
  const LayerDesc L = A.layers[lay];
  return e < L.start + L.len ? lay : -1;
}

// The same for the first entry e of a 4-vector through the per-chunk table: the layer
// that holds the chunk's first entry, then forward (layers shorter than a chunk are rare).
// Every 4-vector starts inside a layer; `nvalid` is how many of its entries the layer has.
__device__ __forceinline__ int layer_of_vector(const Args& A, int e, int& nvalid) {
  const int4 ci = A.chunk_layer[e >> 8];   // {layer of the chunk's first entry, its end, start of the next layer}
  int lay = ci.x, end = ci.y;
  if (e >= ci.z) {                         // the chunk holds a layer boundary and e lies past it
    while (lay + 1 < A.nlayers && A.layers[lay + 1].start <= e) ++lay;
    const LayerDesc L = A.layers[lay];
    end = L.start + L.len;
  }
  const int left = end - e;
  nvalid = left < 4 ? left : 4;
  return lay;
}

// Entries of a 4-vector that lie in the padding after a layer (or in the pad columns after
// the row's last entry) are not compressed: they keep their xhat and send the code 0.
__device__ __forceinline__ void mask_padding(int nvalid, const vf4& xh_old, vf4& xh_new, vi4& code) {
#pragma unroll
  for (int c = 1; c < 4; ++c)
    if (c >= nvalid) {
      xh_new[c] = xh_old[c];
      code[c] = 0;
    }
}

// random_a, unbiased version: the factor d / k of the vector entry e was compressed in
// (Appendix C) - the whole row, or the layer of e.
__device__ __forceinline__ float randk_scale_at(const Args& A, int e) {
  if (!A.nlayers) return A.randk_scale;
  const LayerDesc L = A.layers[layer_of(A, e)];
  return (float)((double)L.len / (double)L.k);
}

// ---------------------------------------------------------------------------
// Memory helpers.  NT = non-temporal (streaming) access.
// ---------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ vf4 load4(const float* p) {
  const vf4* q = reinterpret_cast<const vf4*>(p);
  return NT ? __builtin_nontemporal_load(q) : *q;
}
template <bool NT>
__device__ __forceinline__ void store4(float* p, vf4 v) {
  vf4* q = reinterpret_cast<vf4*>(p);
  if (NT) __builtin_nontemporal_store(v, q);
  else *q = v;
}
// The local update of one 4-vector at offset o, riding on a pass that has x in registers:
//   plain (Algorithm 1, gradient step): x <- x - lr g
//   momentum (Algorithm 2, its momentum and gradient steps): m <- (g + lambda x) + beta m (stored);  x <- x - lr m
// Every product and sum rounded on its own, as in k_sgd / k_momentum.
template <bool NT, class ArgsT>
__device__ __forceinline__ vf4 local_update4(const ArgsT& A, int64_t o, vf4 x) {
  const vf4 g = load4<true>(A.G + o);   // a gradient is read once: always streamed
  if (A.M) {
    vf4 m = load4<NT>(A.M + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float gg = g[c] + A.lambda * x[c];
      const float mn = gg + A.beta * m[c];
      m[c] = mn;
      x[c] = x[c] - A.lr * mn;
    }
    store4<NT>(A.M + o, m);
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) x[c] = x[c] - A.lr * g[c];
  }
  return x;
}

// The same on values already in registers (g, and m if there is a momentum memory, loaded
// by the caller together with its other loads); m is updated in place, the caller stores it.
template <class ArgsT>
__device__ __forceinline__ vf4 local_update_regs(const ArgsT& A, vf4 x, const vf4& g, vf4& m) {
  if (A.M) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float gg = g[c] + A.lambda * x[c];
      const float mn = gg + A.beta * m[c];
      m[c] = mn;
      x[c] = x[c] - A.lr * mn;
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) x[c] = x[c] - A.lr * g[c];
  }
  return x;
}

// One entry of x as this step sees it.  random_a under choco_step: no pass reads X before
// the final mix, so the local update is folded into that mix and the few entries that the
// select and the scatter gather are updated on the fly (same operations on the same, not
// yet updated, x, g and m).
template <class ArgsT>
__device__ __forceinline__ float x_entry(const ArgsT& A, int64_t o) {
  const float x = A.X[o];
  if (!A.deferred_sgd) return x;
  if (A.M) {
    const float gg = A.G[o] + A.lambda * x;
    const float mn = gg + A.beta * A.M[o];
    return x - A.lr * mn;
  }
  return x - A.lr * A.G[o];
}
__device__ __forceinline__ vf4 lds_load4(const float* p) { return *reinterpret_cast<const vf4*>(p); }
__device__ __forceinline__ void lds_store4(float* p, vf4 v) { *reinterpret_cast<vf4*>(p) = v; }

// ---------------------------------------------------------------------------
// Philox4x32, 10 rounds (Salmon et al., SC'11): counter-based, so the word for
// (seed, step, worker, index) is the same in whatever order entries are visited.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    // one 32 x 32 -> 64 bit product per counter word (a single multiply-add instruction on this
    // target; written as two separate products it costs two quarter-rate multiplies)
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  return make_uint4(c0, c1, c2, c3);
}

// Four words for entries 4m .. 4m+3 of a worker on one stream.
__device__ __forceinline__ uint4 random_words(const Args& A, int worker, uint32_t m, uint32_t stream) {
  return philox4x32_10(m, (uint32_t)worker, A.t_lo, stream | (A.t_hi << 8), A.seed_lo, A.seed_hi);
}

__device__ __forceinline__ uint32_t pick(const uint4& v, int c) {
  return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w;
}

// 64-lane butterfly sum in fp64; every lane ends with the halving-tree result
// t[l] += t[l+off] for off = 32,16,...,1 (the sum is commutative, so the xor
// exchange builds exactly that tree in every lane).
__device__ __forceinline__ double wave_tree_sum(double t) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) t = t + __shfl_xor(t, off, 64);
  return t;
}

// The same over aligned sub-groups of kGroup = 16 lanes (halving 8,4,2,1): lanes
// 16q..16q+15 end with the tree sum of their own 16 values.
__device__ __forceinline__ double group_tree_sum(double t) {
#pragma unroll
  for (int off = kGroup / 2; off >= 1; off >>= 1) t = t + __shfl_xor(t, off, 64);
  return t;
}

// ---------------------------------------------------------------------------
// Element-wise encoders of the dense operators.  v is one entry of x - xhat.
// ---------------------------------------------------------------------------
template <int COMP>
struct RowScale {
  float c, r, step;
  int nonzero;
  __device__ __forceinline__ void load(const WorkerCtl* ctl) {
    if (COMP == Q_SIGN) c = ctl->scale_c;
    if (COMP == Q_QSGD) { r = ctl->scale_r; step = ctl->scale_step; nonzero = ctl->nonzero; }
  }
  __device__ __forceinline__ void load(const LayerScale& ls) {
    c = ls.c; r = ls.r; step = ls.step; nonzero = ls.nonzero;
  }
};

template <int COMP>
__device__ __forceinline__ float encode(float v, const RowScale<COMP>& sc, uint32_t word, int32_t& code) {
  if (COMP == Q_IDENTITY) { code = 0; return v; }
  const bool neg = v < 0.0f;
  if (COMP == Q_SIGN) {              // (||v||_1/d) sgn(v), sgn = -1 iff v < 0
    code = neg ? -1 : 1;
    return neg ? -sc.c : sc.c;
  }
  // gsgd_b: level = floor(s |v| / ||v||_2 + u), value = sig(v) * level * ||v||_2 / (tau s)
  int32_t level = 0;
  if (sc.nonzero) {
    const float u = (float)(word >> 8) * (1.0f / 16777216.0f);
    const float a = fabsf(v) * sc.r;
    level = (int32_t)floorf(a + u);
  }
  const float mag = (float)level * sc.step;
  code = neg ? -level : level;
  return neg ? -mag : mag;
}

// xhat += Q(x - xhat) on one 4-vector (Algorithm 1: compression and update of the public copy).
template <int COMP>
__device__ __forceinline__ vf4 absorb(const vf4& x, vf4 xh, const RowScale<COMP>& sc, const uint4& words,
                                      vi4& code) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    int32_t cd;
    const float v = x[c] - xh[c];
    const float qv = encode<COMP>(v, sc, pick(words, c), cd);
    xh[c] = xh[c] + qv;
    code[c] = cd;
  }
  return xh;
}

// The same for a generic layer table (any disjoint ascending slices): every entry takes the
// scales of the layer that holds it; an entry in no layer keeps its xhat and sends nothing.
template <int COMP>
__device__ __forceinline__ vf4 absorb_by_entry(const Args& A, int r, int e, const vf4& x, vf4 xh,
                                               const uint4& words, vi4& code) {
  int fl = e >= A.layers[0].start ? layer_of(A, e) : -1;   // last layer that starts at or before the entry
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int ee = e + c;
    while (fl + 1 < A.nlayers && A.layers[fl + 1].start <= ee) ++fl;
    code[c] = 0;
    if (fl < 0 || ee >= A.d) continue;
    const LayerDesc L = A.layers[fl];
    if (ee >= L.start + L.len) continue;
    RowScale<COMP> sc;
    sc.load(A.layer_scale[(int64_t)r * A.nlayers + fl]);
    int32_t cd;
    const float v = x[c] - xh[c];
    const float qv = encode<COMP>(v, sc, pick(words, c), cd);
    xh[c] = xh[c] + qv;
    code[c] = cd;
  }
  return xh;
}

// Workgroups are handed to the eight accelerator dies in turn (workgroup b runs on die b mod 8) and
// every die has an L2 of its own.  A tile of 256 columns writes 32 bytes of each bit plane, a
// quarter of a cache line; tile number for workgroup b such that the four tiles of a line run on
// one die one after the other (b, b + 8, b + 16, b + 24), so that their pieces meet in that die's
// L2 and leave it as one whole line.  Super-groups of 32 tiles keep the order of the streams
// otherwise; the last, partial super-group is left as it is.
__device__ __forceinline__ int line_sharing_tile(int b, int ntiles) {
  const int base = b & ~31;
  if (base + 32 > ntiles) return b;
  return base + ((b & 7) << 2) + ((b >> 3) & 3);
}

// The bits of a wave's 256 codes (four per lane, entries e..e+3 of row r) go to the row's bit
// planes: eight lanes share a 32-bit word, their nibbles are combined with three lane moves and
// the first of the eight stores the word.  Every lane of the wave calls this (lanes without
// entries pass code 0); `lay` is the layer of the lane's entries (0 without layers).
template <int COMP>
__device__ __forceinline__ void emit_code_planes(const Args& A, int r, int e, int lane, const vi4& code, int lay) {
  if (COMP != Q_SIGN && COMP != Q_QSGD) return;
  if (!A.planes) return;
  const int sh = 4 * (lane & 7);
  const bool writer = (lane & 7) == 0 && e < A.d;
  uint32_t* P = A.planes + (int64_t)r * A.nplanes * A.plane_words + ((uint32_t)e >> 5);
  // OR over the eight lanes of a word with three data-parallel-primitive moves (no LDS traffic,
  // unlike a general lane exchange): lane ^ 1 and lane ^ 2 inside the quad, then the mirror image
  // inside the group of eight, which lies in the other quad
  auto word_of = [&](uint32_t nibble) {
    uint32_t w = nibble << sh;
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x141, 0xF, 0xF, true);   // row_half_mirror
    return w;
  };
  // bits 0, 8, 16, 24 of y -> bits 0..3
  auto nibble_of = [](uint32_t y) {
    y |= y >> 7;
    y |= y >> 14;
    return y & 0xFu;
  };
  // one byte per entry: bit 7 = negative, bits 0..6 = min(level, 2^mb - 1) (levels above 127 are
  // handled plane by plane below)
  const uint32_t negs = ((uint32_t)code[0] >> 31) | (((uint32_t)code[1] >> 31) << 8) |
                        (((uint32_t)code[2] >> 31) << 16) | (((uint32_t)code[3] >> 31) << 24);
  // (a plane with no bit set anywhere in the wave - the usual case for the upper magnitude planes
  // of a long vector, whose levels are nearly all 0 or 1 - is stored as zeros without the lane moves)
  if (__ballot(negs != 0u) == 0ull) {
    if (writer) P[0] = 0u;
  } else {
    const uint32_t sw = word_of(nibble_of(negs));
    if (writer) P[0] = sw;
  }
  if (COMP == Q_QSGD) {
    const int32_t maxmag = (1 << A.mb) - 1;
    int32_t mag[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      mag[c] = code[c] < 0 ? -code[c] : code[c];
      if (mag[c] > maxmag) {   // the level s itself: at most four entries of a vector can reach it
        const int lay_c = (A.nlayers && A.layers_generic) ? layer_holding(A, e + c) : lay;
        const int64_t unit = A.nlayers ? (int64_t)r * A.nlayers + lay_c : (int64_t)r;
        const int32_t base = A.nlayers ? A.layers[lay_c].start : 0;
        const uint32_t pos = atomicAdd(A.ovf_pos + unit, 1u);
        A.ovf_ring[unit * kOvfRing + (pos & (uint32_t)(kOvfRing - 1))] =
            make_uint4(A.t_lo, A.t_hi + 1u, (uint32_t)(e + c - base), 0u);
        mag[c] = maxmag;
      }
    }
    for (int p0 = 0; p0 < A.mb; p0 += 8) {   // eight planes at a time out of one byte per entry
      const uint32_t M = ((uint32_t)(mag[0] >> p0) & 0xFFu) | (((uint32_t)(mag[1] >> p0) & 0xFFu) << 8) |
                         (((uint32_t)(mag[2] >> p0) & 0xFFu) << 16) | (((uint32_t)(mag[3] >> p0) & 0xFFu) << 24);
      const int pend = A.mb - p0 < 8 ? A.mb - p0 : 8;
      for (int p = 0; p < pend; ++p) {
        const uint32_t y = (M >> p) & 0x01010101u;
        uint32_t w = 0u;
        if (__ballot(y != 0u) != 0ull) w = word_of(nibble_of(y));
        if (writer) P[(int64_t)(1 + p0 + p) * A.plane_words] = w;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Local updates (the gradient step of Algorithm 1; the momentum and gradient steps of Algorithm 2).
// grid (ceil(nvec / (256 * kStreamVecs)), n)
// ---------------------------------------------------------------------------
template <bool NT>
__global__ __launch_bounds__(256) void k_sgd(float* X, const float* G, int64_t ld, int32_t nvec, float lr) {
  const int64_t row = (int64_t)blockIdx.y * ld;
  const int m0 = blockIdx.x * (256 * kStreamVecs) + threadIdx.x;
  vf4 x[kStreamVecs], g[kStreamVecs];
#pragma unroll
  for (int u = 0; u < kStreamVecs; ++u) {
    const int m = m0 + u * 256;
    if (m < nvec) {
      x[u] = load4<NT>(X + row + 4 * (int64_t)m);
      g[u] = load4<NT>(G + row + 4 * (int64_t)m);
    }
  }
#pragma unroll
  for (int u = 0; u < kStreamVecs; ++u) {
    const int m = m0 + u * 256;
    if (m < nvec) {
#pragma unroll
      for (int c = 0; c < 4; ++c) x[u][c] = x[u][c] - lr * g[u][c];
      store4<NT>(X + row + 4 * (int64_t)m, x[u]);
    }
  }
}

template <bool NT>
__global__ __launch_bounds__(256) void k_momentum(float* X, const float* G, float* M, int64_t ld,
                                                  int32_t nvec, float lr, float beta, float lambda) {
  const int64_t row = (int64_t)blockIdx.y * ld;
  const int m0 = blockIdx.x * (256 * kStreamVecs) + threadIdx.x;
  vf4 x[kStreamVecs], g[kStreamVecs], mo[kStreamVecs];   // all loads before the first store
#pragma unroll
  for (int u = 0; u < kStreamVecs; ++u) {
    const int m = m0 + u * 256;
    if (m < nvec) {
      const int64_t o = row + 4 * (int64_t)m;
      x[u] = load4<NT>(X + o);
      g[u] = load4<NT>(G + o);
      mo[u] = load4<NT>(M + o);
    }
  }
#pragma unroll
  for (int u = 0; u < kStreamVecs; ++u) {
    const int m = m0 + u * 256;
    if (m < nvec) {
      const int64_t o = row + 4 * (int64_t)m;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float gg = g[u][c] + lambda * x[u][c];
        const float mn = gg + beta * mo[u][c];
        mo[u][c] = mn;
        x[u][c] = x[u][c] - lr * mn;
      }
      store4<NT>(M + o, mo[u]);
      store4<NT>(X + o, x[u]);
    }
  }
}

// ---------------------------------------------------------------------------
// Norm tree.
// ---------------------------------------------------------------------------
template <int COMP>
__device__ __forceinline__ double norm_term(float v) {
  const double a = (double)v;
  return COMP == Q_SIGN ? fabs(a) : a * a;
}

// ((t0 + t1) + t2) + t3 with entries past d counting as +0.0
template <int COMP>
__device__ __forceinline__ double lane_terms(const vf4& v, int e, int d) {
  double acc = (e < d) ? norm_term<COMP>(v[0]) : 0.0;
  acc = acc + ((e + 1 < d) ? norm_term<COMP>(v[1]) : 0.0);
  acc = acc + ((e + 2 < d) ? norm_term<COMP>(v[2]) : 0.0);
  acc = acc + ((e + 3 < d) ? norm_term<COMP>(v[3]) : 0.0);
  return acc;
}

// Per-worker scales from the finished norm sum (Appendix C: sign, gsgd_b); fp64
// sqrt and divisions, rounded once to fp32.  Optionally recorded in the control block.
template <int COMP>
__device__ __forceinline__ void scales_from_total(const Args& A, double total, RowScale<COMP>& sc,
                                                  WorkerCtl* record) {
  double nrm = 0.0;
  sc.c = sc.r = sc.step = 0.0f;
  sc.nonzero = 0;
  if (COMP == Q_SIGN) {
    sc.c = (float)(total / (double)A.d);
  } else if (COMP == Q_QSGD) {
    nrm = sqrt(total);
    const double s = (double)A.levels;
    sc.nonzero = nrm > 0.0 ? 1 : 0;
    sc.r = nrm > 0.0 ? (float)(s / nrm) : 0.0f;
    sc.step = nrm > 0.0 ? (float)(nrm / (A.tau * s)) : 0.0f;
  }
  if (record) {
    record->stat = total;
    record->nrm = nrm;
    record->scale_c = sc.c;
    record->scale_r = sc.r;
    record->scale_step = sc.step;
    record->nonzero = sc.nonzero;
  }
}

// Level 3 of the norm tree done by one wave when there are at most 256 group
// sums: lane l stands for tree lanes l, l+64, l+128, l+192 (one group sum each),
// the halvings by 128 and 64 are two adds in registers and the rest is the wave
// butterfly - the same additions in the same order as k_dense_finalise.
__device__ __forceinline__ double wave_level3(const Args& A, int i, int lane) {
  const double* gs = A.group_sums + (int64_t)i * A.ngroups;
  double a0 = lane < A.ngroups ? gs[lane] : 0.0;
  double a1 = lane + 64 < A.ngroups ? gs[lane + 64] : 0.0;
  const double a2 = lane + 128 < A.ngroups ? gs[lane + 128] : 0.0;
  const double a3 = lane + 192 < A.ngroups ? gs[lane + 192] : 0.0;
  a0 = a0 + a2;
  a1 = a1 + a3;
  a0 = a0 + a1;
  return wave_tree_sum(a0);
}

// Third level of the tree over the group sums and the per-worker scales.
// grid n, block 256.  (A separate launch on purpose: handing the group sums to a
// "last block" of the producing kernel needs a device-scope fence per block,
// which on this multi-die part writes back the L2 and cost 8x the pass itself.)
template <int COMP>
__global__ __launch_bounds__(256) void k_dense_finalise(Args A) {
  __shared__ double sh[256];
  const int i = blockIdx.x, l = threadIdx.x;
  const double* gs = A.group_sums + (int64_t)i * A.ngroups;
  // lane l adds group sums l, l+256, ... in that order; loads run eight ahead of the adds
  double acc = 0.0;
  bool first = true;
  for (int g0 = l; g0 < A.ngroups; g0 += 256 * 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int g = g0 + 256 * u;
      v[u] = g < A.ngroups ? gs[g] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (g0 + 256 * u < A.ngroups) {
        acc = first ? v[u] : acc + v[u];
        first = false;
      }
    }
  }
  sh[l] = acc;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if (l < off) sh[l] = sh[l] + sh[l + off];
    __syncthreads();
  }
  if (l == 0) {
    RowScale<COMP> sc;
    scales_from_total<COMP>(A, sh[0], sc, A.ctl + i);
  }
}

// Dense operators, statistic pass (compress-then-mix order): v = x - xhat, one
// block per group of 16 chunks (4096 entries), one wave per CPW chunks, all of them
// in flight at once (CPW = stat_cpw(NT)).  grid (ngroups, n), block stat_threads(NT).  One chunk
// per wave (1024 threads) against four (256 threads): n = 8, d = 270 k 10.8 against 11.8 us (the
// launch is a single round of workgroups and lasts as long as one of them), d = 28 M 571 against
// 597 us.
template <int COMP, bool NT>
__global__ __launch_bounds__(stat_threads(NT)) void k_dense_stat(Args A) {
  constexpr int CPW = stat_cpw(NT);
  __shared__ double cs[kGroup];
  const int i = blockIdx.y, g = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float* x = A.X + (int64_t)i * A.ld;
  const float* xh = A.Xhat + (int64_t)i * A.ld;
  vf4 a[CPW], b[CPW];
  int e[CPW];
#pragma unroll
  for (int u = 0; u < CPW; ++u) {
    const int c = g * kGroup + CPW * wave + u;
    e[u] = c < A.nchunks ? c * kChunk + lane * 4 : A.d;   // chunks past the end hold nothing
    if (e[u] < A.d) {
      a[u] = load4<NT>(x + e[u]);
      b[u] = load4<NT>(xh + e[u]);
    }
  }
  if (A.G) {   // fused local update: x <- x - lr g, stored for the apply pass
    float* xw = A.X + (int64_t)i * A.ld;
    vf4 g[CPW];   // all gradient loads before the first store (see compact_chunk); the momentum
                // memory, when there is one, is read in turn: registers for it would cost occupancy
#pragma unroll
    for (int u = 0; u < CPW; ++u)
      if (e[u] < A.d) g[u] = load4<true>(A.G + (int64_t)i * A.ld + e[u]);
#pragma unroll
    for (int u = 0; u < CPW; ++u) {
      if (e[u] < A.d) {
        vf4 mm = vf4{0.f, 0.f, 0.f, 0.f};
        if (A.M) mm = load4<NT>(A.M + (int64_t)i * A.ld + e[u]);
        a[u] = local_update_regs(A, a[u], g[u], mm);
        if (A.M) store4<NT>(A.M + (int64_t)i * A.ld + e[u], mm);
        store4<NT>(xw + e[u], a[u]);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < CPW; ++u) {
    double t = 0.0;
    if (e[u] < A.d) {
      const vf4 v = a[u] - b[u];
      t = lane_terms<COMP>(v, e[u], A.d);
    }
    t = wave_tree_sum(t);
    if (lane == 0) cs[CPW * wave + u] = t;
  }
  __syncthreads();
  if (wave == 0) {
    const double t = group_tree_sum(lane < kGroup ? cs[lane] : 0.0);
    if (lane == 0) A.group_sums[(int64_t)i * A.ngroups + g] = t;
  }
}

// Second level from chunk sums already in memory (printed order: the tile kernel
// below produces chunk sums).  Sixteen lanes per group, four groups per wave;
// grid (ceil(ngroups/16), n), block 256.
__global__ __launch_bounds__(256) void k_group_reduce(Args A) {
  const int i = blockIdx.y;
  const int g = (blockIdx.x * 256 + threadIdx.x) / kGroup;
  const int c = g * kGroup + (threadIdx.x & (kGroup - 1));
  double t = (g < A.ngroups && c < A.nchunks) ? A.chunk_sums[(int64_t)i * A.nchunks + c] : 0.0;
  t = group_tree_sum(t);
  if (g < A.ngroups && (threadIdx.x & (kGroup - 1)) == 0) A.group_sums[(int64_t)i * A.ngroups + g] = t;
}

// ---------------------------------------------------------------------------
// Dense operators, fused apply + mix, compress-then-mix order, direct form.
// One block owns a tile of 256 consecutive columns for ALL n rows, so every
// xhat row is read from HBM once and shared through LDS by the (at most 5)
// workers that mix with it:
//   phase 1  q = Q(x - xhat), xhat += q   (Algorithm 1, compression and exchange), new xhat -> HBM + LDS
//   phase 2  x += gamma * sum_p w_p (xhat_j - xhat_i)   (its mixing step), CSR order, from LDS
// A block has NW waves (4 for n <= 16, else 16); wave w owns rows w, w+NW, ...; RPW = rows
// per wave (compile-time bound, x stays in registers between the phases).  Dynamic LDS:
// n * 256 floats (64 KiB at n = 64: two 1024-thread blocks per CU keep it fully occupied).
// ---------------------------------------------------------------------------
// The rows of W that a wave mixes (up to four), fetched when the kernel starts, beside the loads
// of x and xhat: lane 16 q + j holds neighbour j of the wave's q-th row - its weight, and its
// column with the row's length above it - and the mix reads them back lane by lane (readlane:
// no memory access in the loop but the tile's).  A row with more than 16 neighbours is read from
// memory in the loop instead.  (Read there for every row - the row pointers, then the columns
// and weights, then the tile rows - this was a chain of dependent fetches during which the
// workgroup had no load in flight: 4.0 of the 13.6 us a workgroup lived at n = 64.  Scalar loads
// inside the loop were slower still: they share a counter with the LDS loads, and every wait
// for one is a wait for all.)
constexpr int kNbrLanes = 16;

struct RowNbrs {
  int col_deg;   // column | row length << 8
  float w;
};

// In two steps, so that a kernel can put the first behind the loads it issues first and the
// second where those have returned: where the lane's row starts and how long it is ...
struct RowSpan {
  int beg, deg;
};

template <int RPW, int NW>
__device__ __forceinline__ RowSpan nbr_span(const Args& A, int wave, int lane) {
  static_assert(RPW * kNbrLanes <= 64, "a lane group per row of the wave");
  RowSpan sp{0, 0};
  const int q = lane / kNbrLanes;
  const int r = wave + NW * q;
  if (q < RPW && r < A.n) {
    sp.beg = A.row_ptr[r];
    sp.deg = A.row_ptr[r + 1] - sp.beg;
  }
  return sp;
}

// ... and the lane's neighbour of that row.
__device__ __forceinline__ RowNbrs nbr_fetch(const Args& A, const RowSpan& sp, int lane) {
  RowNbrs nb{sp.deg << 8, 0.0f};
  const int j = lane % kNbrLanes;
  if (j < sp.deg) {
    nb.col_deg |= A.col[sp.beg + j];
    nb.w = A.w[sp.beg + j];
  }
  return nb;
}

template <int RPW, int NW>
__device__ __forceinline__ void tile_mix_rows_staged(const Args& A, const float* tile, int wave, int lane,
                                                     bool valid, vf4 (&xr)[RPW], const RowNbrs& nb) {
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (r < A.n) {                                   // uniform over the wave (readlane takes every lane)
      const vf4 me = lds_load4(tile + r * kChunk + lane * 4);
      vf4 acc = {0.f, 0.f, 0.f, 0.f};
      const int deg = __builtin_amdgcn_readlane(nb.col_deg, q * kNbrLanes) >> 8;
      if (deg <= kNbrLanes) {                        // neighbours in the order of the CSR row
        for (int j = 0; j < deg; ++j) {
          const int cj = __builtin_amdgcn_readlane(nb.col_deg, q * kNbrLanes + j) & 0xFF;
          const float wj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(nb.w), q * kNbrLanes + j));
          const vf4 o = lds_load4(tile + cj * kChunk + lane * 4);
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[c] = acc[c] + wj * (o[c] - me[c]);
        }
      } else {
        const int pbeg = A.row_ptr[r];
        for (int p = pbeg; p < pbeg + deg; ++p) {
          const float wj = A.w[p];
          const vf4 o = lds_load4(tile + A.col[p] * kChunk + lane * 4);
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[c] = acc[c] + wj * (o[c] - me[c]);
        }
      }
      if (valid) {
#pragma unroll
        for (int c = 0; c < 4; ++c) xr[q][c] = xr[q][c] + A.gamma * acc[c];
      }
    }
  }
}

// The same with every row of W read from memory in the loop (k_dense_apply_mix, whose registers
// and issue slots before the barrier are spoken for by the encoding: staged rows made it 3-7 %
// slower at n = 8 and no faster at n = 64).
template <int RPW, int NW>
__device__ __forceinline__ void tile_mix_rows(const Args& A, const float* tile, int wave, int lane,
                                              bool valid, vf4 (&xr)[RPW]) {
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (r < A.n && valid) {
      const vf4 me = lds_load4(tile + r * kChunk + lane * 4);
      vf4 acc = {0.f, 0.f, 0.f, 0.f};
      const int pend = A.row_ptr[r + 1];
      for (int p = A.row_ptr[r]; p < pend; ++p) {
        const float wj = A.w[p];
        const vf4 o = lds_load4(tile + A.col[p] * kChunk + lane * 4);
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = acc[c] + wj * (o[c] - me[c]);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) xr[q][c] = xr[q][c] + A.gamma * acc[c];
    }
  }
}

// LAYERED: the operator is applied layer by layer; the scales come per (worker, layer) from
// the layer-wise norm pass.
template <int COMP, int RPW, int NW, bool CAPTURE, bool NT, bool LAYERED>
__global__ __launch_bounds__(64 * NW) void k_dense_apply_mix(Args A) {
  extern __shared__ float tile[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int tile_no = line_sharing_tile((int)blockIdx.x, (int)gridDim.x);
  const int e = tile_no * kChunk + lane * 4;
  const bool valid = e < A.d;
  int lay = 0, nvalid = A.d - e < 4 ? A.d - e : 4;   // the last 4-vector of a row may end in pad columns
  const bool generic = LAYERED && A.layers_generic;   // a 4-vector may span layers and gaps: scales entry by entry
  if (LAYERED && valid && !generic) lay = layer_of_vector(A, e, nvalid);
  vf4 xr[RPW], xh[RPW];
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (r < A.n && valid) {
      const int64_t o = (int64_t)r * A.ld + e;
      xr[q] = load4<NT>(A.X + o);
      xh[q] = load4<NT>(A.Xhat + o);
    }
  }
  // scales of this wave's rows: read from the control block, or (few group sums) finished here
  RowScale<COMP> sc[RPW];
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (LAYERED) {
      if (r < A.n && valid && !generic) sc[q].load(A.layer_scale[(int64_t)r * A.nlayers + lay]);
    } else if (r < A.n) {
      if ((COMP == Q_SIGN || COMP == Q_QSGD) && A.fold_finalise) {
        const double total = wave_level3(A, r, lane);
        scales_from_total<COMP>(A, total, sc[q], (tile_no == 0 && lane == 0) ? A.ctl + r : nullptr);
      } else {
        sc[q].load(A.ctl + r);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (r < A.n) {
      vf4 nh = {0.f, 0.f, 0.f, 0.f};
      vi4 code = {0, 0, 0, 0};
      if (valid) {
        const int64_t o = (int64_t)r * A.ld + e;
        uint4 words = make_uint4(0, 0, 0, 0);
        if (COMP == Q_QSGD) words = random_words(A, r, (uint32_t)(e >> 2), STREAM_DITHER);
        if (generic) {
          nh = absorb_by_entry<COMP>(A, r, e, xr[q], xh[q], words, code);
        } else {
          nh = absorb<COMP>(xr[q], xh[q], sc[q], words, code);
          mask_padding(nvalid, xh[q], nh, code);
        }
        store4<NT>(A.Xhat + o, nh);
        if (CAPTURE) *reinterpret_cast<vi4*>(A.codes + o) = code;
      }
      emit_code_planes<COMP>(A, r, e, lane, code, lay);   // the message itself: sign and level bits
      lds_store4(tile + r * kChunk + lane * 4, nh);
    }
  }
  __syncthreads();
  tile_mix_rows<RPW, NW>(A, tile, wave, lane, valid, xr);
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (r < A.n && valid) store4<NT>(A.X + (int64_t)r * A.ld + e, xr[q]);
  }
}

// ---------------------------------------------------------------------------
// Tile mix with the xhat that is in memory now (Algorithm 1, mixing step, direct
// form), optionally followed by the chunk sums of v = x_new - xhat for the
// printed order (mix, then compress).  Same tiling as above; the tile is one
// first-level norm chunk, so the chunk sum falls out of one wave butterfly.
// ---------------------------------------------------------------------------
// SPARSE (top_a / random_a, compress-then-mix order): the update of the public copies rides on
// this pass.  The wave that loads (x, xhat) of a row also reads the row's kept-entry bits for its
// 4-vectors; where a bit is set it forms q = x - xhat (x with this step's local update, which
// the pass may itself carry), adds it to xhat, stores that 4-vector of xhat and hands the new
// value to the tile, so that the mix sees the xhat of after the exchange.  Rows whose bits live
// in the global bit map clear the words they used (as k_xhat_update does).
template <int STAT, int RPW, int NW, bool NT, bool SPARSE>
__global__ __launch_bounds__(64 * NW) void k_tile_mix(Args A) {
  extern __shared__ float tile[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int e = blockIdx.x * kChunk + lane * 4;
  const bool valid = e < A.d;
  const bool sgd = A.G != nullptr, mom = sgd && A.M != nullptr;
  RowSpan span{0, 0};
  RowNbrs nb{0, 0.0f};
  // The loads of (up to) two of the wave's rows first - x, xhat, the gradient, the kept-entry
  // word -, then their arithmetic and stores: a store, or a test of a loaded word, between two
  // loads would put the later load behind the round trip of the earlier one.  Two rows at a
  // time because four rows' loads at once need more than the 64 registers that let two
  // 1024-thread workgroups share a compute unit at n = 64 (57 against 43 us); the momentum
  // memory is read row by row for the same reason.
  constexpr int HB = RPW >= 2 ? 2 : 1;
  vf4 xr[RPW];
#pragma unroll
  for (int q0 = 0; q0 < RPW; q0 += HB) {
    vf4 xhv[HB], gv[HB];
    uint32_t word[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) {
      const int q = q0 + j;
      const int r = wave + NW * q;
      word[j] = 0u;
      if (q < RPW && r < A.n && valid) {
        const int64_t o = (int64_t)r * A.ld + e;
        xr[q] = load4<NT>(A.X + o);
        xhv[j] = load4<NT>(A.Xhat + o);
        if (sgd) gv[j] = load4<true>(A.G + o);   // a gradient is read once: always streamed
        if (SPARSE)
          word[j] = A.bitmap_words ? A.bitmap[(int64_t)r * A.bitmap_words + ((uint32_t)e >> 5)]
                                   : A.keptmap[(int64_t)r * A.map_words + ((uint32_t)e >> 5)];
      }
    }
    // the rows of W for the mix: the row pointers behind the first rows' loads, the neighbours
    // where those have returned (the arithmetic below waits for them anyway)
    if (q0 == 0) span = nbr_span<RPW, NW>(A, wave, lane);
#pragma unroll
    for (int j = 0; j < HB; ++j) {
      const int q = q0 + j;
      const int r = wave + NW * q;
      if (q0 == 0 && j == 0) nb = nbr_fetch(A, span, lane);
      if (q < RPW && r < A.n) {
        vf4 xh = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
          const int64_t o = (int64_t)r * A.ld + e;
          xh = xhv[j];
          if (sgd) {
            vf4 mv = vf4{0.f, 0.f, 0.f, 0.f};
            if (mom) mv = load4<NT>(A.M + o);
            xr[q] = local_update_regs(A, xr[q], gv[j], mv);
            if (mom) store4<NT>(A.M + o, mv);
          }
          if (SPARSE) {
            const uint32_t bits = (word[j] >> ((uint32_t)e & 31u)) & 0xFu;
            if (bits) {
#pragma unroll
              for (int c = 0; c < 4; ++c)
                if ((bits >> c) & 1u) {
                  float qv = xr[q][c] - xh[c];
                  if (A.randk_rescale) qv = randk_scale_at(A, e + c) * qv;
                  xh[c] = xh[c] + qv;
                  if (A.Qv) A.Qv[o + c] = qv;
                }
              store4<false>(A.Xhat + o, xh);
            }
            // eight lanes share a word of 32 entries; the lane of its first 4-vector clears it
            // (every lane's load of the word has returned by now: the test above needed its value)
            if (!A.bitmap_words && word[j] != 0u && (lane & 7) == 0)
              A.keptmap[(int64_t)r * A.map_words + ((uint32_t)e >> 5)] = 0u;
          }
        }
        lds_store4(tile + r * kChunk + lane * 4, xh);
      }
    }
  }
  __syncthreads();
  tile_mix_rows_staged<RPW, NW>(A, tile, wave, lane, valid, xr, nb);
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + NW * q;
    if (r < A.n) {
      double t = 0.0;
      if (valid) {
        store4<NT>(A.X + (int64_t)r * A.ld + e, xr[q]);
        if (STAT != Q_NONE) {
          const vf4 v = xr[q] - lds_load4(tile + r * kChunk + lane * 4);
          t = lane_terms<STAT>(v, e, A.d);
        }
      }
      if (STAT != Q_NONE) {
        t = wave_tree_sum(t);
        if (lane == 0) A.chunk_sums[(int64_t)r * A.nchunks + blockIdx.x] = t;
      }
    }
  }
}

// Element-wise xhat += Q(x - xhat) (Algorithm 1, compression and exchange) with no mixing.
// grid (ceil(nvec / (256 * kStreamVecs)), n)
template <int COMP, bool CAPTURE, bool NT, bool LAYERED>
__global__ __launch_bounds__(256) void k_dense_apply(Args A) {
  const int i = blockIdx.y;
  RowScale<COMP> sc;
  if (!LAYERED) sc.load(A.ctl + i);
  const int nvec = (A.d + 3) >> 2;
  const int m0 = blockIdx.x * (256 * kStreamVecs) + threadIdx.x;
  vf4 xs[kStreamVecs], xhs[kStreamVecs];   // all loads before the first store
#pragma unroll
  for (int u = 0; u < kStreamVecs; ++u) {
    const int m = m0 + u * 256;
    if (m < nvec) {
      const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
      xs[u] = load4<NT>(A.X + o);
      xhs[u] = load4<NT>(A.Xhat + o);
    }
  }
#pragma unroll
  for (int u = 0; u < kStreamVecs; ++u) {
    const int m = m0 + u * 256;
    vi4 code = {0, 0, 0, 0};
    int lay = 0;
    if (m < nvec) {
      const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
      const vf4 x = xs[u];
      const vf4 xh = xhs[u];
      uint4 words = make_uint4(0, 0, 0, 0);
      if (COMP == Q_QSGD) words = random_words(A, i, (uint32_t)m, STREAM_DITHER);
      int nvalid = A.d - 4 * m < 4 ? A.d - 4 * m : 4;   // the last 4-vector of a row may end in pad columns
      vf4 nh;
      if (LAYERED && A.layers_generic) {
        nh = absorb_by_entry<COMP>(A, i, 4 * m, x, xh, words, code);
      } else {
        if (LAYERED) {
          lay = layer_of_vector(A, 4 * m, nvalid);
          sc.load(A.layer_scale[(int64_t)i * A.nlayers + lay]);
        }
        nh = absorb<COMP>(x, xh, sc, words, code);
        mask_padding(nvalid, xh, nh, code);
      }
      store4<NT>(A.Xhat + o, nh);
      if (CAPTURE) *reinterpret_cast<vi4*>(A.codes + o) = code;
    }
    // (every lane of the wave: a wave's 4-vectors are consecutive, eight lanes to a word)
    emit_code_planes<COMP>(A, i, m < nvec ? 4 * m : A.d, threadIdx.x & 63, code, lay);
  }
}

// Direct-form mix reading neighbour rows from global memory (any n; used when
// the tile of all rows does not fit in LDS).  grid (ceil(nvec/256), n)
__global__ __launch_bounds__(256) void k_mix_direct_global(Args A) {
  const int i = blockIdx.y;
  const int nvec = (A.d + 3) >> 2;
  const int pbeg = A.row_ptr[i], pend = A.row_ptr[i + 1];
  const int m = blockIdx.x * 256 + threadIdx.x;
  if (m >= nvec) return;
  const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
  const vf4 me = load4<false>(A.Xhat + o);
  vf4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int p = pbeg; p < pend; ++p) {
    const float wj = A.w[p];
    const vf4 ot = load4<false>(A.Xhat + (int64_t)A.col[p] * A.ld + 4 * (int64_t)m);
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = acc[c] + wj * (ot[c] - me[c]);
  }
  vf4 x = load4<false>(A.X + o);
#pragma unroll
  for (int c = 0; c < 4; ++c) x[c] = x[c] + A.gamma * acc[c];
  store4<false>(A.X + o, x);
}

// Incremental-form mix: x_i += gamma (S_i - xhat_i).  Pure streaming, 16 B/entry.
// grid (ceil(nvec / (256 * VECS)), n).  VECS 4-vectors per thread, a wave's pieces consecutive
// (VECS KiB per array and wave): 4 for long rows (6.1 against 6.0 TB/s at d = 28 M), 2 for
// short ones (twice the blocks: 50 against 53 us at n = 64, d = 270 k).
template <bool NT, int VECS, int THREADS = 256>
__global__ __launch_bounds__(THREADS) void k_mix_incremental(Args A) {
  const int i = blockIdx.y;
  const int nvec = (A.d + 3) >> 2;
  // a wave's VECS 4-vectors are consecutive 1 KiB pieces (wave-contiguous)
  const int m0 = blockIdx.x * (THREADS * VECS) + (threadIdx.x >> 6) * (64 * VECS) + (threadIdx.x & 63);
  vf4 x[VECS], s[VECS], xh[VECS];
#pragma unroll
  for (int u = 0; u < VECS; ++u) {
    const int m = m0 + u * 64;
    if (m < nvec) {
      const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
      x[u] = load4<NT>(A.X + o);
      s[u] = load4<NT>(A.S + o);
      xh[u] = load4<NT>(A.Xhat + o);
      if (A.G) x[u] = local_update4<NT>(A, o, x[u]);
      if (A.fold_xhat) {
        // short rows, compress-then-mix order: xhat += q for this step's kept entries
        // (Algorithm 1, update of the public copies) rides on this pass, read off the worker's bitmap
        const uint32_t e = 4u * (uint32_t)m;
        const uint32_t bits = (A.bitmap[(int64_t)i * A.bitmap_words + (e >> 5)] >> (e & 31u)) & 0xFu;
        if (bits) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if ((bits >> c) & 1u) {
              float q = x[u][c] - xh[u][c];
              if (A.randk_rescale) q = A.randk_scale * q;
              xh[u][c] = xh[u][c] + q;
            }
          store4<false>(A.Xhat + o, xh[u]);
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < VECS; ++u) {
    const int m = m0 + u * 64;
    if (m < nvec) {
#pragma unroll
      for (int c = 0; c < 4; ++c) x[u][c] = x[u][c] + A.gamma * (s[u][c] - xh[u][c]);
      store4<NT>(A.X + (int64_t)i * A.ld + 4 * (int64_t)m, x[u]);
    }
  }
}

// ---------------------------------------------------------------------------
// Radix select for top_a / random_a.
//
// Every entry gets a 64-bit composite key  K = (key32 << 32) | ~index  where
//   top_a:    key32 = bits(v) & 0x7fffffff   (monotone in |v| for finite v)
//   random_a: key32 = ~word                  (k smallest words = k largest ~word)
// All composites of a worker are distinct, so "the k largest K" is exactly the
// selection rule (|v| descending, or word ascending; ties to the lower index).
//
// Fast path (every step): ONE pass over the row appends the entries with
// key32 >= guess to a short candidate list; if the list holds at least k (and at
// most its capacity) entries it contains the k largest, and the exact k-th
// composite kstar is found by a radix select over the list alone.  The guess for
// the next step is placed below this step's threshold so that about k + extra
// entries qualify.  Fallback (first step, or when the distribution moved): a
// 16-bit histogram of key32 over the row fixes a guess that is certainly low
// enough, and the list is rebuilt; if even one 16-bit bucket overflows the list,
// the select scans the row itself.  Either way the result is exact.
// ---------------------------------------------------------------------------
template <int COMP>
struct Digits {
  // the six digits of the composite key, most significant first
  __device__ __forceinline__ static int shift(int level) {
    if (COMP == Q_TOPK) return level == 0 ? 52 : level == 1 ? 41 : level == 2 ? 32 : level == 3 ? 21 : level == 4 ? 10 : 0;
    return level == 0 ? 53 : level == 1 ? 42 : level == 2 ? 32 : level == 3 ? 21 : level == 4 ? 10 : 0;
  }
  __device__ __forceinline__ static int bits(int level) {
    if (COMP == Q_TOPK) return level == 2 ? 9 : level == 5 ? 10 : 11;
    return (level == 2 || level == 5) ? 10 : 11;
  }
  __device__ __forceinline__ static uint32_t key32(uint32_t a) {
    return COMP == Q_TOPK ? (a & 0x7fffffffu) : a;
  }
  __device__ __forceinline__ static uint64_t composite(uint32_t a, uint32_t idx) {
    return ((uint64_t)key32(a) << 32) | (uint64_t)(~idx);
  }
  __device__ __forceinline__ static uint32_t bin16(uint32_t a) {
    return COMP == Q_TOPK ? (key32(a) >> 15) : (a >> 16);
  }
  __device__ __forceinline__ static uint32_t bin16_floor(uint32_t bin) {   // smallest key32 in a bucket
    return COMP == Q_TOPK ? (bin << 15) : (bin << 16);
  }
};

// The candidate list of a worker holds the k largest entries iff at least k
// entries qualified in total and no sub-list overflowed.
__device__ __forceinline__ bool list_is_good(const WorkerCtl* ctl, const Args& A) {
  uint64_t total = 0;
  bool fits = true;
#pragma unroll
  for (int s = 0; s < kSegs; ++s) {
    const uint32_t c = ctl->seg_count[s];
    total += c;
    fits = fits && (c <= A.seg_cap);
  }
  return fits && total >= (uint64_t)A.k;
}

// a[c] for the four entries of 4-vector m of worker i (raw bits of v for top_a,
// complemented random word for random_a).  DO_MIX (top_a, printed order with
// incremental sums): first x += gamma (S - xhat), stored, then v = x - xhat.
// FIRST: this is the step's first pass over X (the only one that may carry the fused
// local update x <- x - lr g).
template <int COMP, bool DO_MIX, bool NT, bool FIRST>
__device__ __forceinline__ void entry_bits(const Args& A, int i, int m, uint32_t (&a)[4]) {
  if (COMP == Q_TOPK) {
    const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
    vf4 x = load4<NT>(A.X + o);
    const vf4 xh = load4<NT>(A.Xhat + o);
    const bool sgd = FIRST && A.G != nullptr;
    if (sgd) x = local_update4<NT>(A, o, x);
    if (DO_MIX) {
      const vf4 s = load4<NT>(A.S + o);
#pragma unroll
      for (int c = 0; c < 4; ++c) x[c] = x[c] + A.gamma * (s[c] - xh[c]);
    }
    if (DO_MIX || sgd) store4<NT>(A.X + o, x);
#pragma unroll
    for (int c = 0; c < 4; ++c) a[c] = __float_as_uint(x[c] - xh[c]);
  } else {
    const uint4 wds = random_words(A, i, A.vec_base + (uint32_t)m, STREAM_RANDK);
    a[0] = ~wds.x; a[1] = ~wds.y; a[2] = ~wds.z; a[3] = ~wds.w;
  }
}

// Append the candidates (key32 >= guess) among the 256 * VECS 4-vectors of
// one chunk of worker i to sub-list chunk % kSegs.  Hits are staged in LDS and
// flushed with one global atomic per block.
template <int COMP, bool DO_MIX, bool NT, bool FIRST, int VECS, int THREADS = 256>
__device__ __forceinline__ void compact_chunk(const Args& A, int i, int chunk, uint2* stage,
                                              uint32_t* s_count, uint32_t* s_base) {
  WorkerCtl* ctl = A.ctl + i;
  const uint32_t guess = ctl->guess_key;
  const int seg = chunk % kSegs;
  uint2* cand = A.cand + ((int64_t)i * kSegs + seg) * A.seg_cap;
  const int nvec = (A.d + 3) >> 2;
  // a wave's VECS 4-vectors are consecutive 1 KiB pieces of the row
  const int m0 = chunk * (THREADS * VECS) + (threadIdx.x >> 6) * (64 * VECS) + (threadIdx.x & 63);
  uint32_t a[VECS][4];
  if (COMP == Q_TOPK) {
    // all loads of the chunk first, then the arithmetic and the stores: a store to X between
    // two groups of loads would hold the later loads back (the compiler must assume that the
    // arrays overlap)
    const bool sgd = FIRST && A.G != nullptr;
    const bool mom = sgd && A.M != nullptr;
    vf4 x[VECS], xh[VECS], g[VECS], sm[VECS];   // sm: S (DO_MIX) or the momentum
#pragma unroll
    for (int u = 0; u < VECS; ++u) {
      const int m = m0 + u * 64;
      if (m < nvec) {
        const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
        x[u] = load4<NT>(A.X + o);
        xh[u] = load4<NT>(A.Xhat + o);
        if (sgd) g[u] = load4<true>(A.G + o);
        if (DO_MIX) sm[u] = load4<NT>(A.S + o);
        else if (mom) sm[u] = load4<NT>(A.M + o);
      }
    }
#pragma unroll
    for (int u = 0; u < VECS; ++u) {
      const int m = m0 + u * 64;
      if (m < nvec) {
        const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
        if (sgd) {
          if (DO_MIX) {           // S occupies the spare registers: the momentum is read here
            vf4 mm = vf4{0.f, 0.f, 0.f, 0.f};
            if (mom) mm = load4<NT>(A.M + o);
            x[u] = local_update_regs(A, x[u], g[u], mm);
            if (mom) store4<NT>(A.M + o, mm);
          } else {
            x[u] = local_update_regs(A, x[u], g[u], sm[u]);
            if (mom) store4<NT>(A.M + o, sm[u]);
          }
        }
        if (DO_MIX) {
#pragma unroll
          for (int c = 0; c < 4; ++c) x[u][c] = x[u][c] + A.gamma * (sm[u][c] - xh[u][c]);
        }
        if (DO_MIX || sgd) store4<NT>(A.X + o, x[u]);
#pragma unroll
        for (int c = 0; c < 4; ++c) a[u][c] = __float_as_uint(x[u][c] - xh[u][c]);
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < VECS; ++u) {
      const int m = m0 + u * 64;
      if (m < nvec) entry_bits<COMP, DO_MIX, NT, FIRST>(A, i, m, a[u]);
    }
  }
#pragma unroll
  for (int u = 0; u < VECS; ++u) {
    const int m = m0 + u * 64;
    if (m < nvec) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int e = 4 * m + c;
        const uint32_t key = Digits<COMP>::key32(a[u][c]);
        if (e >= A.e_lo && e < A.d && key >= guess) {
          const uint32_t slot = atomicAdd(s_count, 1u);
          if (slot < (uint32_t)kStageCap) {
            stage[slot] = make_uint2(a[u][c], (uint32_t)e);
          } else {   // more hits than the stage holds: append one by one
            const uint32_t pos = atomicAdd(&ctl->seg_count[seg], 1u);
            if (pos < A.seg_cap) cand[pos] = make_uint2(a[u][c], (uint32_t)e);
          }
        }
      }
    }
  }
  __syncthreads();
  const uint32_t count = *s_count < (uint32_t)kStageCap ? *s_count : (uint32_t)kStageCap;
  if (count != 0) {
    if (threadIdx.x == 0) *s_base = atomicAdd(&ctl->seg_count[seg], count);
    __syncthreads();
    const uint32_t base = *s_base;
    for (uint32_t t = threadIdx.x; t < count; t += THREADS)
      if (base + t < A.seg_cap) cand[base + t] = stage[t];
  }
}

// The one pass of the fast path: every worker, one block per chunk.
// grid (ceil(nvec / (THREADS * VECS)), n), block THREADS.  Chunks of 4096 entries for long rows,
// of 2048 for short ones (twice the blocks and the occupancy: 49 against 57 us at n = 64,
// d = 270 k).  A long row's chunk: top_a one 4-vector per thread of 1024 threads (6.2 TB/s at
// d = 28 M; four per thread of 256 threads 6.0; two per thread 5.5), random_a four per thread of
// 256 threads (its pass draws Philox words beside another pass and should get in its way little).
// BATCH: grid.z counts the long layers of A.long_tab, grid.x covers the longest of them (the
// workgroups past a shorter layer's end leave at once).
template <int COMP, bool DO_MIX, bool NT, int VECS, bool BATCH = false, int THREADS = 256>
__global__ __launch_bounds__(THREADS) void k_sel_compact(Args A0) {
  __shared__ uint2 stage[kStageCap];
  __shared__ uint32_t s_count, s_base;
  const Args A = BATCH ? long_view(A0, A0.long_tab[blockIdx.z]) : A0;
  if (BATCH && (int64_t)blockIdx.x * (THREADS * VECS) >= (int64_t)((A.d + 3) >> 2)) return;
  if (threadIdx.x == 0) s_count = 0;
  __syncthreads();
  compact_chunk<COMP, DO_MIX, NT, true, VECS, THREADS>(A, blockIdx.y, blockIdx.x, stage, &s_count, &s_base);
}

// The fallback of a failed guess on a long row, one launch.  A workgroup whose worker's list is
// good leaves at once: a step whose guesses held pays for one launch of workgroups that read one
// control block each.  For a worker whose list is not good, its workgroups
//   1. histogram the top 16 bits of key32 over a sample of the row (every sample_stride-th
//      4-vector; stride 1 = the whole row) and then count themselves in; the last one in
//   2. walks the histogram from the top to the bucket at which the count reaches sample_need,
//      puts the guess at its floor, sets the worker's mode for this step (with the whole row
//      histogrammed it also knows whether the rebuilt list will fit; a sampled histogram lets
//      the rebuild find out, and the select scans the row if it does not), clears the histogram
//      and lets the others go, which wait for that in a bounded poll; then all of them
//   3. rebuild the candidate list with the new guess, a few chunks each.
// The wait needs the worker's workgroups resident together: the host launches at most 1024 of
// them in all (one per worker above that, which waits for nobody).  A workgroup that polls
// spin_limit times in vain (a device shared with work that never ends) marks the worker's list
// as not to be trusted and leaves; the select then scans the row, which needs no list.
// grid (blocks per worker, n), block 256.
template <int COMP>
__global__ __launch_bounds__(256) void k_sel_fallback(Args A) {
  __shared__ uint2 stage[kStageCap];
  __shared__ uint32_t s_count, s_base;
  __shared__ uint32_t part[256];
  __shared__ uint32_t s_grp, s_above, s_last, s_gen, s_go;
  const int i = blockIdx.y;
  WorkerCtl* ctl = A.ctl + i;
  if (list_is_good(ctl, A)) {
    if (blockIdx.x == 0 && threadIdx.x == 0) ctl->mode = 0;
    return;
  }
  uint32_t* hist = A.hist16 + (int64_t)i * kBins16;
  const int nvec = (A.d + 3) >> 2;
  const int t = threadIdx.x;
  {
    const int64_t nsample = ((int64_t)nvec + A.sample_stride - 1) / A.sample_stride;
    for (int64_t j = (int64_t)blockIdx.x * 256 + t; j < nsample; j += (int64_t)gridDim.x * 256) {
      const int m = (int)(j * (int64_t)A.sample_stride);
      uint32_t a[4];
      entry_bits<COMP, false, false, false>(A, i, m, a);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (4 * m + c >= A.e_lo && 4 * m + c < A.d) atomicAdd(&hist[Digits<COMP>::bin16(a[c])], 1u);
    }
  }
  __syncthreads();
  if (t == 0) {
    __threadfence();   // the workgroup's counts (complete at the barrier) before it counts itself in
    const uint32_t ticket = atomicAdd(&ctl->fb_arrive, 1u);
    s_last = (ticket % gridDim.x == gridDim.x - 1u) ? 1u : 0u;
    s_gen = ticket / gridDim.x + 1u;
  }
  __syncthreads();
  if (s_last) {
    __threadfence();
    // thread t owns the 256 buckets from 256 t
    static_assert(kBins16 == 256 * 256, "256 buckets per thread of a 256-thread workgroup");
    // (plain loads: the fence above has dropped what the caches held of the histogram, and the
    // others' counts were written back before they counted themselves in)
    const uint4* mine = reinterpret_cast<const uint4*>(hist + 256 * t);
    uint32_t sum = 0;
#pragma unroll 8
    for (int b = 0; b < 64; ++b) {
      const uint4 v = mine[b];
      sum += v.x + v.y + v.z + v.w;
    }
    part[t] = sum;
    __syncthreads();
    const uint64_t need = A.sample_need;
    if (t == 0) {
      uint32_t cum = 0;
      int g = 255;
      for (; g > 0; --g) {
        if ((uint64_t)cum + part[g] >= need) break;
        cum += part[g];
      }
      s_grp = (uint32_t)g;
      s_above = cum;
    }
    __syncthreads();
    // the buckets of that group, one per thread, then one thread walks them
    const uint32_t grp = s_grp;
    part[t] = hist[256u * grp + (uint32_t)t];
    __syncthreads();
    if (t == 0) {
      uint32_t cum = s_above, in_b = 0;
      int b = 255;
      for (; b >= 0; --b) {
        in_b = part[b];
        if (b == 0 || (uint64_t)cum + in_b >= need) break;
        cum += in_b;
      }
      const uint32_t bin = 256u * grp + (uint32_t)b;
      const uint64_t listed = (uint64_t)cum + (uint64_t)in_b;   // sampled entries with key32 >= floor(bin)
      ctl->guess_key = Digits<COMP>::bin16_floor(bin);
      ctl->bin_shift = COMP == Q_TOPK ? 9u : 10u;   // 64 candidate bins per 16-bit bucket
      const uint32_t mode = (A.sample_stride > 1u || listed <= (uint64_t)A.cand_cap) ? 1u : 2u;
      ctl->mode = mode;
      if (mode == 1u) {
        ctl->fallbacks += 1;
        for (int sg = 0; sg < kSegs; ++sg) ctl->seg_count[sg] = 0;
      }
    }
    if (t == 0) {
      __threadfence();
      __hip_atomic_store(&ctl->fb_go, s_gen, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int b = 0; b < 256; ++b) hist[256 * b + t] = 0;   // (nobody reads it again in this launch)
    __syncthreads();   // the mode that thread 0 has set is read by all below
  } else {
    if (t == 0) {
      uint32_t ok = 0;
      for (uint32_t it = 0; it < A.spin_limit; ++it) {
        const uint32_t go = __hip_atomic_load(&ctl->fb_go, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
        if ((int32_t)(go - s_gen) >= 0) {
          ok = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(64);
      }
      if (!ok) __hip_atomic_store(&ctl->fb_abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_go = ok;
    }
    __syncthreads();
    if (!s_go) return;
    __threadfence();
  }
  if (__hip_atomic_load(&ctl->mode, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 1u) return;
  const int nchunk = (nvec + 256 * kCompactVecs - 1) / (256 * kCompactVecs);
  for (int chunk = blockIdx.x; chunk < nchunk; chunk += gridDim.x) {
    __syncthreads();
    if (t == 0) s_count = 0;
    __syncthreads();
    compact_chunk<COMP, false, false, false, kCompactVecs>(A, i, chunk, stage, &s_count, &s_base);
  }
}

// ---------------------------------------------------------------------------
// The exact select on the candidates of one worker (device functions shared by the
// one-block and the multi-block kernels below).
// ---------------------------------------------------------------------------
// Lengths and prefix offsets of the candidate sub-lists of worker i, written to LDS (callers
// synchronise afterwards); *good: the list holds the k largest entries.
// By the first wave of a block (threads 0..63 call it): one sub-list per lane, prefix offsets by
// a wave scan - one round trip to memory instead of a thread's 32 loads in turn.
constexpr uint32_t kSpecPerSeg = 256;   // entries of a sub-list that k_sel_refine fetches before it knows the lengths

__device__ __forceinline__ void list_layout_wave(const Args& A, const WorkerCtl* ctl, uint32_t* lens, uint32_t* pre,
                                                 uint32_t* total_out, uint32_t* good_out,
                                                 uint32_t* short_out = nullptr) {
  const int lane = threadIdx.x & 63;
  const uint32_t raw = lane < kSegs ? ctl->seg_count[lane] : 0u;
  const uint32_t len = raw < A.seg_cap ? raw : A.seg_cap;
  uint32_t incl = len;
  unsigned long long rawsum = raw;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
    rawsum += __shfl_xor(rawsum, off, 64);
  }
  if (lane < kSegs) {
    lens[lane] = len;
    pre[lane] = incl - len;
  }
  if (lane == kSegs - 1) {
    pre[kSegs] = incl;
    *total_out = incl;
  }
  const bool fits = __ballot(raw > A.seg_cap) == 0ull;
  const bool all_short = __ballot(raw > kSpecPerSeg) == 0ull;
  if (lane == 0) {
    *good_out = (fits && rawsum >= (unsigned long long)A.k && ctl->fb_abort == 0u) ? 1u : 0u;
    if (short_out) *short_out = all_short ? 1u : 0u;
  }
}

// Entry at flat position f of the concatenated sub-lists (pre = prefix offsets in LDS).
__device__ __forceinline__ uint2 list_entry(const Args& A, int i, const uint32_t* pre, uint32_t f) {
  int lo = 0;   // sub-list holding f: largest s with pre[s] <= f
#pragma unroll
  for (int step = kSegs / 2; step >= 1; step >>= 1)
    if (pre[lo + step] <= f) lo += step;
  return A.cand[((int64_t)i * kSegs + lo) * A.seg_cap + (f - pre[lo])];
}

template <int COMP>
__device__ __forceinline__ void row_entry(const Args& A, int i, uint32_t t, uint32_t& a, uint32_t& idx) {
  idx = t;
  if (COMP == Q_TOPK) {
    const int64_t o = (int64_t)i * A.ld + t;
    a = __float_as_uint(A.X[o] - A.Xhat[o]);   // top_a never defers the local update
  } else {
    const uint4 wds = random_words(A, i, A.vec_base + (t >> 2), STREAM_RANDK);
    a = ~pick(wds, (int)(t & 3u));
  }
}

// Visit every entry of the domain (ROW: the whole row; else the concatenated candidate
// sub-lists, pre = their prefix offsets in LDS, total entries) with f(a, idx).  All threads
// of the block take part; list entries are fetched eight per thread at a time.
template <int COMP, bool ROW, class F>
__device__ __forceinline__ void for_each_entry(const Args& A, int i, const uint32_t* pre, uint32_t total, F f) {
  if (ROW) {
    for (uint32_t t = (uint32_t)A.e_lo + threadIdx.x; t < (uint32_t)A.d; t += blockDim.x) {
      uint32_t a, idx;
      row_entry<COMP>(A, i, t, a, idx);
      f(a, idx);
    }
  } else {
    for (uint32_t base = 0; base < total; base += blockDim.x * 8u) {
      uint2 c[8];
      bool have[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t p = base + (uint32_t)u * blockDim.x + threadIdx.x;
        have[u] = p < total;
        if (have[u]) c[u] = list_entry(A, i, pre, p);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (have[u]) f(c[u].x, c[u].y);
    }
  }
}

// Walk a histogram of 2048 bins in LDS from the top and find the digit at which
// the running count first reaches `need` (the last digit if it never does).  All
// threads of a block with >= 256 threads call it; grp is 256 words of LDS
// scratch.  Wave 0 does the search: lane l owns bins 32l..32l+31, a suffix scan
// over the lane totals finds the lane in which the count is reached, and that
// lane walks its 32 bins.
__device__ __forceinline__ void find_digit(const uint32_t* h, uint32_t* grp, uint32_t need,
                                           uint32_t* out_digit, uint32_t* out_above) {
  const int t = threadIdx.x;
  if (t < 256) {
    uint32_t g = 0;
#pragma unroll
    for (int b = 0; b < 8; ++b) g += h[8 * t + b];
    grp[t] = g;
  }
  __syncthreads();
  if (t < 64) {
    const uint32_t mine = grp[4 * t] + grp[4 * t + 1] + grp[4 * t + 2] + grp[4 * t + 3];
    // inclusive suffix sum over lanes: incl = sum of lane totals of lanes >= t
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t other = __shfl_down(incl, off, 64);
      if (t + off < 64) incl += other;
    }
    const uint32_t above_lane = incl - mine;          // entries in bins above this lane's range
    const bool here = above_lane < need && incl >= need;
    const uint64_t found = __ballot(here);
    if (found == 0) {                                 // fewer than `need` entries in total
      if (t == 0) { *out_digit = 0; *out_above = incl - h[0]; }
    } else if (here) {
      uint32_t cum = above_lane;
      int b = 32 * t + 31;
      for (; b > 32 * t; --b) {
        if (cum + h[b] >= need) break;
        cum += h[b];
      }
      *out_digit = (uint32_t)b;
      *out_above = cum;
    }
  }
  __syncthreads();
}

// Hand one kept entry to the message list of worker i (wave-aggregated slot).
// Every lane of the wave must call it (keep = false for lanes with nothing).
// Record that worker i kept entry idx: in the block's LDS bitmap when the row is short
// enough to have one (it is copied to global memory at the end), else as a bit of the
// kept-entry map in global memory (idx counts from the start of the piece the select works on).
__device__ __forceinline__ void mark_kept(const Args& A, int i, uint32_t idx, uint32_t* lbits) {
  // (lbits is null in the kernels that never see a row with an LDS bitmap)
  if (lbits != nullptr && A.bitmap_words) atomicOr(&lbits[idx >> 5], 1u << (idx & 31u));
  else atomicOr(&A.keptmap[(int64_t)i * A.map_words + ((idx + (uint32_t)A.idx_base) >> 5)], 1u << ((idx + (uint32_t)A.idx_base) & 31u));
}

// Did worker j keep entry e in this step?
__device__ __forceinline__ bool was_kept(const Args& A, int j, int e) {
  if (A.bitmap_words) return (A.bitmap[(int64_t)j * A.bitmap_words + ((uint32_t)e >> 5)] >> ((uint32_t)e & 31u)) & 1u;
  return (A.keptmap[(int64_t)j * A.map_words + ((uint32_t)e >> 5)] >> ((uint32_t)e & 31u)) & 1u;
}

// Copy the block's LDS bitmap of kept entries to global memory (rows short enough to have one).
__device__ __forceinline__ void publish_bitmap(const Args& A, int i, const uint32_t* lbits) {
  for (int64_t wd = threadIdx.x; wd < A.bitmap_words; wd += blockDim.x)
    A.bitmap[(int64_t)i * A.bitmap_words + wd] = lbits[wd];
}

// Bin of a candidate by its distance above the guess.
template <int COMP>
__device__ __forceinline__ uint32_t cand_bin(uint32_t a, uint32_t guess, uint32_t shift) {
  const uint32_t bin = (Digits<COMP>::key32(a) - guess) >> shift;
  return bin < (uint32_t)kBins ? bin : (uint32_t)kBins - 1u;
}

// Store one kept entry at a known slot of worker i's message list and mark it.
template <int COMP>
__device__ __forceinline__ void store_kept(const Args& A, int i, uint32_t slot, uint32_t a, uint32_t idx,
                                           uint32_t* lbits) {
  if (slot >= (uint32_t)A.k) return;
  // top_a carries the value in the entry; random_a gathers it afterwards (k_sel_values)
  A.sel_idx[(int64_t)i * A.sel_stride + slot] = A.idx_base + (int32_t)idx;
  if (COMP == Q_TOPK) A.sel_val[(int64_t)i * A.sel_stride + slot] = __uint_as_float(a);
  mark_kept(A, i, idx, lbits);
}

template <int COMP>
__device__ __forceinline__ void emit_entry(const Args& A, int i, bool keep, uint32_t a, uint32_t idx,
                                           uint32_t* s_emit, uint32_t* lbits) {
  const uint64_t mask = __ballot(keep);
  if (mask == 0) return;
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((unsigned long long)mask) - 1;
  uint32_t base = 0;
  if (lane == leader) base = atomicAdd(s_emit, (uint32_t)__popcll(mask));
  base = __shfl(base, leader, 64);
  if (keep) {
    const uint32_t slot = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
    store_kept<COMP>(A, i, slot, a, idx, lbits);
  }
}

// Place the guess (and the bin width) for the next step below this step's
// threshold key T: by the distance that, at the key density seen between the old
// guess and T, holds `want` entries (for top_a the k entries kept now leave the
// race, so want includes k).  Also resets the per-step counters.
__device__ __forceinline__ void next_guess(const Args& A, WorkerCtl* ctl, uint64_t kstar, uint32_t total,
                                           bool from_list, uint32_t emitted, uint32_t mode,
                                           bool have_floor = false, uint32_t floor_key = 0) {
  const uint32_t T = (uint32_t)(kstar >> 32);
  const uint32_t G = ctl->guess_key;
  uint64_t delta = A.delta0;
  if (from_list && total > (uint32_t)A.k && T > G)
    delta = (uint64_t)(T - G) * (uint64_t)A.want / (uint64_t)(total - (uint32_t)A.k);
  else if (have_floor && T > floor_key)
    delta = (uint64_t)(T - floor_key);   // row scan: the first-digit histogram located rank k + want
  if (delta < 1) delta = 1;
  if (delta > 0xFFFFFFFFull) delta = 0xFFFFFFFFull;
  ctl->guess_key = delta >= (uint64_t)T ? 0u : T - (uint32_t)delta;
  // 256-511 bins between the guess and where the threshold is expected: the 2048 bins then
  // still resolve a threshold that lands 4-8 times further above the guess than predicted
  const int lg = 63 - __clzll((unsigned long long)delta);
  ctl->bin_shift = lg > 8 ? (uint32_t)(lg - 8) : 0u;
  ctl->kstar = kstar;
  ctl->kept = emitted;
  ctl->last_candidates = total;
  ctl->mode = mode;
  ctl->emit_count = 0;
  ctl->small_count = 0;
  ctl->fb_abort = 0;
  if (mode == 2u) ctl->fallbacks += 1;
  for (int s = 0; s < kSegs; ++s) ctl->seg_count[s] = 0;
}

// Digit-by-digit radix select over the composite keys of the candidate list (ROW = false)
// or of the row itself (ROW = true: the list is not good); emits the kept entries, marks
// them and places the next guess.  All threads of a 1024-thread block.
template <int COMP, bool ROW>
__device__ void refine_and_emit(const Args& A, int i, const uint32_t* pre, uint32_t total, uint32_t* h,
                                uint32_t* grp, uint64_t* s_prefix, uint32_t* s_need, uint32_t* s_digit,
                                uint32_t* s_above, uint32_t* s_emit, uint32_t* lbits) {
  WorkerCtl* ctl = A.ctl + i;
  int last = 0;
  bool done = false;
  uint32_t floor_key = 0;
  for (int level = 0; level < 6 && !done; ++level) {
    for (int b = threadIdx.x; b < kBins; b += blockDim.x) h[b] = 0;
    __syncthreads();
    const uint64_t prefix = *s_prefix;
    const int scur = Digits<COMP>::shift(level);
    const int sprev = level > 0 ? Digits<COMP>::shift(level - 1) : 63;
    const uint32_t mask = (1u << Digits<COMP>::bits(level)) - 1u;
    for_each_entry<COMP, ROW>(A, i, pre, total, [&](uint32_t a, uint32_t idx) {
      const uint64_t K = Digits<COMP>::composite(a, idx);
      // level 0: every entry takes part (nothing of the composite lies above digit 0)
      const bool match = level == 0 ? true : ((K >> sprev) == prefix);
      if (match) atomicAdd(&h[(uint32_t)(K >> scur) & mask], 1u);
    });
    __syncthreads();
    if (ROW && level == 0) {
      // whole-row histogram of the first digit: also tells where rank k + want lies, which
      // becomes the floor of the next step's guess
      uint64_t target = (uint64_t)A.k + (uint64_t)A.want;
      if (target > (uint64_t)(A.d - A.e_lo)) target = (uint64_t)(A.d - A.e_lo);
      find_digit(h, grp, (uint32_t)target, s_digit, s_above);
      floor_key = (uint32_t)(((uint64_t)*s_digit << scur) >> 32);
      __syncthreads();
    }
    find_digit(h, grp, *s_need, s_digit, s_above);
    const uint32_t digit = *s_digit, above = *s_above;
    const uint32_t in_digit = h[digit];
    const uint32_t need = *s_need - above;
    __syncthreads();
    if (threadIdx.x == 0) {
      *s_prefix = (level == 0 ? 0ull : (prefix << Digits<COMP>::bits(level))) | (uint64_t)digit;
      *s_need = need;
    }
    last = level;
    done = (in_digit == need);
    __syncthreads();
  }
  const uint64_t kstar = *s_prefix << Digits<COMP>::shift(last);
  // emit every entry with composite >= kstar
  for_each_entry<COMP, ROW>(A, i, pre, total, [&](uint32_t a, uint32_t idx) {
    if (Digits<COMP>::composite(a, idx) >= kstar) {
      const uint32_t slot = atomicAdd(s_emit, 1u);
      if (slot < (uint32_t)A.k) {
        A.sel_idx[(int64_t)i * A.sel_stride + slot] = A.idx_base + (int32_t)idx;
        if (COMP == Q_TOPK) A.sel_val[(int64_t)i * A.sel_stride + slot] = __uint_as_float(a);
        mark_kept(A, i, idx, lbits);
      }
    }
  });
  __syncthreads();
  publish_bitmap(A, i, lbits);
  __syncthreads();
  if (threadIdx.x == 0) next_guess(A, ctl, kstar, total, !ROW, *s_emit, ROW ? 2u : 0u, ROW, floor_key);
}

// Exact selection from the candidates by one block per worker: emission of the kept
// (index, value) pairs and of the kept-entry map, next guess.  Fast path: an LDS
// histogram of the candidates by their distance above the guess tells which bin holds
// the k-th largest key; everything above that bin is emitted as it is and the few
// entries inside it are ranked against each other in LDS (lists of up to 8192 entries
// stay in registers between the two sweeps).  If that bin is crowded (ties) the
// digit-by-digit select runs on the list; if the list itself is not good, on the row.
// grid n, block 1024, dynamic LDS = the worker's bitmap (short rows) or nothing.
// BATCH: grid (n, long layers of A.long_tab).
template <int COMP, bool BATCH = false>
__global__ __launch_bounds__(1024) void k_sel_refine(Args A0) {
  const Args A = BATCH ? long_view(A0, A0.long_tab[blockIdx.y]) : A0;
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t grp[256];
  __shared__ uint32_t lens[kSegs];
  __shared__ uint32_t pre[kSegs + 1];
  __shared__ uint2 small[kSmallCap];
  __shared__ uint64_t s_prefix, s_kstar;
  __shared__ uint32_t s_need, s_digit, s_above, s_emit, s_total, s_good, s_small, s_short;
  extern __shared__ uint32_t lbits[];   // bitmap_words words: kept entries of this worker (short rows)
  const int i = blockIdx.x;
  WorkerCtl* ctl = A.ctl + i;
  // The first kSpecPerSeg entries of every sub-list are fetched before the lengths are known (32
  // threads per sub-list, eight entries each; what lies beyond a list's end is old data inside
  // the list's capacity and is masked below): one round trip to memory instead of two when no
  // sub-list is longer, which is the rule at the list lengths this kernel is launched for.
  // (Not for the long layers of a layer table: their lists are a few hundred entries, hundreds of
  // workgroups fetch at once, and the 64 KiB per workgroup cost more than the round trip saved:
  // 18.1 against 15.8 us.)
  constexpr bool SPECULATE = !BATCH;
  uint2 c[8];
  bool have[8];
  const int sseg = threadIdx.x >> 5, sj = threadIdx.x & 31;
  static_assert(kSegs * 32 == 1024 && kSpecPerSeg == 8 * 32, "32 threads per sub-list, eight entries each");
  if (SPECULATE) {
    const uint2* seg = A.cand + ((int64_t)i * kSegs + sseg) * A.seg_cap;
#pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = (uint32_t)(sj + 32 * u) < A.seg_cap ? seg[sj + 32 * u] : make_uint2(0u, 0u);
  }
  for (int b = threadIdx.x; b < kBins; b += 1024) h[b] = 0;
  for (int64_t wd = threadIdx.x; wd < A.bitmap_words; wd += 1024) lbits[wd] = 0;
  if (threadIdx.x == 0) {
    s_prefix = 0;
    s_need = (uint32_t)A.k;
    s_emit = 0;
    s_small = 0;
  }
  if (threadIdx.x < 64) list_layout_wave(A, ctl, lens, pre, &s_total, &s_good, &s_short);
  __syncthreads();
  const uint32_t total = s_total;
  if (!s_good) {
    refine_and_emit<COMP, true>(A, i, pre, total, h, grp, &s_prefix, &s_need, &s_digit, &s_above, &s_emit, lbits);
    return;
  }
  const uint32_t guess = ctl->guess_key, shift = ctl->bin_shift;
  auto entry_at = [&](uint32_t f) -> uint2 { return list_entry(A, i, pre, f); };
  auto bin_of = [&](uint32_t a) -> uint32_t { return cand_bin<COMP>(a, guess, shift); };
  // sweep 1: histogram of the candidates by their distance above the guess (eight
  // entries per thread in flight; a list of up to 8192 entries stays in registers)
  const bool fetched = SPECULATE && s_short != 0u;   // the entries fetched above are the whole list
  const bool resident = fetched || total <= 1024u * 8u;
  if (fetched) {
    const uint32_t len = lens[sseg];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      have[u] = (uint32_t)(sj + 32 * u) < len;
      if (have[u]) atomicAdd(&h[bin_of(c[u].x)], 1u);
    }
  } else {
    for (uint32_t base = 0; base < total; base += 1024u * 8u) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t f = base + (uint32_t)u * 1024u + threadIdx.x;
        have[u] = f < total;
        if (have[u]) c[u] = entry_at(f);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (have[u]) atomicAdd(&h[bin_of(c[u].x)], 1u);
    }
  }
  __syncthreads();
  find_digit(h, grp, (uint32_t)A.k, &s_digit, &s_above);
  const uint32_t tbin = s_digit;            // bin of the k-th largest key
  const uint32_t need_in_bin = (uint32_t)A.k - s_above;
  const uint32_t in_bin = h[tbin];
  if (in_bin > (uint32_t)kSmallCap) {
    __syncthreads();
    refine_and_emit<COMP, false>(A, i, pre, total, h, grp, &s_prefix, &s_need, &s_digit, &s_above, &s_emit, lbits);
    return;
  }
  // sweep 2: emit everything above the threshold bin, collect the bin itself
  if (resident) {
    // the list is in registers: a thread counts its entries above the bin, a scan over the wave
    // and one LDS atomic per wave give it its slots (instead of a ballot and an atomic per entry)
    uint32_t mine = 0;
    bool above[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      above[u] = false;
      if (have[u]) {
        const uint32_t bin = bin_of(c[u].x);
        above[u] = bin > tbin;
        if (bin == tbin) {
          const uint32_t pos = atomicAdd(&s_small, 1u);
          if (pos < (uint32_t)kSmallCap) small[pos] = c[u];
        }
      }
      mine += above[u] ? 1u : 0u;
    }
    const int lane = threadIdx.x & 63;
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    uint32_t wave_base = 0;
    if (lane == 63 && incl != 0u) wave_base = atomicAdd(&s_emit, incl);
    wave_base = __shfl(wave_base, 63, 64);
    uint32_t slot = wave_base + incl - mine;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (above[u]) store_kept<COMP>(A, i, slot++, c[u].x, c[u].y, lbits);
  } else
  for (uint32_t base = 0; base < total; base += 1024u * 8u) {
    if (!resident) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint32_t f = base + (uint32_t)u * 1024u + threadIdx.x;
        have[u] = f < total;
        if (have[u]) c[u] = entry_at(f);
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      bool above = false;
      if (have[u]) {
        const uint32_t bin = bin_of(c[u].x);
        above = bin > tbin;
        if (bin == tbin) {
          const uint32_t pos = atomicAdd(&s_small, 1u);
          if (pos < (uint32_t)kSmallCap) small[pos] = c[u];
        }
      }
      emit_entry<COMP>(A, i, above, c[u].x, c[u].y, &s_emit, lbits);
    }
  }
  __syncthreads();
  // rank the entries of the threshold bin against each other; the need_in_bin largest are kept
  const uint32_t m = s_small < (uint32_t)kSmallCap ? s_small : (uint32_t)kSmallCap;
  {
    bool keep = false;
    uint2 mine = make_uint2(0, 0);
    if (threadIdx.x < m) {
      mine = small[threadIdx.x];
      const uint64_t K = Digits<COMP>::composite(mine.x, mine.y);
      uint32_t rank = 0;
      for (uint32_t u = 0; u < m; ++u) {
        const uint2 o = small[u];
        rank += Digits<COMP>::composite(o.x, o.y) > K ? 1u : 0u;
      }
      keep = rank < need_in_bin;
      if (rank + 1u == need_in_bin) s_kstar = K;
    }
    emit_entry<COMP>(A, i, keep, mine.x, mine.y, &s_emit, lbits);
  }
  __syncthreads();
  publish_bitmap(A, i, lbits);
  if (threadIdx.x == 0) next_guess(A, ctl, s_kstar, total, true, s_emit, 0u);
}

// ---------------------------------------------------------------------------
// Multi-block select for long candidate lists (k + want > 16384 per worker): the
// one-block-per-worker kernel above would leave all but n CUs idle.  Three launches:
//   k_sel_hist_parts  kRefineParts blocks per worker histogram a slice of the list each
//   k_sel_emit_parts  every block sums the partial histograms, finds the threshold bin,
//                     emits the entries of its slice above that bin (one global atomic per
//                     block) and hands the entries inside the bin to a short global list
//   k_sel_finish      one block per worker ranks that short list, emits the rest, places
//                     the next guess; also takes the digit-by-digit and row-scan paths when
//                     the threshold bin is crowded or the list is not good
// grid (kRefineParts, n) for the first two, n for the last; block 1024.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void part_slice(uint32_t total, uint32_t part, uint32_t* lo, uint32_t* hi) {
  const uint32_t per = (total + (uint32_t)kRefineParts - 1u) / (uint32_t)kRefineParts;
  *lo = part * per < total ? part * per : total;
  *hi = (part + 1u) * per < total ? (part + 1u) * per : total;
}

template <int COMP>
__global__ __launch_bounds__(1024) void k_sel_hist_parts(Args A) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t lens[kSegs];
  __shared__ uint32_t pre[kSegs + 1];
  __shared__ uint32_t s_total, s_good;
  const int i = blockIdx.y;
  const WorkerCtl* ctl = A.ctl + i;
  for (int b = threadIdx.x; b < kBins; b += 1024) h[b] = 0;
  if (threadIdx.x < 64) list_layout_wave(A, ctl, lens, pre, &s_total, &s_good);
  __syncthreads();
  if (!s_good) return;
  uint32_t lo, hi;
  part_slice(s_total, blockIdx.x, &lo, &hi);
  const uint32_t guess = ctl->guess_key, shift = ctl->bin_shift;
  for (uint32_t base = lo; base < hi; base += 1024u * 8u) {
    uint2 c[8];
    bool have[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t f = base + (uint32_t)u * 1024u + threadIdx.x;
      have[u] = f < hi;
      if (have[u]) c[u] = list_entry(A, i, pre, f);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (have[u]) atomicAdd(&h[cand_bin<COMP>(c[u].x, guess, shift)], 1u);
  }
  __syncthreads();
  uint32_t* out = A.hist_parts + ((int64_t)i * kRefineParts + blockIdx.x) * kBins;
  for (int b = threadIdx.x; b < kBins; b += 1024) out[b] = h[b];
}

// Sum of the partial histograms of worker i into LDS (all threads; caller synchronises).
__device__ __forceinline__ void sum_hist_parts(const Args& A, int i, uint32_t* h) {
  for (int b = threadIdx.x; b < kBins; b += blockDim.x) {
    uint32_t acc = 0;
#pragma unroll
    for (int p = 0; p < kRefineParts; ++p) acc += A.hist_parts[((int64_t)i * kRefineParts + p) * kBins + b];
    h[b] = acc;
  }
}

template <int COMP>
__global__ __launch_bounds__(1024) void k_sel_emit_parts(Args A) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t grp[256];
  __shared__ uint32_t lens[kSegs];
  __shared__ uint32_t pre[kSegs + 1];
  __shared__ uint32_t s_total, s_good, s_digit, s_above, s_count, s_base;
  const int i = blockIdx.y;
  WorkerCtl* ctl = A.ctl + i;
  if (threadIdx.x < 64) list_layout_wave(A, ctl, lens, pre, &s_total, &s_good);
  __syncthreads();
  if (!s_good) return;
  sum_hist_parts(A, i, h);
  __syncthreads();
  find_digit(h, grp, (uint32_t)A.k, &s_digit, &s_above);
  const uint32_t tbin = s_digit;
  if (h[tbin] > (uint32_t)kSmallCap) return;   // crowded threshold bin: k_sel_finish selects digit by digit
  uint32_t lo, hi;
  part_slice(s_total, blockIdx.x, &lo, &hi);
  const uint32_t guess = ctl->guess_key, shift = ctl->bin_shift;
  const int lane = threadIdx.x & 63;
  for (uint32_t base = lo; base < hi; base += 1024u * 8u) {
    __syncthreads();
    if (threadIdx.x == 0) s_count = 0;
    __syncthreads();
    uint2 c[8];
    bool have[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t f = base + (uint32_t)u * 1024u + threadIdx.x;
      have[u] = f < hi;
      if (have[u]) c[u] = list_entry(A, i, pre, f);
    }
    // which of my entries lie above the threshold bin; the bin's own entries go to the short list
    uint64_t masks[8];
    uint32_t wave_total = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      bool above = false;
      if (have[u]) {
        const uint32_t bin = cand_bin<COMP>(c[u].x, guess, shift);
        above = bin > tbin;
        if (bin == tbin) {
          const uint32_t pos = atomicAdd(&ctl->small_count, 1u);
          if (pos < (uint32_t)kSmallCap) A.small_list[(int64_t)i * kSmallCap + pos] = c[u];
        }
      }
      masks[u] = __ballot(above);
      wave_total += (uint32_t)__popcll(masks[u]);
    }
    // slots: wave offset inside the block through LDS, block offset through one global atomic
    uint32_t wave_base = 0;
    if (lane == 0 && wave_total) wave_base = atomicAdd(&s_count, wave_total);
    wave_base = __shfl(wave_base, 0, 64);
    __syncthreads();
    if (threadIdx.x == 0 && s_count) s_base = atomicAdd(&ctl->emit_count, s_count);
    __syncthreads();
    uint32_t running = s_base + wave_base;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if ((masks[u] >> lane) & 1ull) {
        const uint32_t slot = running + (uint32_t)__popcll(masks[u] & ((1ull << lane) - 1ull));
        store_kept<COMP>(A, i, slot, c[u].x, c[u].y, nullptr);
      }
      running += (uint32_t)__popcll(masks[u]);
    }
  }
}

template <int COMP>
__global__ __launch_bounds__(1024) void k_sel_finish(Args A) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t grp[256];
  __shared__ uint32_t lens[kSegs];
  __shared__ uint32_t pre[kSegs + 1];
  __shared__ uint2 small[kSmallCap];
  __shared__ uint64_t s_prefix, s_kstar;
  __shared__ uint32_t s_need, s_digit, s_above, s_emit, s_total, s_good;
  const int i = blockIdx.x;
  WorkerCtl* ctl = A.ctl + i;
  if (threadIdx.x == 0) {
    s_prefix = 0;
    s_need = (uint32_t)A.k;
    s_emit = 0;
  }
  if (threadIdx.x < 64) list_layout_wave(A, ctl, lens, pre, &s_total, &s_good);
  __syncthreads();
  const uint32_t total = s_total;
  if (!s_good) {
    refine_and_emit<COMP, true>(A, i, pre, total, h, grp, &s_prefix, &s_need, &s_digit, &s_above, &s_emit, nullptr);
    return;
  }
  sum_hist_parts(A, i, h);
  __syncthreads();
  find_digit(h, grp, (uint32_t)A.k, &s_digit, &s_above);
  const uint32_t tbin = s_digit, above = s_above;
  const uint32_t need_in_bin = (uint32_t)A.k - above;
  const uint32_t in_bin = h[tbin];
  if (in_bin > (uint32_t)kSmallCap) {
    __syncthreads();
    refine_and_emit<COMP, false>(A, i, pre, total, h, grp, &s_prefix, &s_need, &s_digit, &s_above, &s_emit, nullptr);
    return;
  }
  // the blocks of k_sel_emit_parts emitted `above` entries into slots 0..above-1 and collected
  // the in_bin entries of the threshold bin; rank those and emit the need_in_bin largest
  const uint32_t m = in_bin;
  for (uint32_t t = threadIdx.x; t < m; t += 1024) small[t] = A.small_list[(int64_t)i * kSmallCap + t];
  __syncthreads();
  if (threadIdx.x < m) {
    const uint2 mine = small[threadIdx.x];
    const uint64_t K = Digits<COMP>::composite(mine.x, mine.y);
    uint32_t rank = 0;
    for (uint32_t u = 0; u < m; ++u) {
      const uint2 o = small[u];
      rank += Digits<COMP>::composite(o.x, o.y) > K ? 1u : 0u;
    }
    if (rank < need_in_bin) store_kept<COMP>(A, i, above + rank, mine.x, mine.y, nullptr);
    if (rank + 1u == need_in_bin) s_kstar = K;
  }
  __syncthreads();
  if (threadIdx.x == 0) next_guess(A, ctl, s_kstar, total, true, above + need_in_bin, 0u);
}

// random_a with the fused update-and-mix pass: the kept values were left at their entries of Qv;
// collect them into the list (on request only: read-back and message encoding, not a step).
// grid (ceil(k/256), n)
__global__ __launch_bounds__(256) void k_gather_values(Args A) {
  const int j = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  const int e = A.sel_idx[(int64_t)j * A.k + m];
  A.sel_val[(int64_t)j * A.k + m] = A.Qv[(int64_t)j * A.ld + e];
}

// q_j[e] = x_j[e] - xhat_j[e] (rescaled on request) as the message kernels recompute it.
__device__ __forceinline__ float fresh_value(const Args& A, int j, int e) {
  const int64_t o = (int64_t)j * A.ld + e;
  float q = x_entry(A, o) - A.Xhat[o];
  if (A.randk_rescale) q = randk_scale_at(A, e) * q;
  return q;
}

// random_a with incremental neighbour sums: the kept values are gathered once the indices are
// known (top_a carries the value in the candidate entry instead).  A launch of its own: n k
// gathers spread over all CUs; inside the scatter, where every one of the nnz k threads would
// gather its own value, they cost more than this launch (n = 64 ring, 65 layers: scatter 47
// against 21 + 12.5 us).  grid (ceil(k/256), n)
__global__ __launch_bounds__(256) void k_sel_values(Args A) {
  const int j = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  A.sel_val[(int64_t)j * A.k + m] = fresh_value(A, j, A.sel_idx[(int64_t)j * A.k + m]);
}

// S_i[e] += sum_p w_p q_j[e] over the neighbours j = col[p] that kept entry e,
// in CSR order (the incremental neighbour sums).  One thread per (i, p, kept
// entry m of j); the thread of the FIRST neighbour in row i that kept e owns
// the whole chain for (i, e), so each S entry has one writer and the order of
// the additions is fixed.  Must run before xhat is updated (values of other
// neighbours are recomputed as x - xhat).  grid (ceil(k/256), maxdeg, n)
__global__ __launch_bounds__(256) void k_scatter_s(Args A) {
  const int i = blockIdx.z;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int pbeg = A.row_ptr[i], pend = A.row_ptr[i + 1];
  const int p = pbeg + (int)blockIdx.y;
  if (m >= A.k || p >= pend) return;
  const int j = A.col[p];
  const int e = A.sel_idx[(int64_t)j * A.k + m];
  for (int p2 = pbeg; p2 < p; ++p2)
    if (was_kept(A, A.col[p2], e)) return;
  float* s = A.S + (int64_t)i * A.ld + e;
  float acc = *s;
  acc = acc + A.w[p] * A.sel_val[(int64_t)j * A.k + m];
  for (int p2 = p + 1; p2 < pend; ++p2) {
    const int j2 = A.col[p2];
    if (was_kept(A, j2, e)) acc = acc + A.w[p2] * fresh_value(A, j2, e);
  }
  *s = acc;
}

// p[0 .. words) = 0.  grid (ceil(words / 256))
__global__ __launch_bounds__(256) void k_zero_words(uint32_t* p, int64_t words) {
  const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (o < words) p[o] = 0u;
}

// xhat_j[e] += q_j[e] for the kept entries (Algorithm 1, update of the public copies); clears the
// words of the bit map it used.  With update_values (random_a where no scatter ran) it forms q
// itself and leaves it in the list.  grid (ceil(k/256), n)
__global__ __launch_bounds__(256) void k_xhat_update(Args A) {
  const int j = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  const int e = A.sel_idx[(int64_t)j * A.k + m];
  float* xh = A.Xhat + (int64_t)j * A.ld + e;
  float q;
  if (A.update_values) {
    q = fresh_value(A, j, e);
    A.sel_val[(int64_t)j * A.k + m] = q;
  } else {
    q = A.sel_val[(int64_t)j * A.k + m];
  }
  *xh = *xh + q;
  // (the bitmap is rewritten whole every step; the words of the bit map are cleared by whoever kept an entry in them)
  if (!A.bitmap_words) A.keptmap[(int64_t)j * A.map_words + ((uint32_t)e >> 5)] = 0u;
}

// ---------------------------------------------------------------------------
// Metrics (not on the timed path): per-block partial sums in fp64, then a
// single-block sum in block order, so the result is repeatable.
//   out[0] = sum_i ||x_i - xbar||^2, out[1] = ||xbar||^2, out[2] = ||X - Xhat||_F^2
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_metrics_partial(Args A, double* part) {
  __shared__ double sh[3][256];
  double dev = 0.0, mn = 0.0, gap = 0.0;
  for (int e = blockIdx.x * 256 + threadIdx.x; e < A.d; e += gridDim.x * 256) {
    double mean = 0.0;
    for (int i = 0; i < A.n; ++i) mean += (double)A.X[(int64_t)i * A.ld + e];
    mean /= (double)A.n;
    mn += mean * mean;
    for (int i = 0; i < A.n; ++i) {
      const double x = (double)A.X[(int64_t)i * A.ld + e];
      const double a = x - mean;
      const double b = x - (double)A.Xhat[(int64_t)i * A.ld + e];
      dev += a * a;
      gap += b * b;
    }
  }
  sh[0][threadIdx.x] = dev; sh[1][threadIdx.x] = mn; sh[2][threadIdx.x] = gap;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off)
      for (int q = 0; q < 3; ++q) sh[q][threadIdx.x] += sh[q][threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0)
    for (int q = 0; q < 3; ++q) part[3 * blockIdx.x + q] = sh[q][0];
}

__global__ void k_metrics_final(const double* part, int nblocks, double* out) {
  if (threadIdx.x < 3) {
    double acc = 0.0;
    for (int b = 0; b < nblocks; ++b) acc += part[3 * b + threadIdx.x];
    out[threadIdx.x] = acc;
  }
}

// The same last step with the three figures finished on the device (no host arithmetic):
//   out[0] = consensus distance (1/n) sum_i ||x_i - xbar||^2, out[1] = ||xbar||_2,
//   out[2] = Psi = ||X - Xbar||_F^2 + ||X - Xhat||_F^2
__global__ void k_metrics_final_dev(const double* part, int nblocks, int n, double* out) {
  __shared__ double sums[3];
  if (threadIdx.x < 3) {
    double acc = 0.0;
    for (int b = 0; b < nblocks; ++b) acc += part[3 * b + threadIdx.x];
    sums[threadIdx.x] = acc;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    out[0] = sums[0] / (double)n;
    out[1] = sqrt(sums[1]);
    out[2] = sums[0] + sums[2];
  }
}

}  // namespace choco
