// Layer-wise compression (Section 5, set-up of the deep-learning runs: the operator is
// applied to every layer of the network on its own).
//
// sign / gsgd_b: the whole-row pipeline with per-layer norms.  k_layer_stat streams the rows
// once (one block per group of up to 16 chunks of ONE layer: the norm tree of a layer
// starts at the layer's first entry), k_layer_finalise sums each layer's group sums and
// turns them into the layer's scales, and the apply kernels of the whole-row path look the
// scale of each 4-vector up by its layer.  Any layer length.
//
// top_a / random_a: k_layer_compress, for layers of up to kMidLayerLen = 10,240 entries (longer
// ones stream through the guessed-threshold select of the whole-row path, all of them in one
// launch of its pass over the rows and one of its exact select).  A layer of a worker is
// selected by one 1024-thread workgroup (above 3,072 entries), one 256-thread workgroup (above
// 768) or one wave (smaller layers, four to a workgroup), with the layer's x - xhat (or its
// random words) in registers: at most kLayerVecs = 3 4-vectors per thread, all loaded at once -
// a thread's entries are worked through one after the other, so the time of a layer goes with
// their number (with 10 per thread the 0.27 M model's layers of 2,304 to 9,216 entries took 35 us,
// whatever the sweeps cost).
// The exact k-th largest key: a bracket [lo, hi) around a guess (last step's threshold for
// top_a, the expected order statistic for random_a) is counted in one sweep over the
// registers; if the k-th key provably lies inside, only the few keys in the bracket are
// searched (bit by bit, in LDS); otherwise the whole layer is searched bit by bit (31 or 32
// sweeps with block-wide counts).  Ties on the threshold key go to the lower index.  List
// positions and kept-entry slots are handed out per wave from a ballot (a wave that has a
// layer to itself counts in a register); no histogram, no global counters.
#pragma once

#include "choco_kernels.h"

namespace choco {

constexpr int kLayerVecs = 3;
constexpr int kWaveLayerLen = 64 * kLayerVecs * 4;     // up to here a single wave takes the layer
constexpr int kSmallLayerLen = 256 * kLayerVecs * 4;   // up to here a 256-thread workgroup does
constexpr int kMidLayerLen = 10240;                    // ... and up to here a 1024-thread one
static_assert(kMidLayerLen <= 1024 * kLayerVecs * 4, "a 1024-thread workgroup holds a layer of this class");

// Block total of per-wave counts (each already uniform over its wave).
template <int THREADS>
__device__ __forceinline__ uint32_t block_total(uint32_t wave_count, uint32_t* sh, int& phase) {
  if (THREADS == 64) return wave_count;
  // two buffers in turn: a wave may write round j+1 while another still reads round j
  uint32_t* buf = sh + 16 * phase;
  phase ^= 1;
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = wave_count;
  __syncthreads();
  uint32_t tot = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) tot += buf[w];
  return tot;
}

// lanes of the wave for which pred holds (a compare and a scalar bit count, no cross-lane traffic)
__device__ __forceinline__ uint32_t wave_count(bool pred) { return (uint32_t)__popcll(__ballot(pred)); }

// Sum of a small per-lane count over the wave (the same in every lane afterwards).
__device__ __forceinline__ uint32_t wave_count_sum(uint32_t v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Lanes below this one whose bit is set in a ballot mask.
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Positions for the lanes of `mask` (not empty, the same in every lane) in a list shared by
// the THREADS threads of a layer: one wave counts in a register, several waves take a range
// each with one LDS atomic by the wave's first such lane.
template <int THREADS>
__device__ __forceinline__ uint32_t claim(uint64_t mask, uint32_t& running, uint32_t* shared_count) {
  const uint32_t cnt = (uint32_t)__popcll(mask);
  uint32_t base;
  if (THREADS == 64) {
    base = running;
    running += cnt;
  } else {
    const int leader = __ffsll((unsigned long long)mask) - 1;
    uint32_t got = 0;
    if ((int)(threadIdx.x & 63) == leader) got = atomicAdd(shared_count, cnt);
    base = (uint32_t)__builtin_amdgcn_readlane((int)got, leader);
  }
  return base + lanes_below(mask);
}

// Barrier among the THREADS threads that share a layer (one wave needs none: its LDS
// accesses execute in order; the fence only stops the compiler from reordering them).
template <int THREADS>
__device__ __forceinline__ void layer_sync() {
  if (THREADS == 64) __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  else __syncthreads();
}

// The LDS of the THREADS threads that share a layer.
struct LayerShared {
  uint32_t* cnt;      // 2 x 16 per-wave counts, then two words for a result one wave hands to the others
  uint32_t* emit;     // kept entries emitted so far
  uint32_t* list_n;   // keys in the bracket
  uint2* list;        // (key, index in the layer) of the keys in the bracket
};

template <int COMP, int THREADS, bool NT>
__device__ __forceinline__ void layer_body(const Args& A, const int i, const LayerDesc L, const int tid,
                                           const LayerShared sh) {
  static_assert(COMP == Q_TOPK || COMP == Q_RANDK, "sign and gsgd layers go through k_layer_stat");
  constexpr int NW = THREADS / 64;
  constexpr int kBatch = kLayerVecs;   // 4-vectors per thread whose loads are in flight together
  constexpr int kBatches = (kLayerVecs + kBatch - 1) / kBatch;
  constexpr uint32_t CAP = 2 * THREADS;
  // local index e counts from the 4-vector boundary at or below the layer's first entry: the
  // layer's entries are head <= e < end (head = 0 unless the table is generic)
  const int head = L.head, end = L.head + L.len, base = L.start - L.head;
  auto inside = [&](int e) { return e >= head && e < end; };
  const int nvec = (end + 3) >> 2;
  const int nit = (nvec + THREADS - 1) / THREADS;   // sweeps of the threads over the layer (<= kLayerVecs)
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t row = (int64_t)i * A.ld + base;
  double* scal = A.layer_scal + ((int64_t)i * A.nlayers + L.id) * 4;
  float* __restrict__ X = A.X;
  float* __restrict__ Xhat = A.Xhat;
  const float* __restrict__ G = A.G;
  float* __restrict__ Mom = A.M;
  if (tid == 0) {
    *sh.emit = 0;
    *sh.list_n = 0;
  }
  layer_sync<THREADS>();   // no wave may count into the list before it is reset (waves start in any order)

  // ---- load: v = x - xhat (after the local update, if this pass carries it) ----
  vf4 v[kLayerVecs];
  uint32_t word_key[COMP == Q_RANDK ? kLayerVecs : 1][4];
  if constexpr (COMP == Q_RANDK) {
#pragma unroll
    for (int it = 0; it < kLayerVecs; ++it) {
      const int m = it * THREADS + tid;
      // keys are ~word: the k smallest words are the k largest keys
      uint4 wd = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
      if (it < nit && m < nvec) wd = random_words(A, i, (uint32_t)(base >> 2) + (uint32_t)m, STREAM_RANDK);
#pragma unroll
      for (int c = 0; c < 4; ++c) word_key[it][c] = inside(4 * m + c) ? ~pick(wd, c) : 0u;
    }
  } else {
#pragma unroll
    for (int b = 0; b < kBatches; ++b) {
      vf4 x[kBatch], g[kBatch], h[kBatch];
      if (b * kBatch < nit) {                    // uniform over the threads of the layer
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
          const int m = (b * kBatch + j) * THREADS + tid;
          if (b * kBatch + j < kLayerVecs && m < nvec) {
            const int64_t o = row + 4 * (int64_t)m;
            x[j] = load4<NT>(X + o);
            h[j] = load4<NT>(Xhat + o);
            if (G) g[j] = load4<true>(G + o);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int it = b * kBatch + j;
        if (it >= kLayerVecs) continue;
        const int m = it * THREADS + tid;
        v[it] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
        if (it < nit && m < nvec) {
          const int64_t o = row + 4 * (int64_t)m;
          if (G) {
            vf4 mom = vf4{0.0f, 0.0f, 0.0f, 0.0f};
            if (Mom) mom = load4<NT>(Mom + o);
            x[j] = local_update_regs(A, x[j], g[j], mom);
            if (Mom) store4<NT>(Mom + o, mom);
            store4<NT>(X + o, x[j]);
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) v[it][c] = inside(4 * m + c) ? x[j][c] - h[j][c] : 0.0f;
        }
      }
    }
  }

  {
    // ---- top_a / random_a: exact k-th largest key ----
    const uint32_t k = (uint32_t)L.k;
    if (k == 0) {
      if (tid == 0) scal[0] = scal[1] = scal[2] = scal[3] = 0.0;
      return;
    }
    auto key_of = [&](int it, int c) -> uint32_t {
      if constexpr (COMP == Q_RANDK) return word_key[it][c];
      else return __float_as_uint(v[it][c]) & 0x7FFFFFFFu;
    };
    constexpr int TOPBIT = COMP == Q_RANDK ? 31 : 30;
    uint32_t* guess = A.layer_guess + (int64_t)i * A.nlayers + L.id;
    // a bracket that should hold the k-th largest key
    bool have = true;
    uint32_t lo, hi;
    if (COMP == Q_RANDK) {
      // keys are uniform on [0, 2^32): the k-th largest of len sits near (1 - k/len) 2^32,
      // give or take sqrt(k)/len 2^32; the half-width is counted in expected entries
      const double hw = fmin(6.0 * sqrt((double)k) + 8.0, 0.4 * (double)CAP);
      const double centre = (1.0 - (double)k / (double)L.len) * 4294967296.0;
      const double width = hw / (double)L.len * 4294967296.0;
      lo = (uint32_t)fmax(centre - width, 0.0);
      hi = (uint32_t)fmin(centre + width, 4294967295.0);
    } else {
      const uint32_t g = *guess;             // last step's threshold of this layer
      have = g != 0xFFFFFFFFu;
      // +-6 % in magnitude around it, narrower when k is large for the list
      uint32_t delta = 1u << 19;
      if (5u * k > 3u * CAP) delta = (uint32_t)(((uint64_t)delta * 3u * CAP) / (5ull * k));
      if (delta < 256u) delta = 256u;
      lo = g > delta ? g - delta : 0u;
      hi = g < 0x7FFFFFFFu - delta ? g + delta : 0x7FFFFFFFu;
    }
    int phase = 0;
    uint32_t T = 0, at_or_above = 0xFFFFFFFFu;
    uint32_t listed_n = 0;   // one wave per layer: the length of its list
    bool found = false;
    if (have) {                                   // uniform
      uint32_t nhi = 0, listed = 0;
#pragma unroll
      for (int it = 0; it < kLayerVecs; ++it)
        if (it < nit) {
          const int m = it * THREADS + tid;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t key = key_of(it, c);
            nhi += wave_count(key >= hi);
            const bool in = key >= lo && key < hi && inside(4 * m + c);
            const uint64_t hits = __ballot(in);
            if (hits != 0) {                      // uniform over the wave
              const uint32_t pos = claim<THREADS>(hits, listed, sh.list_n);
              if (in && pos < CAP) sh.list[pos] = make_uint2(key, (uint32_t)(4 * m + c));
            }
          }
        }
      nhi = block_total<THREADS>(nhi, sh.cnt, phase);
      layer_sync<THREADS>();
      const uint32_t nin = THREADS == 64 ? listed : *sh.list_n;
      listed_n = listed;
      if (nhi < k && k - nhi <= nin && nin <= CAP) {
        // the k-th largest key is the r-th largest of the list: bit by bit on key - lo
        found = true;
        const uint32_t r = k - nhi;
        const uint32_t span = hi - lo;            // >= 1: the list is not empty
        uint32_t Trel = 0, got = nin;
        constexpr uint32_t SOLO = 512;     // list lengths that one wave searches on its own
        if (THREADS > 64 && nin <= SOLO) {
          // several waves: the first one searches the list on its own, eight keys per lane, and
          // the others wait once (a block-wide count per bit costs a barrier per bit)
          if (wave == 0) {
            uint32_t rel[SOLO / 64];
#pragma unroll
            for (int j = 0; j < (int)(SOLO / 64); ++j) {
              const uint32_t p = (uint32_t)(lane + 64 * j);
              // (keys of the list lie at or above lo; a slot past the list counts for no candidate >= 1)
              rel[j] = p < nin ? sh.list[p].x - lo + 1u : 0u;
            }
            for (int bit = 31 - __clz((int)(span | 1u)); bit >= 0 && got != r; --bit) {
              const uint32_t cand = Trel | (1u << bit);
              uint32_t cnt = 0;
#pragma unroll
              for (int j = 0; j < (int)(SOLO / 64); ++j) cnt += wave_count(rel[j] > cand);
              if (cnt >= r) {
                Trel = cand;
                got = cnt;
              }
            }
            if (lane == 0) {
              sh.cnt[32] = Trel;
              sh.cnt[33] = got;
            }
          }
          __syncthreads();
          Trel = sh.cnt[32];
          got = sh.cnt[33];
        } else {
          const uint32_t rel0 = (uint32_t)tid < nin ? sh.list[tid].x - lo : 0u;
          const uint32_t rel1 = (uint32_t)tid + THREADS < nin ? sh.list[tid + THREADS].x - lo : 0u;
          const bool has0 = (uint32_t)tid < nin, has1 = (uint32_t)tid + THREADS < nin;
          for (int bit = 31 - __clz((int)(span | 1u)); bit >= 0 && got != r; --bit) {
            const uint32_t cand = Trel | (1u << bit);
            uint32_t cnt = wave_count(has0 && rel0 >= cand) + wave_count(has1 && rel1 >= cand);
            cnt = block_total<THREADS>(cnt, sh.cnt, phase);
            if (cnt >= r) {
              Trel = cand;
              got = cnt;
            }
          }
        }
        T = lo + Trel;
        at_or_above = nhi + got;
      }
    }
    if (!found) {
      // the whole layer, bit by bit: the largest T with count(key >= T) >= k; it may stop
      // as soon as exactly k keys lie at or above T (the lower bits cannot matter)
      for (int bit = TOPBIT; bit >= 0 && at_or_above != k; --bit) {
        const uint32_t cand = T | (1u << bit);
        uint32_t cnt = 0;
#pragma unroll
        for (int it = 0; it < kLayerVecs; ++it)
          if (it < nit) {
#pragma unroll
            for (int c = 0; c < 4; ++c) cnt += wave_count(key_of(it, c) >= cand);
          }
        cnt = block_total<THREADS>(cnt, sh.cnt, phase);
        if (cnt >= k) {
          T = cand;
          at_or_above = cnt;
        }
      }
    }
    if (COMP == Q_TOPK && tid == 0) *guess = T;
    // entries above the threshold key are all kept; of those equal to it, the first `need`
    // by index (entries outside the layer carry key 0 and are told apart by their index)
    uint32_t above = 0, equals = 0;
    if (found) {
      // the threshold lies in the bracket, so every entry that holds it is in the list
      const uint32_t nin = THREADS == 64 ? listed_n : *sh.list_n;
      for (uint32_t p = (uint32_t)tid; p < nin; p += THREADS) equals += sh.list[p].x == T ? 1u : 0u;
      equals = wave_count_sum(equals);
      equals = block_total<THREADS>(equals, sh.cnt, phase);
      above = at_or_above - equals;
    } else {
#pragma unroll
      for (int it = 0; it < kLayerVecs; ++it)
        if (it < nit) {
          const int m = it * THREADS + tid;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t key = key_of(it, c);
            above += wave_count(key > T);
            equals += wave_count(key == T && inside(4 * m + c));
          }
        }
      above = block_total<THREADS>(above, sh.cnt, phase);
      equals = block_total<THREADS>(equals, sh.cnt, phase);
    }
    const uint32_t need = k - above;
    if (tid == 0) {
      scal[0] = (double)T;
      scal[1] = (double)need;
      scal[2] = (double)equals;
      scal[3] = found ? 1.0 : 0.0;
    }
    const bool ties = equals > need;   // uniform over the layer's threads
    uint32_t running = 0;              // threshold-key entries in earlier sweeps (index order)
    uint32_t emitted = 0;              // one wave per layer: kept entries handed out so far
#pragma unroll
    for (int it = 0; it < kLayerVecs; ++it) {
      if (it < nit) {
        const int m = it * THREADS + tid;
        uint32_t rank = 0;
        if (ties) {
          uint32_t mine = 0;
#pragma unroll
          for (int c = 0; c < 4; ++c) mine += (key_of(it, c) == T && inside(4 * m + c)) ? 1u : 0u;
          uint32_t incl = mine;
#pragma unroll
          for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
          }
          uint32_t base = 0, total = __shfl(incl, 63, 64);
          if (THREADS > 64) {
            uint32_t* buf = sh.cnt + 16 * phase;
            phase ^= 1;
            if (lane == 63) buf[wave] = incl;
            __syncthreads();
            total = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
              const uint32_t t = buf[w];
              if (w < wave) base += t;
              total += t;
            }
          }
          rank = running + base + incl - mine;
          running += total;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int e = 4 * m + c;
          const uint32_t key = key_of(it, c);
          bool keep = key > T;
          if (key == T && inside(e)) {
            keep = !ties || rank < need;
            ++rank;
          }
          const uint64_t kept = __ballot(keep);
          if (kept != 0) {   // uniform over the wave
            const uint32_t slot = claim<THREADS>(kept, emitted, sh.emit);
            if (keep && slot < k) {   // exactly k entries pass; the test only keeps a wrong count inside the layer's slots
              const int64_t dst = (int64_t)i * A.k + L.sel_base + slot;
              A.sel_idx[dst] = base + e;
              if (COMP == Q_TOPK) A.sel_val[dst] = v[it][c];
              atomicOr(&A.keptmap[(int64_t)i * A.map_words + ((uint32_t)(base + e) >> 5)], 1u << ((uint32_t)(base + e) & 31u));
            }
          }
        }
      }
    }
  }
}

// A launch covers a piece of the work list A.layer_work (layers by falling length) from `first`
// on: the first `nblock` layers from there take a whole workgroup each, any others a wave each,
//   THREADS = 1024: grid (nmid, n): the layers above 3,072 entries;
//   THREADS = 256:  grid (nsmall + ceil(ntiny / 4), n): a workgroup per layer above 768
//                   entries, four smaller layers to a workgroup.
// Few workers (the chip is not full either way): one launch of 1024-thread workgroups, one for
// every layer above 768 entries and one for every sixteen smaller ones.
// (64 registers: two 1024-thread workgroups share a compute unit.)
template <int COMP, int THREADS, bool NT>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8)))
void k_layer_compress(Args A, int32_t first, int32_t nblock) {
  constexpr int NW = THREADS / 64;
  __shared__ uint32_t sh_cnt[34];   // 2 x 16 per-wave counts, the result of the first wave's search
  __shared__ uint32_t sh_emit[NW];
  __shared__ uint32_t sh_list_n[NW];
  __shared__ uint2 sh_list[2 * THREADS];
  const int i = blockIdx.y;
  if ((int)blockIdx.x < nblock) {
    const LayerShared sh{sh_cnt, sh_emit, sh_list_n, sh_list};
    layer_body<COMP, THREADS, NT>(A, i, A.layer_work[first + (int)blockIdx.x], (int)threadIdx.x, sh);
  } else {
    const int wave = (int)threadIdx.x >> 6;
    const int idx = first + nblock + ((int)blockIdx.x - nblock) * NW + wave;
    if (idx < A.nlayers) {
      const LayerShared sh{sh_cnt, sh_emit + wave, sh_list_n + wave, sh_list + 128 * wave};
      layer_body<COMP, 64, NT>(A, i, A.layer_work[idx], (int)threadIdx.x & 63, sh);
    }
  }
}

// ---------------------------------------------------------------------------
// sign / gsgd_b layer by layer: norm pass and scales.
// ---------------------------------------------------------------------------

// v = x - xhat over one group (up to 16 chunks = 4096 entries) of one layer: chunk and
// group sums of the layer's norm tree.  One wave per one or two chunks (the shape of k_dense_stat);
// carries the fused local update.  The work items tile every row, padding included, so the
// update reaches every entry.  grid (ngroup_items, n), block stat_threads(NT).
template <int COMP, bool NT>
__global__ __launch_bounds__(stat_threads(NT)) void k_layer_stat(Args A) {
  __shared__ double cs[kGroup];
  const int i = blockIdx.y;
  const LayerGroup item = A.layer_groups[blockIdx.x];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t row = (int64_t)i * A.ld + item.off;
  constexpr int CPW = stat_cpw(NT);
  vf4 a[CPW], b[CPW];
  int e[CPW];   // index of the lane's first entry counted from the group's start
#pragma unroll
  for (int u = 0; u < CPW; ++u) {
    e[u] = (CPW * wave + u) * kChunk + lane * 4;
    if (e[u] < item.rem) {
      if (A.layers_generic) {
        // the layer may start anywhere: entry by entry, and none past the layer's end (the next
        // one may be the first of another layer, or lie beyond the array)
        a[u] = b[u] = vf4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (e[u] + c < item.rem) {
            a[u][c] = A.X[row + e[u] + c];
            b[u][c] = A.Xhat[row + e[u] + c];
          }
      } else {
        a[u] = load4<NT>(A.X + row + e[u]);
        b[u] = load4<NT>(A.Xhat + row + e[u]);
      }
    }
  }
  if (A.G) {   // (never with a generic table: the local update is then a pass of its own)
    vf4 g[CPW];   // all gradient loads before the first store; the momentum memory is read in turn
#pragma unroll
    for (int u = 0; u < CPW; ++u)
      if (e[u] < item.rem) g[u] = load4<true>(A.G + row + e[u]);
#pragma unroll
    for (int u = 0; u < CPW; ++u) {
      if (e[u] < item.rem) {
        vf4 mm = vf4{0.f, 0.f, 0.f, 0.f};
        if (A.M) mm = load4<NT>(A.M + row + e[u]);
        a[u] = local_update_regs(A, a[u], g[u], mm);
        if (A.M) store4<NT>(A.M + row + e[u], mm);
        store4<NT>(A.X + row + e[u], a[u]);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < CPW; ++u) {
    double t = 0.0;
    if (e[u] < item.rem) {
      const vf4 v = a[u] - b[u];
      t = lane_terms<COMP>(v, e[u], item.rem);
    }
    t = wave_tree_sum(t);
    if (lane == 0) cs[CPW * wave + u] = t;
  }
  __syncthreads();
  if (wave == 0) {
    const double t = group_tree_sum(lane < kGroup ? cs[lane] : 0.0);
    if (lane == 0) A.layer_group_sums[(int64_t)i * A.ngroup_items + blockIdx.x] = t;
  }
}

// Third level of a layer's norm tree (256 strided lanes over its group sums, then the
// halving tree, as k_dense_finalise) and the layer's scales (Appendix C with the layer's
// length in the place of d).  grid (nlayers, n), block 256.
template <int COMP>
__global__ __launch_bounds__(256) void k_layer_finalise(Args A) {
  __shared__ double sh[256];
  const int lay = blockIdx.x, i = blockIdx.y, l = threadIdx.x;
  const int g_first = A.layer_group_first[lay];
  const int ngroups = A.layer_group_first[lay + 1] - g_first;
  const double* gs = A.layer_group_sums + (int64_t)i * A.ngroup_items + g_first;
  double acc = 0.0;
  bool first = true;
  for (int g0 = l; g0 < ngroups; g0 += 256 * 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int g = g0 + 256 * u;
      v[u] = g < ngroups ? gs[g] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (g0 + 256 * u < ngroups) {
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
  if (l != 0) return;
  const double total = sh[0];
  const int len = A.layers[lay].len;
  LayerScale ls;
  ls.c = ls.r = ls.step = 0.0f;
  ls.nonzero = 0;
  double nrm = 0.0;
  if (COMP == Q_SIGN) {
    ls.c = (float)(total / (double)len);
  } else {
    nrm = sqrt(total);
    const double s = (double)A.levels, dl = (double)len;
    const double tau = A.qsgd_biased ? 1.0 + fmin(dl / (s * s), sqrt(dl) / s) : 1.0;
    ls.nonzero = nrm > 0.0 ? 1 : 0;
    ls.r = nrm > 0.0 ? (float)(s / nrm) : 0.0f;
    ls.step = nrm > 0.0 ? (float)(nrm / (tau * s)) : 0.0f;
  }
  A.layer_scale[(int64_t)i * A.nlayers + lay] = ls;
  double* scal = A.layer_scal + ((int64_t)i * A.nlayers + lay) * 4;
  scal[0] = total;
  scal[1] = COMP == Q_SIGN ? (double)ls.c : nrm;
  scal[2] = COMP == Q_SIGN ? 0.0 : (double)ls.r;
  scal[3] = COMP == Q_SIGN ? 0.0 : (double)ls.step;
}

}  // namespace choco
