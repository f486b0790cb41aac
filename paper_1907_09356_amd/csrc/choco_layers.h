// Layer-wise compression (Section 5, set-up of the deep-learning runs: the operator is
// applied to every layer of the network on its own).
//
// One block per (worker, layer); the layer's x - xhat lives in registers (kLayerVecs
// 4-vectors per thread, so a block of T threads holds up to 40 T entries and the largest
// layer a 1024-thread block can take has 40,960 entries), so one launch reads x, g, xhat
// once and does the whole operator:
//   sign / gsgd_b   the norm tree of the layer (same three levels as for a whole row:
//                   a wave's 64 lanes x 4 entries are exactly one 256-entry chunk), the
//                   per-layer scale, the codes, xhat += q
//   top_a/random_a  an exact k-th largest key by a bitwise search on block-wide counts
//                   (31 or 32 rounds over the registers, no atomics, no histogram), ties
//                   on the threshold key broken by ascending index, then the kept
//                   (index, value) pairs and the kept-entry map
// Layers are grouped by size into three launches (64, 256 and 1024 threads per block).
#pragma once

#include "choco_kernels.h"

namespace choco {

constexpr int kLayerVecs = 10;
constexpr int kMaxLayerLen = 1024 * kLayerVecs * 4;
constexpr int kLayerMaxChunks = 16 * kLayerVecs;   // 256-entry chunks of the largest layer

template <int THREADS>
__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* sh, int& phase) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  if (THREADS == 64) return v;
  // two buffers in turn: a wave may write round j+1 while another still reads round j
  uint32_t* buf = sh + 16 * phase;
  phase ^= 1;
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
  __syncthreads();
  uint32_t tot = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) tot += buf[w];
  return tot;
}

// grid (layers of this size class, n); `first` indexes A.layer_ids
template <int COMP, int THREADS, bool NT>
__global__ __launch_bounds__(THREADS) void k_layer_compress(Args A, int32_t first) {
  constexpr bool DENSE = (COMP == Q_SIGN || COMP == Q_QSGD);
  constexpr int NW = THREADS / 64;
  __shared__ double sh_chunk[DENSE ? kLayerMaxChunks : 1];
  __shared__ uint32_t sh_cnt[32];
  __shared__ uint32_t sh_emit;
  const int i = blockIdx.y;
  const int l = A.layer_ids[first + (int)blockIdx.x];
  const LayerDesc L = A.layers[l];
  const int nvec = (L.len + 3) >> 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = (int64_t)i * A.ld + L.start;
  double* scal = A.layer_scal + ((int64_t)i * A.nlayers + l) * 4;
  if (tid == 0) sh_emit = 0;

  // ---- load: v = x - xhat (after the local update, if this pass carries it) ----
  vf4 v[kLayerVecs], xh[DENSE ? kLayerVecs : 1];
  uint32_t word_key[COMP == Q_RANDK ? kLayerVecs : 1][4];
#pragma unroll
  for (int it = 0; it < kLayerVecs; ++it) {
    const int m = it * THREADS + tid;
    v[it] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (COMP == Q_RANDK) {
      // keys are ~word: the k smallest words are the k largest keys
      uint4 wd = make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu);
      if (m < nvec) wd = random_words(A, i, (uint32_t)(L.start >> 2) + (uint32_t)m, STREAM_RANDK);
#pragma unroll
      for (int c = 0; c < 4; ++c) word_key[it][c] = (4 * m + c < L.len) ? ~pick(wd, c) : 0u;
    } else if (m < nvec) {
      const int64_t o = row + 4 * (int64_t)m;
      vf4 x = load4<NT>(A.X + o);
      if (A.G) {
        x = local_update4<NT>(A, o, x);
        store4<NT>(A.X + o, x);
      }
      const vf4 h = load4<NT>(A.Xhat + o);
      if constexpr (DENSE) xh[it] = h;
#pragma unroll
      for (int c = 0; c < 4; ++c) v[it][c] = (4 * m + c < L.len) ? x[c] - h[c] : 0.0f;
    }
  }

  if constexpr (DENSE) {
    // ---- norm tree of the layer ----
    constexpr int STAT = DENSE ? COMP : Q_SIGN;
    const int nchunks = (L.len + kChunk - 1) / kChunk;
#pragma unroll
    for (int it = 0; it < kLayerVecs; ++it) {
      const int chunk = it * NW + wave;
      if (chunk < nchunks) {                       // uniform over the wave
        const int m = it * THREADS + tid;
        double t = lane_terms<STAT>(v[it], 4 * m, L.len);
        t = wave_tree_sum(t);
        if (lane == 0) sh_chunk[chunk] = t;
      }
    }
    __syncthreads();
    // levels 2 and 3, done by every wave for itself: groups of 16 chunk sums (four groups
    // per round over the 64 lanes), then the lanes that stand for a group sum each
    const int ngroups = (nchunks + kGroup - 1) / kGroup;
    double g = 0.0;
#pragma unroll
    for (int r = 0; r < (kLayerMaxChunks / kGroup + 3) / 4; ++r) {
      const int chunk = 64 * r + lane;
      double t = chunk < nchunks ? sh_chunk[chunk] : 0.0;
      t = group_tree_sum(t);
      const double got = __shfl(t, 16 * (lane & 3), 64);
      if ((lane >> 2) == r && lane < ngroups) g = got;
    }
    const double total = wave_tree_sum(g);
    // ---- per-layer scales (Appendix C with the layer's length in the place of d) ----
    RowScale<STAT> sc;
    sc.c = sc.r = sc.step = 0.0f;
    sc.nonzero = 0;
    double nrm = 0.0;
    if (COMP == Q_SIGN) {
      sc.c = (float)(total / (double)L.len);
    } else {
      nrm = sqrt(total);
      const double s = (double)A.levels, dl = (double)L.len;
      const double tau = A.qsgd_biased ? 1.0 + fmin(dl / (s * s), sqrt(dl) / s) : 1.0;
      sc.nonzero = nrm > 0.0 ? 1 : 0;
      sc.r = nrm > 0.0 ? (float)(s / nrm) : 0.0f;
      sc.step = nrm > 0.0 ? (float)(nrm / (tau * s)) : 0.0f;
    }
    if (tid == 0) {
      scal[0] = total;
      scal[1] = COMP == Q_SIGN ? (double)sc.c : nrm;
      scal[2] = COMP == Q_SIGN ? 0.0 : (double)sc.r;
      scal[3] = COMP == Q_SIGN ? 0.0 : (double)sc.step;
    }
    // ---- codes and xhat += q ----
#pragma unroll
    for (int it = 0; it < kLayerVecs; ++it) {
      const int m = it * THREADS + tid;
      if (m < nvec) {
        uint4 wd = make_uint4(0u, 0u, 0u, 0u);
        if (COMP == Q_QSGD) wd = random_words(A, i, (uint32_t)(L.start >> 2) + (uint32_t)m, STREAM_DITHER);
        vi4 code = vi4{0, 0, 0, 0};
        vf4 h = xh[it];
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (4 * m + c < L.len) {
            int32_t cd;
            const float qv = encode<STAT>(v[it][c], sc, pick(wd, c), cd);
            h[c] = h[c] + qv;
            code[c] = cd;
          }
        const int64_t o = row + 4 * (int64_t)m;
        store4<NT>(A.Xhat + o, h);
        if (A.codes) *reinterpret_cast<vi4*>(A.codes + o) = code;
      }
    }
    return;
  } else {
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
  int phase = 0;
  uint32_t T = 0;
  for (int bit = (COMP == Q_RANDK ? 31 : 30); bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    uint32_t cnt = 0;
#pragma unroll
    for (int it = 0; it < kLayerVecs; ++it)
#pragma unroll
      for (int c = 0; c < 4; ++c) cnt += key_of(it, c) >= cand ? 1u : 0u;
    if (block_sum_u32<THREADS>(cnt, sh_cnt, phase) >= k) T = cand;
  }
  // entries above the threshold key are all kept; of those equal to it, the first `need`
  // by index (entries past the layer's end carry key 0 and are told apart by their index)
  uint32_t above = 0, equals = 0;
#pragma unroll
  for (int it = 0; it < kLayerVecs; ++it) {
    const int m = it * THREADS + tid;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t key = key_of(it, c);
      above += key > T ? 1u : 0u;
      equals += (key == T && 4 * m + c < L.len) ? 1u : 0u;
    }
  }
  above = block_sum_u32<THREADS>(above, sh_cnt, phase);
  equals = block_sum_u32<THREADS>(equals, sh_cnt, phase);
  const uint32_t need = k - above;
  if (tid == 0) {
    scal[0] = (double)T;
    scal[1] = (double)need;
    scal[2] = (double)equals;
    scal[3] = (double)k;
  }
  const bool ties = equals > need;   // uniform over the block
  uint32_t running = 0;              // threshold-key entries in earlier rounds (index order)
#pragma unroll
  for (int it = 0; it < kLayerVecs; ++it) {
    const int m = it * THREADS + tid;
    uint32_t rank = 0;
    if (ties) {
      uint32_t mine = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) mine += (key_of(it, c) == T && 4 * m + c < L.len) ? 1u : 0u;
      uint32_t incl = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
      }
      uint32_t base = 0, total = __shfl(incl, 63, 64);
      if (THREADS > 64) {
        uint32_t* buf = sh_cnt + 16 * phase;
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
      if (key == T && e < L.len) {
        keep = !ties || rank < need;
        ++rank;
      }
      if (keep) {
        const uint32_t slot = atomicAdd(&sh_emit, 1u);
        if (slot < k) {   // exactly k entries pass; the test only keeps a wrong count inside the layer's slots
          const int64_t dst = (int64_t)i * A.k + L.sel_base + slot;
          A.sel_idx[dst] = L.start + e;
          if (COMP == Q_TOPK) A.sel_val[dst] = v[it][c];
          A.keptmap[row + e] = 1;
        }
      }
    }
  }
  }
}

}  // namespace choco
