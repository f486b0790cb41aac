// Device code of the CHOCO-Gossip / CHOCO-SGD step for gfx950 (wave64).
//
// Layout: all arrays are n x ld fp32, row-major, one row per worker, ld a
// multiple of 4 so every row starts 16-byte aligned and a lane can always load
// a whole float4 (the pad columns d..ld-1 are read but never take part in a
// norm, a histogram or a selection).
//
// Arithmetic rules shared with no other code: every fp32 product and sum is
// rounded on its own (the file is compiled with -ffp-contract=off), neighbour
// contributions are added in CSR order, norms are accumulated in fp64 over a
// fixed tree (chunks of 256 consecutive entries, 4 per lane, 64-lane butterfly;
// then 256 strided lanes over the chunk sums and a halving tree).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace choco {

enum { Q_IDENTITY = 0, Q_TOPK = 1, Q_RANDK = 2, Q_SIGN = 3, Q_QSGD = 4, Q_NONE = 5 };
enum { STREAM_RANDK = 1, STREAM_DITHER = 2 };

constexpr int kBins = 2048;      // radix-select digits are at most 11 bits wide
constexpr int kChunk = 256;      // entries per first-level norm chunk / tile width
constexpr int kTileThreads = 256;

// Per-worker control block in device memory (written by the small "finalise"
// kernels, read by the streaming kernels; the host never reads it on the hot path).
struct WorkerCtl {
  // norms and scales of the dense operators (Appendix C: sign, gsgd_b)
  double stat;        // ||v||_1 (sign) or sum v^2 (gsgd)
  double nrm;         // ||v||_2 (gsgd)
  float scale_c;      // sign: ||v||_1 / d
  float scale_r;      // gsgd: s / ||v||_2
  float scale_step;   // gsgd: ||v||_2 / (tau s)
  int32_t nonzero;    // gsgd: ||v||_2 > 0
  // radix select of the sparsifying operators (Appendix C: top_a, random_a)
  uint32_t guess_bin;   // first-digit bins >= this are appended to the candidate list
  uint32_t guess_next;  // guess for the next step
  uint32_t b1;          // first digit of the k-th largest key
  uint32_t need;        // how many keys to take from digit b1
  uint32_t mode;        // 0: candidate list is complete, 1: rebuild it, 2: scan the row
  uint32_t cand_count;  // append counter of the candidate list
  uint32_t kept;        // number of entries emitted by the last selection
  uint32_t cnt_b1;      // entries whose first digit is b1
  uint64_t kstar;       // composite key of the k-th largest entry: kept <=> key >= kstar
  uint64_t pad1;
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
  // dense operators
  double* partial;     // n x nchunks first-level chunk sums
  int32_t nchunks;
  int32_t levels;      // gsgd: s
  double tau;          // gsgd: 1 + min(d/s^2, sqrt(d)/s) or 1
  int32_t* codes;      // optional capture of the transmitted codes (n x ld)
  // sparse operators
  int64_t k;
  uint32_t* hist;      // n x kBins
  uint2* cand;         // n x cand_cap  (a, index)
  uint32_t cand_cap;
  int32_t* sel_idx;    // n x k
  float* sel_val;      // n x k
  uint32_t* bitmap;    // n x bitmap_words: bit e of row j set <=> worker j kept entry e
  int64_t bitmap_words;
  int32_t randk_rescale;
  float randk_scale;   // (float)(d / k)
  // randomness
  uint32_t seed_lo, seed_hi, t_lo, t_hi;
};

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
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0);
    const uint32_t lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2);
    const uint32_t lo1 = 0xCD9E8D57u * c2;
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
__device__ __forceinline__ float pick(const float4& v, int c) {
  return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w;
}
__device__ __forceinline__ void put(float4& v, int c, float a) {
  if (c == 0) v.x = a; else if (c == 1) v.y = a; else if (c == 2) v.z = a; else v.w = a;
}

__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void store4(float* p, const float4& v) { *reinterpret_cast<float4*>(p) = v; }

// 64-lane butterfly sum in fp64; lane 0 ends with the halving-tree result
// t[l] += t[l+off] for off = 32,16,...,1 (the sum is commutative, so the xor
// exchange builds exactly that tree in every lane).
__device__ __forceinline__ double wave_tree_sum(double t) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) t = t + __shfl_xor(t, off, 64);
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

// ---------------------------------------------------------------------------
// Local updates (Algorithm 1 line 9; Algorithm 2 lines 9-10).
// grid: (blocks over ld/4, n)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_sgd(float* X, const float* G, int64_t ld, int32_t nvec, float lr) {
  const int64_t row = (int64_t)blockIdx.y * ld;
  for (int m = blockIdx.x * 256 + threadIdx.x; m < nvec; m += gridDim.x * 256) {
    float4 x = load4(X + row + 4 * (int64_t)m);
    const float4 g = load4(G + row + 4 * (int64_t)m);
    x.x = x.x - lr * g.x; x.y = x.y - lr * g.y; x.z = x.z - lr * g.z; x.w = x.w - lr * g.w;
    store4(X + row + 4 * (int64_t)m, x);
  }
}

__global__ __launch_bounds__(256) void k_momentum(float* X, const float* G, float* M, int64_t ld,
                                                  int32_t nvec, float lr, float beta, float lambda) {
  const int64_t row = (int64_t)blockIdx.y * ld;
  for (int m = blockIdx.x * 256 + threadIdx.x; m < nvec; m += gridDim.x * 256) {
    const int64_t o = row + 4 * (int64_t)m;
    float4 x = load4(X + o);
    const float4 g = load4(G + o);
    float4 mo = load4(M + o);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float xc = pick(x, c);
      const float gg = pick(g, c) + lambda * xc;
      const float mn = gg + beta * pick(mo, c);
      put(mo, c, mn);
      put(x, c, xc - lr * mn);
    }
    store4(M + o, mo);
    store4(X + o, x);
  }
}

// ---------------------------------------------------------------------------
// Dense operators, statistic pass: chunk sums of |v| (sign) or v^2 (gsgd) with
// v = x - xhat.  One wave per 256-entry chunk; grid (blocks, n), 4 waves/block.
// ---------------------------------------------------------------------------
template <int COMP>
__device__ __forceinline__ double norm_term(float v) {
  const double a = (double)v;
  return COMP == Q_SIGN ? fabs(a) : a * a;
}

template <int COMP>
__device__ __forceinline__ double lane_terms(const float4& v, int e, int d) {
  // ((t0 + t1) + t2) + t3 with entries past d counting as +0.0
  double acc = (e < d) ? norm_term<COMP>(v.x) : 0.0;
  acc = acc + ((e + 1 < d) ? norm_term<COMP>(v.y) : 0.0);
  acc = acc + ((e + 2 < d) ? norm_term<COMP>(v.z) : 0.0);
  acc = acc + ((e + 3 < d) ? norm_term<COMP>(v.w) : 0.0);
  return acc;
}

template <int COMP>
__global__ __launch_bounds__(256) void k_dense_stat(Args A) {
  const int i = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float* x = A.X + (int64_t)i * A.ld;
  const float* xh = A.Xhat + (int64_t)i * A.ld;
  double* partial = A.partial + (int64_t)i * A.nchunks;
  for (int c = blockIdx.x * 4 + wave; c < A.nchunks; c += gridDim.x * 4) {
    const int e = c * kChunk + lane * 4;
    double t = 0.0;
    if (e < A.d) {
      const float4 a = load4(x + e), b = load4(xh + e);
      float4 v;
      v.x = a.x - b.x; v.y = a.y - b.y; v.z = a.z - b.z; v.w = a.w - b.w;
      t = lane_terms<COMP>(v, e, A.d);
    }
    t = wave_tree_sum(t);
    if (lane == 0) partial[c] = t;
  }
}

// Second level of the norm tree and the per-worker scales.  grid n, block 256.
template <int COMP>
__global__ __launch_bounds__(256) void k_dense_finalise(Args A) {
  __shared__ double t[256];
  const int i = blockIdx.x, l = threadIdx.x;
  const double* partial = A.partial + (int64_t)i * A.nchunks;
  double acc = 0.0;
  bool first = true;
  for (int c = l; c < A.nchunks; c += 256) {
    acc = first ? partial[c] : acc + partial[c];
    first = false;
  }
  t[l] = acc;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if (l < off) t[l] = t[l] + t[l + off];
    __syncthreads();
  }
  if (l == 0) {
    WorkerCtl* ctl = A.ctl + i;
    const double total = t[0];
    ctl->stat = total;
    if (COMP == Q_SIGN) {
      ctl->nrm = 0.0;
      ctl->scale_c = (float)(total / (double)A.d);
    } else {
      const double nrm = sqrt(total);
      const double s = (double)A.levels;
      ctl->nrm = nrm;
      ctl->nonzero = nrm > 0.0 ? 1 : 0;
      ctl->scale_r = nrm > 0.0 ? (float)(s / nrm) : 0.0f;
      ctl->scale_step = nrm > 0.0 ? (float)(nrm / (A.tau * s)) : 0.0f;
    }
  }
}

// ---------------------------------------------------------------------------
// Dense operators, fused apply + mix, compress-then-mix order, direct form.
// One block owns a tile of 256 consecutive columns for ALL n rows, so every
// xhat row is read from HBM once and shared through LDS by the (at most 5)
// workers that mix with it:
//   phase 1  q = Q(x - xhat), xhat += q   (Algorithm 1 lines 3-6), new xhat -> HBM + LDS
//   phase 2  x += gamma * sum_p w_p (xhat_j - xhat_i)   (line 2), CSR order, from LDS
// Wave w owns rows w, w+4, ...; RPW = rows per wave (compile-time bound, x stays
// in registers between the phases).  Dynamic LDS: n * 256 floats.
// ---------------------------------------------------------------------------
template <int COMP, int RPW, bool CAPTURE>
__global__ __launch_bounds__(kTileThreads) void k_dense_apply_mix(Args A) {
  extern __shared__ float tile[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int e = blockIdx.x * kChunk + lane * 4;
  const bool valid = e < A.d;
  float4 xr[RPW];
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + 4 * q;
    if (r < A.n) {
      float4 xh = make_float4(0.f, 0.f, 0.f, 0.f);
      xr[q] = xh;
      if (valid) {
        const int64_t o = (int64_t)r * A.ld + e;
        xr[q] = load4(A.X + o);
        xh = load4(A.Xhat + o);
        RowScale<COMP> sc;
        sc.load(A.ctl + r);
        uint4 words = make_uint4(0, 0, 0, 0);
        if (COMP == Q_QSGD) words = random_words(A, r, (uint32_t)(e >> 2), STREAM_DITHER);
        int32_t code[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float v = pick(xr[q], c) - pick(xh, c);
          const float qv = encode<COMP>(v, sc, pick(words, c), code[c]);
          put(xh, c, pick(xh, c) + qv);
        }
        store4(A.Xhat + o, xh);
        if (CAPTURE) *reinterpret_cast<int4*>(A.codes + o) = make_int4(code[0], code[1], code[2], code[3]);
      }
      store4(tile + r * kChunk + lane * 4, xh);
    }
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + 4 * q;
    if (r < A.n && valid) {
      const float4 me = load4(tile + r * kChunk + lane * 4);
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      const int pend = A.row_ptr[r + 1];
      for (int p = A.row_ptr[r]; p < pend; ++p) {
        const float wj = A.w[p];
        const float4 o = load4(tile + A.col[p] * kChunk + lane * 4);
        acc.x = acc.x + wj * (o.x - me.x);
        acc.y = acc.y + wj * (o.y - me.y);
        acc.z = acc.z + wj * (o.z - me.z);
        acc.w = acc.w + wj * (o.w - me.w);
      }
      float4 x = xr[q];
      x.x = x.x + A.gamma * acc.x;
      x.y = x.y + A.gamma * acc.y;
      x.z = x.z + A.gamma * acc.z;
      x.w = x.w + A.gamma * acc.w;
      store4(A.X + (int64_t)r * A.ld + e, x);
    }
  }
}

// ---------------------------------------------------------------------------
// Tile mix with the xhat that is in memory now (Algorithm 1 line 2, direct
// form), optionally followed by the statistic of v = x_new - xhat for the
// printed order (mix, then compress).  Same tiling as above; the tile is one
// first-level norm chunk, so the chunk sum falls out of one wave butterfly.
// ---------------------------------------------------------------------------
template <int STAT, int RPW>
__global__ __launch_bounds__(kTileThreads) void k_tile_mix(Args A) {
  extern __shared__ float tile[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int e = blockIdx.x * kChunk + lane * 4;
  const bool valid = e < A.d;
  float4 xr[RPW];
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + 4 * q;
    if (r < A.n) {
      float4 xh = make_float4(0.f, 0.f, 0.f, 0.f);
      xr[q] = xh;
      if (valid) {
        const int64_t o = (int64_t)r * A.ld + e;
        xr[q] = load4(A.X + o);
        xh = load4(A.Xhat + o);
      }
      store4(tile + r * kChunk + lane * 4, xh);
    }
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int r = wave + 4 * q;
    if (r < A.n) {
      double t = 0.0;
      if (valid) {
        const float4 me = load4(tile + r * kChunk + lane * 4);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        const int pend = A.row_ptr[r + 1];
        for (int p = A.row_ptr[r]; p < pend; ++p) {
          const float wj = A.w[p];
          const float4 o = load4(tile + A.col[p] * kChunk + lane * 4);
          acc.x = acc.x + wj * (o.x - me.x);
          acc.y = acc.y + wj * (o.y - me.y);
          acc.z = acc.z + wj * (o.z - me.z);
          acc.w = acc.w + wj * (o.w - me.w);
        }
        float4 x = xr[q];
        x.x = x.x + A.gamma * acc.x;
        x.y = x.y + A.gamma * acc.y;
        x.z = x.z + A.gamma * acc.z;
        x.w = x.w + A.gamma * acc.w;
        store4(A.X + (int64_t)r * A.ld + e, x);
        if (STAT != Q_NONE) {
          float4 v;
          v.x = x.x - me.x; v.y = x.y - me.y; v.z = x.z - me.z; v.w = x.w - me.w;
          t = lane_terms<STAT>(v, e, A.d);
        }
      }
      if (STAT != Q_NONE) {
        t = wave_tree_sum(t);
        if (lane == 0) A.partial[(int64_t)r * A.nchunks + blockIdx.x] = t;
      }
    }
  }
}

// Element-wise xhat += Q(x - xhat) (Algorithm 1 lines 3-6) with no mixing.
// grid (blocks over ld/4, n)
template <int COMP, bool CAPTURE>
__global__ __launch_bounds__(256) void k_dense_apply(Args A) {
  const int i = blockIdx.y;
  RowScale<COMP> sc;
  sc.load(A.ctl + i);
  const int nvec = (A.d + 3) >> 2;
  for (int m = blockIdx.x * 256 + threadIdx.x; m < nvec; m += gridDim.x * 256) {
    const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
    const float4 x = load4(A.X + o);
    float4 xh = load4(A.Xhat + o);
    uint4 words = make_uint4(0, 0, 0, 0);
    if (COMP == Q_QSGD) words = random_words(A, i, (uint32_t)m, STREAM_DITHER);
    int32_t code[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float v = pick(x, c) - pick(xh, c);
      const float qv = encode<COMP>(v, sc, pick(words, c), code[c]);
      put(xh, c, pick(xh, c) + qv);
    }
    store4(A.Xhat + o, xh);
    if (CAPTURE) *reinterpret_cast<int4*>(A.codes + o) = make_int4(code[0], code[1], code[2], code[3]);
  }
}

// Direct-form mix reading neighbour rows from global memory (any n; used when
// the tile of all rows does not fit in LDS).  grid (blocks over ld/4, n)
__global__ __launch_bounds__(256) void k_mix_direct_global(Args A) {
  const int i = blockIdx.y;
  const int nvec = (A.d + 3) >> 2;
  const int pbeg = A.row_ptr[i], pend = A.row_ptr[i + 1];
  for (int m = blockIdx.x * 256 + threadIdx.x; m < nvec; m += gridDim.x * 256) {
    const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
    const float4 me = load4(A.Xhat + o);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = pbeg; p < pend; ++p) {
      const float wj = A.w[p];
      const float4 ot = load4(A.Xhat + (int64_t)A.col[p] * A.ld + 4 * (int64_t)m);
      acc.x = acc.x + wj * (ot.x - me.x);
      acc.y = acc.y + wj * (ot.y - me.y);
      acc.z = acc.z + wj * (ot.z - me.z);
      acc.w = acc.w + wj * (ot.w - me.w);
    }
    float4 x = load4(A.X + o);
    x.x = x.x + A.gamma * acc.x;
    x.y = x.y + A.gamma * acc.y;
    x.z = x.z + A.gamma * acc.z;
    x.w = x.w + A.gamma * acc.w;
    store4(A.X + o, x);
  }
}

// Incremental-form mix: x_i += gamma (S_i - xhat_i).  Pure streaming, 16 B/entry.
__global__ __launch_bounds__(256) void k_mix_incremental(Args A) {
  const int i = blockIdx.y;
  const int nvec = (A.d + 3) >> 2;
  for (int m = blockIdx.x * 256 + threadIdx.x; m < nvec; m += gridDim.x * 256) {
    const int64_t o = (int64_t)i * A.ld + 4 * (int64_t)m;
    float4 x = load4(A.X + o);
    const float4 s = load4(A.S + o);
    const float4 xh = load4(A.Xhat + o);
    x.x = x.x + A.gamma * (s.x - xh.x);
    x.y = x.y + A.gamma * (s.y - xh.y);
    x.z = x.z + A.gamma * (s.z - xh.z);
    x.w = x.w + A.gamma * (s.w - xh.w);
    store4(A.X + o, x);
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
// The select finds kstar = the k-th largest K digit by digit; digit 0 (11 bits)
// is histogrammed over the whole row, the remaining digits only over a short
// candidate list of the entries whose digit 0 is >= a guess carried over from
// the previous step (verified against the exact histogram every step).
// ---------------------------------------------------------------------------
template <int COMP>
struct Digits {
  // shifts of the six digits inside the composite key, most significant first
  __device__ __forceinline__ static int shift(int level) {
    if (COMP == Q_TOPK) { const int s[6] = {52, 41, 32, 21, 10, 0}; return s[level]; }
    const int s[6] = {53, 42, 32, 21, 10, 0};
    return s[level];
  }
  __device__ __forceinline__ static int bits(int level) {
    if (COMP == Q_TOPK) { const int b[6] = {11, 11, 9, 11, 11, 10}; return b[level]; }
    const int b[6] = {11, 11, 10, 11, 11, 10};
    return b[level];
  }
  __device__ __forceinline__ static uint32_t key32(uint32_t a) {
    return COMP == Q_TOPK ? (a & 0x7fffffffu) : a;
  }
  __device__ __forceinline__ static uint64_t composite(uint32_t a, uint32_t idx) {
    return ((uint64_t)key32(a) << 32) | (uint64_t)(~idx);
  }
  __device__ __forceinline__ static uint32_t bin0(uint32_t a) {
    return COMP == Q_TOPK ? (key32(a) >> 20) : (a >> 21);
  }
};

// Append (a, idx) of the lanes with pred set to a list, one atomic per wave.
// Must be reached by all 64 lanes of the wave.
__device__ __forceinline__ void wave_append(bool pred, uint32_t a, uint32_t idx, uint32_t* counter,
                                            uint2* list, uint32_t cap) {
  const uint64_t mask = __ballot(pred);
  if (mask == 0) return;
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((unsigned long long)mask) - 1;
  uint32_t base = 0;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(mask));
  base = __shfl(base, leader, 64);
  if (pred) {
    const uint32_t slot = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
    if (slot < cap) list[slot] = make_uint2(a, idx);
  }
}

// One pass over the rows.  HIST: count digit 0 of every entry (first pass of a
// step, all workers).  !HIST: rebuild pass, only for workers whose guess failed.
// DO_MIX (top_a, printed order): first x += gamma (S - xhat), then key x - xhat.
// grid (blocks, n), block 256.
template <int COMP, bool HIST, bool DO_MIX>
__global__ __launch_bounds__(256) void k_sel_pass(Args A) {
  __shared__ uint32_t h[HIST ? kBins : 1];
  const int i = blockIdx.y;
  WorkerCtl* ctl = A.ctl + i;
  if (!HIST && ctl->mode != 1u) return;
  if (HIST) {
    for (int b = threadIdx.x; b < kBins; b += 256) h[b] = 0;
    __syncthreads();
  }
  const uint32_t guess = ctl->guess_bin;
  uint2* cand = A.cand + (int64_t)i * A.cand_cap;
  const int nvec = (A.d + 3) >> 2;
  for (int base = blockIdx.x * 256; base < nvec; base += gridDim.x * 256) {
    const int m = base + threadIdx.x;
    const bool valid = m < nvec;
    const int e = 4 * m;
    uint32_t a[4] = {0, 0, 0, 0};
    if (COMP == Q_TOPK) {
      if (valid) {
        const int64_t o = (int64_t)i * A.ld + e;
        float4 x = load4(A.X + o);
        const float4 xh = load4(A.Xhat + o);
        if (DO_MIX) {
          const float4 s = load4(A.S + o);
          x.x = x.x + A.gamma * (s.x - xh.x);
          x.y = x.y + A.gamma * (s.y - xh.y);
          x.z = x.z + A.gamma * (s.z - xh.z);
          x.w = x.w + A.gamma * (s.w - xh.w);
          store4(A.X + o, x);
        }
        a[0] = __float_as_uint(x.x - xh.x);
        a[1] = __float_as_uint(x.y - xh.y);
        a[2] = __float_as_uint(x.z - xh.z);
        a[3] = __float_as_uint(x.w - xh.w);
      }
    } else {
      if (valid) {
        const uint4 wds = random_words(A, i, (uint32_t)m, STREAM_RANDK);
        a[0] = ~wds.x; a[1] = ~wds.y; a[2] = ~wds.z; a[3] = ~wds.w;
      }
    }
    bool pred[4];
    bool any = false;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool ok = valid && (e + c < A.d);
      const uint32_t bin = Digits<COMP>::bin0(a[c]);
      if (HIST && ok) atomicAdd(&h[bin], 1u);
      pred[c] = ok && bin >= guess;
      any = any || pred[c];
    }
    if (__any(any)) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        wave_append(pred[c], a[c], (uint32_t)(e + c), &ctl->cand_count, cand, A.cand_cap);
    }
  }
  if (HIST) {
    __syncthreads();
    uint32_t* hist = A.hist + (int64_t)i * kBins;
    for (int b = threadIdx.x; b < kBins; b += 256)
      if (h[b]) atomicAdd(&hist[b], h[b]);
  }
}

// Walk a 2048-bin histogram in LDS from the top and find the digit at which the
// running count first reaches `need`.  Called by all threads of a block with
// >= 256 threads; grp is 256 words of LDS scratch; results through LDS words.
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
  if (t == 0) {
    uint32_t cum = 0;
    int g = 255;
    for (; g > 0; --g) {
      if (cum + grp[g] >= need) break;
      cum += grp[g];
    }
    int b = 8 * g + 7;
    for (; b > 8 * g; --b) {
      if (cum + h[b] >= need) break;
      cum += h[b];
    }
    *out_digit = (uint32_t)b;
    *out_above = cum;   // entries in digits above b
  }
  __syncthreads();
}

// Digit 0: find b1, decide whether the candidate list built with the old guess
// is complete, set the next guess.  grid n, block 256.  Clears the histogram.
__global__ __launch_bounds__(256) void k_sel_final0(Args A) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t grp[256];
  __shared__ uint32_t s_digit, s_above;
  const int i = blockIdx.x;
  WorkerCtl* ctl = A.ctl + i;
  uint32_t* hist = A.hist + (int64_t)i * kBins;
  for (int b = threadIdx.x; b < kBins; b += 256) {
    h[b] = hist[b];
    hist[b] = 0;
  }
  __syncthreads();
  find_digit(h, grp, (uint32_t)A.k, &s_digit, &s_above);
  if (threadIdx.x == 0) {
    const uint32_t b1 = s_digit, above = s_above;
    const uint32_t guess = ctl->guess_bin;
    // exact number of entries the old guess put (or tried to put) on the list
    uint64_t listed = 0;
    for (uint32_t b = guess; b < (uint32_t)kBins; ++b) listed += h[b];
    const bool ok = (guess <= b1) && (listed <= (uint64_t)A.cand_cap);
    uint32_t mode = 0;
    if (!ok) {
      const uint64_t rebuilt = (uint64_t)above + (uint64_t)h[b1];
      if (rebuilt <= (uint64_t)A.cand_cap) {
        mode = 1;
        ctl->guess_bin = b1;
        ctl->cand_count = 0;
      } else {
        mode = 2;
      }
    }
    // next step: one digit of slack below b1 if that list still fits
    uint32_t next = b1;
    if (b1 > 0) {
      const uint64_t wide = (uint64_t)above + (uint64_t)h[b1] + (uint64_t)h[b1 - 1];
      if (wide <= (uint64_t)A.cand_cap) next = b1 - 1;
    }
    ctl->guess_next = next;
    ctl->b1 = b1;
    ctl->cnt_b1 = h[b1];
    ctl->need = (uint32_t)A.k - above;
    ctl->mode = mode;
  }
}

// Finish the select on the candidate list (or, in the degenerate case that the
// list cannot hold digit b1, on the row itself), emit the kept (index, value)
// pairs and mark them in the bitmap.  grid n, block 1024.
template <int COMP, bool ROW>
__device__ __forceinline__ void fetch_entry(const Args& A, int i, const uint2* cand, uint32_t t,
                                            uint32_t& a, uint32_t& idx) {
  if (!ROW) {
    const uint2 c = cand[t];
    a = c.x;
    idx = c.y;
  } else {
    idx = t;
    if (COMP == Q_TOPK) {
      const int64_t o = (int64_t)i * A.ld + t;
      a = __float_as_uint(A.X[o] - A.Xhat[o]);
    } else {
      const uint4 wds = random_words(A, i, t >> 2, STREAM_RANDK);
      a = ~pick(wds, (int)(t & 3u));
    }
  }
}

template <int COMP, bool ROW>
__device__ void refine_and_emit(const Args& A, int i, uint32_t count, uint32_t* h, uint32_t* grp,
                                uint64_t* s_prefix, uint32_t* s_need, uint32_t* s_digit,
                                uint32_t* s_above, uint32_t* s_emit) {
  WorkerCtl* ctl = A.ctl + i;
  const uint2* cand = A.cand + (int64_t)i * A.cand_cap;
  int last = 0;  // last digit that has been resolved
  // digit 0 is known; if all of digit b1 is needed there is nothing to refine
  bool done = (ctl->cnt_b1 == *s_need);
  for (int level = 1; level < 6 && !done; ++level) {
    for (int b = threadIdx.x; b < kBins; b += blockDim.x) h[b] = 0;
    __syncthreads();
    const uint64_t prefix = *s_prefix;
    const int sprev = Digits<COMP>::shift(level - 1);
    const int scur = Digits<COMP>::shift(level);
    const uint32_t mask = (1u << Digits<COMP>::bits(level)) - 1u;
    for (uint32_t t = threadIdx.x; t < count; t += blockDim.x) {
      uint32_t a, idx;
      fetch_entry<COMP, ROW>(A, i, cand, t, a, idx);
      const uint64_t K = Digits<COMP>::composite(a, idx);
      if ((K >> sprev) == prefix) atomicAdd(&h[(uint32_t)(K >> scur) & mask], 1u);
    }
    __syncthreads();
    find_digit(h, grp, *s_need, s_digit, s_above);
    const uint32_t digit = *s_digit, above = *s_above;
    const uint32_t in_digit = h[digit];
    const uint32_t need = *s_need - above;
    __syncthreads();
    if (threadIdx.x == 0) {
      *s_prefix = (prefix << Digits<COMP>::bits(level)) | (uint64_t)digit;
      *s_need = need;
    }
    last = level;
    done = (in_digit == need);
    __syncthreads();
  }
  const uint64_t kstar = *s_prefix << Digits<COMP>::shift(last);
  // emit every entry with composite >= kstar
  int32_t* sel_idx = A.sel_idx + (int64_t)i * A.k;
  float* sel_val = A.sel_val + (int64_t)i * A.k;
  uint32_t* bitmap = A.bitmap + (int64_t)i * A.bitmap_words;
  const uint32_t rounds = (count + blockDim.x - 1) / blockDim.x;
  for (uint32_t rd = 0; rd < rounds; ++rd) {
    const uint32_t t = rd * blockDim.x + threadIdx.x;
    uint32_t a = 0, idx = 0;
    bool keep = false;
    if (t < count) {
      fetch_entry<COMP, ROW>(A, i, cand, t, a, idx);
      keep = Digits<COMP>::composite(a, idx) >= kstar;
    }
    const uint64_t mask = __ballot(keep);
    if (mask != 0) {
      const int lane = threadIdx.x & 63;
      const int leader = __ffsll((unsigned long long)mask) - 1;
      uint32_t base = 0;
      if (lane == leader) base = atomicAdd(s_emit, (uint32_t)__popcll(mask));
      base = __shfl(base, leader, 64);
      if (keep) {
        const uint32_t slot = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        if (slot < (uint32_t)A.k) {
          float val;
          if (COMP == Q_TOPK) {
            val = __uint_as_float(a);
          } else {
            const int64_t o = (int64_t)i * A.ld + idx;
            val = A.X[o] - A.Xhat[o];
            if (A.randk_rescale) val = A.randk_scale * val;
          }
          sel_idx[slot] = (int32_t)idx;
          sel_val[slot] = val;
          atomicOr(&bitmap[idx >> 5], 1u << (idx & 31u));
        }
      }
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ctl->kstar = kstar;
    ctl->kept = *s_emit;
    ctl->cand_count = 0;
    ctl->guess_bin = ctl->guess_next;
  }
}

template <int COMP>
__global__ __launch_bounds__(1024) void k_sel_refine(Args A) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t grp[256];
  __shared__ uint64_t s_prefix;
  __shared__ uint32_t s_need, s_digit, s_above, s_emit;
  const int i = blockIdx.x;
  WorkerCtl* ctl = A.ctl + i;
  const uint32_t mode = ctl->mode;
  if (threadIdx.x == 0) {
    s_prefix = ctl->b1;
    s_need = ctl->need;
    s_emit = 0;
  }
  __syncthreads();
  if (mode == 2u) {
    refine_and_emit<COMP, true>(A, i, (uint32_t)A.d, h, grp, &s_prefix, &s_need, &s_digit, &s_above, &s_emit);
  } else {
    uint32_t count = ctl->cand_count;
    if (count > A.cand_cap) count = A.cand_cap;
    __syncthreads();
    refine_and_emit<COMP, false>(A, i, count, h, grp, &s_prefix, &s_need, &s_digit, &s_above, &s_emit);
  }
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
  const uint32_t word = (uint32_t)e >> 5, bit = 1u << ((uint32_t)e & 31u);
  for (int p2 = pbeg; p2 < p; ++p2)
    if (A.bitmap[(int64_t)A.col[p2] * A.bitmap_words + word] & bit) return;
  float* s = A.S + (int64_t)i * A.ld + e;
  float acc = *s;
  acc = acc + A.w[p] * A.sel_val[(int64_t)j * A.k + m];
  for (int p2 = p + 1; p2 < pend; ++p2) {
    const int j2 = A.col[p2];
    if (A.bitmap[(int64_t)j2 * A.bitmap_words + word] & bit) {
      const int64_t o = (int64_t)j2 * A.ld + e;
      float q = A.X[o] - A.Xhat[o];
      if (A.randk_rescale) q = A.randk_scale * q;
      acc = acc + A.w[p2] * q;
    }
  }
  *s = acc;
}

// xhat_j[e] += q_j[e] for the kept entries (Algorithm 1 line 6); clears the
// bitmap words it touched.  grid (ceil(k/256), n)
__global__ __launch_bounds__(256) void k_xhat_update(Args A) {
  const int j = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  const int e = A.sel_idx[(int64_t)j * A.k + m];
  float* xh = A.Xhat + (int64_t)j * A.ld + e;
  *xh = *xh + A.sel_val[(int64_t)j * A.k + m];
  A.bitmap[(int64_t)j * A.bitmap_words + ((uint32_t)e >> 5)] = 0u;
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

}  // namespace choco
