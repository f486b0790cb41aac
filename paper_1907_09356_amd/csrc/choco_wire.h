// Messages on the wire (Appendix C states a size with each operator: d + 32 bits for
// sign, 2*32*k for top_a, 32*k for random_a, b bits per entry for gsgd_b).  These kernels
// encode the q of the last gossip step into those sizes and decode them again; they are
// not on the timed path (on one GPU "sending" is memory traffic), they are what a
// worker-per-GPU mapping would put on the links.  For sign and gsgd the bits of the message
// are written by the compress pass itself (the bit planes of choco_kernels.h); packing is a
// copy of those planes behind the header (whole vector) or their re-alignment layer by layer.
//
// Layout, 32-bit words, W = ceil(d / 32), one message per worker, messages back to back:
//   sign      [c as float][W words: bit e%32 of word e/32 set iff the entry is -c]
//   gsgd      [step as float][4 words: ascending indices of entries whose level exceeds
//             the magnitude bits, 0xFFFFFFFF when unused][plane 0: signs of the non-zero
//             levels][planes 1..mb: bit p-1 of min(level, 2^mb - 1)], mb = bit length of s-1
//   top_a     k pairs [index][value]; the order of the pairs is not specified
//   random_a  k values in ascending order of index (the receiver draws the same mask)
#pragma once

#include "choco_kernels.h"

namespace choco {

constexpr int kOverflowSlots = 4;

struct WireArgs {
  int32_t n, d;
  int64_t ld;
  int64_t words;            // words per message
  int64_t W;                // words per bit plane
  int32_t mb;               // gsgd: magnitude bits
  int32_t levels;
  const uint32_t* planes;   // n x nplanes x plane_words: bit planes of the last step's codes (sign, gsgd)
  int64_t plane_words;      // ceil(ld / 32)
  int32_t nplanes;
  const uint4* ovf_ring;    // gsgd: entries at level s remembered by the compress pass, tagged with the step
  uint32_t t_lo, t_hi;      // the step the messages are of
  const WorkerCtl* ctl;
  int64_t k;
  const int32_t* sel_idx;
  const float* sel_val;
  const uint32_t* bitmap;
  int64_t bitmap_words;
  // random_a without a bitmap built by the select (long rows, layer by layer): ranks come from the
  // bit map of kept entries, marked anew from the kept-index list for the duration of the call
  uint32_t* keptmap;        // n x map_words, all zero between steps
  int64_t map_words;        // ceil(ld / 32)
  uint32_t* chunk_rank;     // n x nchunk: kept entries of a worker below each 1024-entry chunk
  int64_t nchunk;           // ceil(ld / 1024)
  // layer by layer: a worker's message is its layers' messages one after the other
  const LayerDesc* layers;
  int32_t nlayers;
  const int64_t* layer_word_off;    // nlayers + 1: where each layer's message starts (words)
  const int64_t* layer_plane_off;   // nlayers + 1: prefix of the layers' plane lengths ceil(len / 32)
  const LayerScale* layer_scale;    // n x nlayers
};

// The layer that holds word pw of the row's concatenated bit planes.
__device__ __forceinline__ int plane_layer(const WireArgs& A, int64_t pw) {
  int lo = 0, hi = A.nlayers - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (A.layer_plane_off[mid] <= pw) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

// The index slots of a gsgd message: the entries the compress pass remembered for this step,
// ascending, 0xFFFFFFFF where unused.  (At most four entries of a vector reach level s: each
// needs |v| r + u >= s with u < 1, i.e. more than half of the norm up to rounding, and the squares
// of four such shares already add up to the whole.)
__device__ __forceinline__ void ring_slots(const WireArgs& A, int64_t unit, uint32_t (&v)[kOverflowSlots]) {
  int cnt = 0;
#pragma unroll
  for (int j = 0; j < kOverflowSlots; ++j) v[j] = 0xFFFFFFFFu;
  for (int s = 0; s < kOvfRing; ++s) {
    const uint4 r = A.ovf_ring[unit * kOvfRing + s];
    if (r.x == A.t_lo && r.y == A.t_hi + 1u && cnt < kOverflowSlots) v[cnt++] = r.z;
  }
  for (int a = 1; a < kOverflowSlots; ++a)
    for (int b = a; b > 0 && v[b] < v[b - 1]; --b) {
      const uint32_t t = v[b];
      v[b] = v[b - 1];
      v[b - 1] = t;
    }
}

// Word w of plane p of layer L of worker i: the row's plane holds bit e of the row at bit e%32 of
// word e/32, the layer's message counts bits from the layer's first entry.
__device__ __forceinline__ uint32_t layer_plane_word(const WireArgs& A, int i, int p, const LayerDesc& L, int64_t w) {
  const uint32_t* P = A.planes + ((int64_t)i * A.nplanes + p) * A.plane_words;
  const int64_t b0 = (int64_t)L.start + 32 * w;
  const int sh = (int)(b0 & 31);
  const int64_t i0 = b0 >> 5;
  uint32_t v = P[i0] >> sh;
  if (sh && i0 + 1 < A.plane_words) v |= P[i0 + 1] << (32 - sh);
  const int64_t left = (int64_t)L.len - 32 * w;     // bits of this word that belong to the layer
  if (left < 32) v &= (1u << left) - 1u;
  return v;
}

// sign / gsgd layer by layer.  grid (ceil(total plane words / 256), n): one thread per word position
// of one layer, all planes.  GSGD = false: sign.
template <bool GSGD>
__global__ __launch_bounds__(256) void k_pack_dense_layers(WireArgs A, uint32_t* msg) {
  const int i = blockIdx.y;
  const int64_t pw = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (pw >= A.layer_plane_off[A.nlayers]) return;
  const int lay = plane_layer(A, pw);
  const LayerDesc L = A.layers[lay];
  const int64_t w = pw - A.layer_plane_off[lay];
  const int64_t W = A.layer_plane_off[lay + 1] - A.layer_plane_off[lay];
  uint32_t* out = msg + (int64_t)i * A.words + A.layer_word_off[lay];
  const LayerScale ls = A.layer_scale[(int64_t)i * A.nlayers + lay];
  if (w == 0) out[0] = __float_as_uint(GSGD ? ls.step : ls.c);
  if (!GSGD) {
    out[1 + w] = layer_plane_word(A, i, 0, L, w);
    return;
  }
  if (w == 0) {
    uint32_t v[kOverflowSlots];
    ring_slots(A, (int64_t)i * A.nlayers + lay, v);
#pragma unroll
    for (int j = 0; j < kOverflowSlots; ++j) out[1 + j] = v[j];
  }
  uint32_t* planes = out + 1 + kOverflowSlots;
  for (int p = 0; p < A.nplanes; ++p) planes[(int64_t)p * W + w] = layer_plane_word(A, i, p, L, w);
}

// after k_wire_zero.  grid (ceil(total plane words / 256), n)
template <bool GSGD>
__global__ __launch_bounds__(256) void k_unpack_dense_layers(WireArgs A, const uint32_t* msg, float* q) {
  const int i = blockIdx.y;
  const int64_t pw = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (pw >= A.layer_plane_off[A.nlayers]) return;
  const int lay = plane_layer(A, pw);
  const LayerDesc L = A.layers[lay];
  const int64_t w = pw - A.layer_plane_off[lay];
  const int64_t W = A.layer_plane_off[lay + 1] - A.layer_plane_off[lay];
  const uint32_t* in = msg + (int64_t)i * A.words + A.layer_word_off[lay];
  const float scale = __uint_as_float(in[0]);
  float* dst = q + (int64_t)i * A.ld + L.start + 32 * w;
  if (!GSGD) {
    const uint32_t bits = in[1 + w];
    for (int j = 0; j < 32; ++j)
      if (32 * w + j < L.len) dst[j] = ((bits >> j) & 1u) ? -scale : scale;
    return;
  }
  const uint32_t* planes = in + 1 + kOverflowSlots;
  const uint32_t sign = planes[w];
  for (int j = 0; j < 32; ++j) {
    if (32 * w + j >= L.len) break;
    int32_t level = 0;
    for (int p = 0; p < A.mb; ++p) level |= (int32_t)((planes[(int64_t)(1 + p) * W + w] >> j) & 1u) << p;
    for (int s = 0; s < kOverflowSlots; ++s)
      if (in[1 + s] == (uint32_t)(32 * w + j)) level = A.levels;
    const float mag = (float)level * scale;
    dst[j] = ((sign >> j) & 1u) ? -mag : mag;
  }
}

// sign / gsgd on the whole vector: the header (scale or step, and for gsgd the index slots), then
// the planes as the compress pass wrote them.  grid (ceil(W / 256), nplanes, n)
template <bool GSGD>
__global__ __launch_bounds__(256) void k_pack_planes(WireArgs A, uint32_t* msg) {
  const int i = blockIdx.z, p = blockIdx.y;
  const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t* out = msg + (int64_t)i * A.words;
  if (w == 0 && p == 0) {
    out[0] = __float_as_uint(GSGD ? A.ctl[i].scale_step : A.ctl[i].scale_c);
    if (GSGD) {
      uint32_t v[kOverflowSlots];
      ring_slots(A, (int64_t)i, v);
#pragma unroll
      for (int j = 0; j < kOverflowSlots; ++j) out[1 + j] = v[j];
    }
  }
  if (w >= A.W) return;
  const int64_t hdr = GSGD ? 1 + kOverflowSlots : 1;
  out[hdr + (int64_t)p * A.W + w] = A.planes[((int64_t)i * A.nplanes + p) * A.plane_words + w];
}

// grid (ceil(k / 256), n)
__global__ __launch_bounds__(256) void k_pack_topk(WireArgs A, uint32_t* msg) {
  const int i = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  uint32_t* out = msg + (int64_t)i * A.words;
  out[2 * m] = (uint32_t)A.sel_idx[(int64_t)i * A.k + m];
  out[2 * m + 1] = __float_as_uint(A.sel_val[(int64_t)i * A.k + m]);
}

// Exclusive prefix of the bit counts of a worker's kept-entry bitmap into LDS.
// block 1024; pre holds bitmap_words entries.
__device__ __forceinline__ void bitmap_prefix(const WireArgs& A, int i, uint32_t* pre, uint32_t* sh_wave) {
  const uint32_t* bm = A.bitmap + (int64_t)i * A.bitmap_words;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t per = (A.bitmap_words + 1023) / 1024;      // consecutive words per thread
  const int64_t w0 = (int64_t)tid * per;
  uint32_t mine = 0;
  for (int64_t w = w0; w < w0 + per && w < A.bitmap_words; ++w) mine += __popc(bm[w]);
  uint32_t incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  if (lane == 63) sh_wave[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += sh_wave[w];
  uint32_t run = base + incl - mine;
  for (int64_t w = w0; w < w0 + per && w < A.bitmap_words; ++w) {
    pre[w] = run;
    run += __popc(bm[w]);
  }
  __syncthreads();
}

// random_a with a bitmap per worker: the value of kept entry e goes to position
// rank(e) = number of kept entries below e.  grid n, block 1024, dynamic LDS = bitmap_words words
__global__ __launch_bounds__(1024) void k_pack_randk(WireArgs A, uint32_t* msg) {
  extern __shared__ uint32_t pre[];
  __shared__ uint32_t sh_wave[16];
  const int i = blockIdx.x;
  bitmap_prefix(A, i, pre, sh_wave);
  const uint32_t* bm = A.bitmap + (int64_t)i * A.bitmap_words;
  uint32_t* out = msg + (int64_t)i * A.words;
  for (int64_t m = threadIdx.x; m < A.k; m += 1024) {
    const uint32_t e = (uint32_t)A.sel_idx[(int64_t)i * A.k + m];
    const uint32_t rank = pre[e >> 5] + __popc(bm[e >> 5] & ((1u << (e & 31u)) - 1u));
    out[rank] = __float_as_uint(A.sel_val[(int64_t)i * A.k + m]);
  }
}

// ---- the receiver's side: dense q (n x ld) from the messages ----

// grid (ceil(ld / 1024), n): q = 0
__global__ __launch_bounds__(256) void k_wire_zero(float* q, int64_t ld) {
  const int64_t o = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (o < ld) *reinterpret_cast<vf4*>(q + (int64_t)blockIdx.y * ld + o) = vf4{0.0f, 0.0f, 0.0f, 0.0f};
}

// The dense decoders: a workgroup decodes 256 words of every plane (8192 entries), a thread one
// 4-vector of q per turn with the 4-vectors of a wave next to each other, so that a store
// instruction fills whole lines (a thread that decodes a word of its own stores 128 bytes apart
// from its neighbour's: 800 us for the 896 MB of q at n = 8, d = 28 M).  The eight lanes that
// share a plane word read it through the vector cache.  Pad columns of the last 4-vector get
// zeros; grid (ceil(W / 256), n); the gsgd decoder takes (1 + mb) KiB of dynamic LDS.
__device__ __forceinline__ void store_vec(const WireArgs& A, float* q, int i, int64_t vec, const float (&v)[4]) {
  vf4 o;
#pragma unroll
  for (int u = 0; u < 4; ++u) o[u] = (4 * vec + u < A.d) ? v[u] : 0.0f;
  *reinterpret_cast<vf4*>(q + (int64_t)i * A.ld + 4 * vec) = o;
}

__global__ __launch_bounds__(256) void k_unpack_sign(WireArgs A, const uint32_t* msg, float* q) {
  const int i = blockIdx.y;
  const uint32_t* in = msg + (int64_t)i * A.words;
  const float c = __uint_as_float(in[0]);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int64_t vec = (int64_t)blockIdx.x * 2048 + j * 256 + threadIdx.x;
    if (4 * vec >= A.d) break;
    const uint32_t bits = in[1 + (vec >> 3)] >> ((int)(vec & 7) * 4);
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = ((bits >> u) & 1u) ? -c : c;
    store_vec(A, q, i, vec, v);
  }
}

// PACKED (levels < 256): the four levels of a 4-vector are the four bytes of one word.
template <bool PACKED>
__global__ __launch_bounds__(256) void k_unpack_gsgd(WireArgs A, const uint32_t* msg, float* q) {
  const int i = blockIdx.y;
  const uint32_t* in = msg + (int64_t)i * A.words;
  const float step = __uint_as_float(in[0]);
  const uint32_t* planes = in + 1 + kOverflowSlots;
  uint32_t ovf[kOverflowSlots];
#pragma unroll
  for (int s = 0; s < kOverflowSlots; ++s) ovf[s] = in[1 + s];
  // the workgroup's 256 words of every plane through LDS: one load per thread and plane, all
  // in flight together, instead of a round trip to memory in each of the eight turns
  extern __shared__ uint32_t pl[];   // (1 + mb) x 256
  {
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (int p = 0; p <= A.mb; ++p) pl[p * 256 + threadIdx.x] = w < A.W ? planes[(int64_t)p * A.W + w] : 0u;
  }
  __syncthreads();
  const int sh = (int)(threadIdx.x & 7) * 4;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int64_t vec = (int64_t)blockIdx.x * 2048 + j * 256 + threadIdx.x;
    if (4 * vec >= A.d) break;
    const int lw = j * 32 + (int)(threadIdx.x >> 3);
    uint32_t level[4] = {0, 0, 0, 0};
    for (int p = 0; p < A.mb; ++p) {
      const uint32_t nib = (pl[(1 + p) * 256 + lw] >> sh) & 15u;
      if (PACKED) {
        // a plane's nibble times 0x204081 puts bit u at bit 8 u (and other bits elsewhere)
        level[0] |= ((nib * 0x204081u) & 0x01010101u) << p;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) level[u] |= ((nib >> u) & 1u) << p;
      }
    }
    if (PACKED) {
#pragma unroll
      for (int u = 1; u < 4; ++u) level[u] = (level[0] >> (8 * u)) & 0xFFu;
      level[0] &= 0xFFu;
    }
#pragma unroll
    for (int s = 0; s < kOverflowSlots; ++s)
      if (ovf[s] != 0xFFFFFFFFu && (int64_t)(ovf[s] >> 2) == vec) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if ((int)(ovf[s] & 3u) == u) level[u] = (uint32_t)A.levels;
      }
    const uint32_t sign = pl[lw] >> sh;
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float mag = (float)level[u] * step;
      v[u] = __uint_as_float(__float_as_uint(mag) | (((sign >> u) & 1u) << 31));
    }
    store_vec(A, q, i, vec, v);
  }
}

// after k_wire_zero.  grid (ceil(k / 256), n)
__global__ __launch_bounds__(256) void k_unpack_topk(WireArgs A, const uint32_t* msg, float* q) {
  const int i = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  const uint32_t* in = msg + (int64_t)i * A.words;
  const uint32_t e = in[2 * m];
  if (e < (uint32_t)A.d) q[(int64_t)i * A.ld + e] = __uint_as_float(in[2 * m + 1]);
}

// after k_wire_zero; the mask is the bitmap of the last step (the draw a receiver repeats
// from the shared seed).  grid n, block 1024, dynamic LDS = bitmap_words words
__global__ __launch_bounds__(1024) void k_unpack_randk(WireArgs A, const uint32_t* msg, float* q) {
  extern __shared__ uint32_t pre[];
  __shared__ uint32_t sh_wave[16];
  const int i = blockIdx.x;
  bitmap_prefix(A, i, pre, sh_wave);
  const uint32_t* bm = A.bitmap + (int64_t)i * A.bitmap_words;
  const uint32_t* in = msg + (int64_t)i * A.words;
  for (int64_t w = threadIdx.x; w < A.bitmap_words; w += 1024) {
    uint32_t bits = bm[w];
    uint32_t rank = pre[w];
    while (bits) {
      const int j = __ffs((int)bits) - 1;
      bits &= bits - 1;
      q[(int64_t)i * A.ld + 32 * w + j] = __uint_as_float(in[rank++]);
    }
  }
}

// ---- random_a without a bitmap built by the select: ranks from the bit map in global memory ----

// Set (or clear the words of) the bits of the entries kept in the last step.  grid (ceil(k / 256), n)
__global__ __launch_bounds__(256) void k_wire_mark(WireArgs A, int set) {
  const int i = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= A.k) return;
  const uint32_t e = (uint32_t)A.sel_idx[(int64_t)i * A.k + m];
  uint32_t* word = A.keptmap + (int64_t)i * A.map_words + (e >> 5);
  if (set) atomicOr(word, 1u << (e & 31u));
  else *word = 0u;
}

// chunk_rank[i][c] = marked entries of worker i in chunk c (1024 entries = 32 words of the map).
// Eight chunks per block, a word per thread.  grid (ceil(nchunk / 8), n), block 256
__global__ __launch_bounds__(256) void k_wire_chunk_counts(WireArgs A) {
  const int i = blockIdx.y;
  const int64_t chunk = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
  const int64_t w = chunk * 32 + (threadIdx.x & 31);
  uint32_t c = (chunk < A.nchunk && w < A.map_words) ? (uint32_t)__popc(A.keptmap[(int64_t)i * A.map_words + w]) : 0u;
#pragma unroll
  for (int off = 16; off >= 1; off >>= 1) c += __shfl_xor(c, off, 64);   // stays inside the 32 lanes of a chunk
  if ((threadIdx.x & 31) == 0 && chunk < A.nchunk) A.chunk_rank[(int64_t)i * A.nchunk + chunk] = c;
}

// In place: chunk_rank[i][c] = marked entries of worker i in the chunks before c.  grid n, block 1024
__global__ __launch_bounds__(1024) void k_wire_chunk_scan(WireArgs A) {
  __shared__ uint32_t sh_wave[16];
  __shared__ uint32_t sh_carry;
  uint32_t* r = A.chunk_rank + (int64_t)blockIdx.x * A.nchunk;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) sh_carry = 0;
  __syncthreads();
  for (int64_t base = 0; base < A.nchunk; base += 1024) {
    const int64_t c = base + tid;
    const uint32_t mine = c < A.nchunk ? r[c] : 0u;
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    if (lane == 63) sh_wave[wave] = incl;
    __syncthreads();
    uint32_t before = sh_carry;
    for (int w = 0; w < wave; ++w) before += sh_wave[w];
    if (c < A.nchunk) r[c] = before + incl - mine;
    __syncthreads();
    if (tid == 1023) sh_carry = before + incl;
    __syncthreads();
  }
}

// Rank of kept entry e of worker i among the worker's kept entries; all 64 lanes of a wave
// call it with the same e and get the same result (they share the words of e's chunk).
__device__ __forceinline__ uint32_t rank_by_map(const WireArgs& A, int i, int64_t e) {
  const int lane = threadIdx.x & 63;
  const int64_t chunk = e >> 10;
  const int64_t w = chunk * 32 + lane, we = e >> 5;
  uint32_t c = 0;
  if (lane < 32 && w <= we) {
    uint32_t bits = A.keptmap[(int64_t)i * A.map_words + w];
    if (w == we) bits &= (1u << ((uint32_t)e & 31u)) - 1u;
    c = (uint32_t)__popc(bits);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off, 64);
  return A.chunk_rank[(int64_t)i * A.nchunk + chunk] + c;
}

// The value of kept entry e goes to position rank(e).  One wave per kept entry:
// grid (ceil(k / 4), n), block 256
__global__ __launch_bounds__(256) void k_pack_randk_ranked(WireArgs A, uint32_t* msg) {
  const int i = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= A.k) return;
  const int64_t e = A.sel_idx[(int64_t)i * A.k + m];
  const uint32_t rank = rank_by_map(A, i, e);
  if ((threadIdx.x & 63) == 0) msg[(int64_t)i * A.words + rank] = __float_as_uint(A.sel_val[(int64_t)i * A.k + m]);
}

// after k_wire_zero; the mask is the kept-index list of the last step (the draw a receiver
// repeats from the shared seed).  grid (ceil(k / 4), n), block 256
__global__ __launch_bounds__(256) void k_unpack_randk_ranked(WireArgs A, const uint32_t* msg, float* q) {
  const int i = blockIdx.y;
  const int64_t m = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= A.k) return;
  const int64_t e = A.sel_idx[(int64_t)i * A.k + m];
  const uint32_t rank = rank_by_map(A, i, e);
  if ((threadIdx.x & 63) == 0) q[(int64_t)i * A.ld + e] = __uint_as_float(msg[(int64_t)i * A.words + rank]);
}

}  // namespace choco
