// CPU oracle for the CHOCO-Gossip / CHOCO-SGD step.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
// statement of what one iteration computes.  It shares no code, header, table
// or helper with the HIP library and must never be called from the product
// path; only the tests, the smoke check and the benchmark's CPU-baseline leg
// load it.
//
// What follows the paper and what is a reading of it:
//   * Algorithm 1 (CHOCO-SGD): its mixing, compression, exchange and local
//     gradient steps, and the matrix form of
//     CHOCO-Gossip in Appendix A ("Example: CHOCO-SGD"):
//         X+ = X + gamma * Xhat (W - I),   Xhat+ = Xhat + Q(X+ - Xhat).
//   * Appendix C (compression schemes): gsgd_b, random_a, top_a, sign.
//   * Assumption 1 (mixing matrix W: symmetric, doubly stochastic).
//   * Assumption 3 / Lyapunov function Psi, and the consensus distance of
//     Section 5 (1/n sum_i ||x_i - xbar||^2) for the metrics.
//   Readings where the paper is silent (tie-breaking, sgn(0), the sampler for
//   random_a, the dither generator, reduction order) are stated at each
//   function.
//
// Parity pins: every function below is pinned by tests/test_oracle_*.py
// against closed forms, invariants and brute force, except the trajectories
// of the five synthetic workloads, for which the paper prints no numbers:
// those are "parity unpinned" and only checked through the invariants.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -shared -fPIC (see build.py).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum Compressor { Q_IDENTITY = 0, Q_TOPK = 1, Q_RANDK = 2, Q_SIGN = 3, Q_QSGD = 4 };
enum Order { ORDER_COMPRESS_THEN_MIX = 0, ORDER_MIX_THEN_COMPRESS = 1 };
enum MixForm { MIX_INCREMENTAL_S = 0, MIX_DIRECT = 1 };
enum Stream { STREAM_RANDK = 1, STREAM_DITHER = 2 };

// ---------------------------------------------------------------------------
// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
// numbers: as easy as 1, 2, 3", SC'11).  The paper only asks for a shared
// seed (Appendix C, random_a); the generator is this build's choice.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// One 32-bit random word for coordinate e of worker i at step t on a stream.
// Counter = (e / 4, i, low 32 bits of t, stream | high bits of t << 8),
// key = the two halves of the seed; the word used is number (e mod 4).
uint32_t random_word(uint64_t seed, uint64_t t, int worker, int64_t e, int stream) {
  uint32_t ctr[4], key[2], out[4];
  ctr[0] = (uint32_t)((uint64_t)e >> 2);
  ctr[1] = (uint32_t)worker;
  ctr[2] = (uint32_t)(t & 0xFFFFFFFFu);
  ctr[3] = (uint32_t)stream | ((uint32_t)(t >> 32) << 8);
  key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
  key[1] = (uint32_t)(seed >> 32);
  philox4x32_10(ctr, key, out);
  return out[e & 3];
}

// ---------------------------------------------------------------------------
// Canonical fp64 sum of d non-negative terms.  The paper does not say how
// ||v||_1 and ||v||_2 are accumulated; because the quantisation levels and
// the sign scale depend on every bit of the norm, both sides of the parity
// test use this fixed three-level tree:
//   level 1: chunks of 256 consecutive terms; "lane" l (0..63) adds its four
//            consecutive terms 4l..4l+3 left to right; the 64 lane sums are
//            combined by halving: for off = 32,16,..,1: t[l] += t[l+off], l<off;
//   level 2: groups of 16 consecutive chunk sums (4096 terms), combined by
//            halving from 8 to 1;
//   level 3: 256 "lanes"; lane l adds group sums l, l+256, l+512, ... in that
//            order; the 256 lane sums are combined by halving from 128 to 1.
// Terms, chunks and groups past the end count as +0.0 (an exact no-op on
// non-negative sums).
// ---------------------------------------------------------------------------
template <class Term>
double canonical_sum(int64_t d, Term term) {
  const int64_t nchunks = (d + 255) / 256;
  const int chunks_per_group = 16;
  const int64_t ngroups = (nchunks + chunks_per_group - 1) / chunks_per_group;
  std::vector<double> group_sum((size_t)ngroups);
  for (int64_t g = 0; g < ngroups; ++g) {
    double chunk[chunks_per_group];
    for (int k = 0; k < chunks_per_group; ++k) {
      const int64_t c = g * chunks_per_group + k;
      double lane[64];
      for (int l = 0; l < 64; ++l) {
        double acc = 0.0;
        for (int m = 0; m < 4; ++m) {
          const int64_t e = c * 256 + 4 * l + m;
          const double a = (e < d) ? term(e) : 0.0;
          acc = (m == 0) ? a : acc + a;
        }
        lane[l] = acc;
      }
      for (int off = 32; off >= 1; off >>= 1)
        for (int l = 0; l < off; ++l) lane[l] = lane[l] + lane[l + off];
      chunk[k] = lane[0];
    }
    for (int off = chunks_per_group / 2; off >= 1; off >>= 1)
      for (int k = 0; k < off; ++k) chunk[k] = chunk[k] + chunk[k + off];
    group_sum[(size_t)g] = chunk[0];
  }
  double lane3[256];
  for (int l = 0; l < 256; ++l) {
    double acc = 0.0;
    bool first = true;
    for (int64_t g = l; g < ngroups; g += 256) {
      acc = first ? group_sum[(size_t)g] : acc + group_sum[(size_t)g];
      first = false;
    }
    lane3[l] = acc;
  }
  for (int off = 128; off >= 1; off >>= 1)
    for (int l = 0; l < off; ++l) lane3[l] = lane3[l] + lane3[l + off];
  return lane3[0];
}

// ---------------------------------------------------------------------------
// Compression operators, Appendix C.  All take v (length d) and write the
// dense q = Q(v) (length d).  Optional side outputs, used for bit-exact
// parity of the discrete decisions:
//   sel    (k entries)  ascending indices kept by top_a / random_a
//   codes  (d entries)  sign: +1/-1;  gsgd: sig(v) * level
//   scal   (4 entries)  sign: {L1, c, 0, 0};  gsgd: {sum v^2, ||v||_2, r, step}
// ---------------------------------------------------------------------------
struct QParams {
  int compressor;
  int64_t k;        // top_a / random_a: number of kept coordinates, floor(a d)
  int levels;       // gsgd_b: s = 2^(b-1)
  int qsgd_biased;  // 1: divide by tau (biased version);  0: unbiased version
  int randk_rescale;// 0: x .* u (biased version);  1: (d/k) x .* u (unbiased)
  uint64_t seed;
};

// top_a: keep the k entries of largest magnitude (Appendix C, top_a).  The
// paper admits any permutation sorting |v| in non-increasing order; the
// reading here orders equal magnitudes by ascending index, so the kept set is
// unique: the k largest under (|v| descending, index ascending).
template <class R>
void select_topk(int64_t d, const R* v, int64_t k, std::vector<int32_t>& sel) {
  std::vector<int32_t> order((size_t)d);
  for (int64_t e = 0; e < d; ++e) order[(size_t)e] = (int32_t)e;
  auto before = [v](int32_t a, int32_t b) {
    const R ma = std::fabs(v[a]), mb = std::fabs(v[b]);
    if (ma != mb) return ma > mb;
    return a < b;
  };
  if (k < d) std::nth_element(order.begin(), order.begin() + k, order.end(), before);
  sel.assign(order.begin(), order.begin() + k);
  std::sort(sel.begin(), sel.end());
}

// random_a: a mask with exactly k ones, uniform over all such masks
// (Appendix C, random_a), reproducible from a shared seed.  The sampler is
// this build's choice: every coordinate draws a 32-bit word and the k
// smallest words win, equal words ordered by ascending index.
void select_randk(int64_t d, int64_t k, uint64_t seed, uint64_t t, int worker,
                  std::vector<int32_t>& sel, int64_t e0 = 0) {
  std::vector<uint32_t> r((size_t)d);
  for (int64_t e = 0; e < d; ++e) r[(size_t)e] = random_word(seed, t, worker, e0 + e, STREAM_RANDK);
  std::vector<int32_t> order((size_t)d);
  for (int64_t e = 0; e < d; ++e) order[(size_t)e] = (int32_t)e;
  auto before = [&r](int32_t a, int32_t b) {
    if (r[(size_t)a] != r[(size_t)b]) return r[(size_t)a] < r[(size_t)b];
    return a < b;
  };
  if (k < d) std::nth_element(order.begin(), order.begin() + k, order.end(), before);
  sel.assign(order.begin(), order.begin() + k);
  std::sort(sel.begin(), sel.end());
}

// e0 is the index that v[0] has in the worker's whole vector: the random word of
// entry e of v is the one of coordinate e0 + e (e0 = 0 unless v is one layer of it).
template <class R>
void compress(const QParams& P, int64_t d, const R* v, uint64_t t, int worker, R* q,
              int32_t* sel_out, int32_t* codes, double* scal, int64_t e0 = 0) {
  if (scal) scal[0] = scal[1] = scal[2] = scal[3] = 0.0;
  switch (P.compressor) {
    case Q_IDENTITY: {
      for (int64_t e = 0; e < d; ++e) q[e] = v[e];
      break;
    }
    case Q_TOPK:
    case Q_RANDK: {
      std::vector<int32_t> sel;
      if (P.compressor == Q_TOPK) select_topk(d, v, P.k, sel);
      else select_randk(d, P.k, P.seed, t, worker, sel, e0);
      for (int64_t e = 0; e < d; ++e) q[e] = (R)0;
      const bool rescale = (P.compressor == Q_RANDK) && P.randk_rescale;
      const R scale = (R)((double)d / (double)P.k);
      for (size_t m = 0; m < sel.size(); ++m) {
        const int32_t e = sel[m];
        q[e] = rescale ? scale * v[e] : v[e];
        if (sel_out) sel_out[m] = e;
      }
      break;
    }
    case Q_SIGN: {
      // sign(v) = (||v||_1 / d) sgn(v)  (Appendix C, sign).  One bit per
      // entry cannot carry a zero, so sgn is read as: -1 if v < 0, else +1.
      const double l1 = canonical_sum(d, [v](int64_t e) { return std::fabs((double)v[e]); });
      const R c = (R)(l1 / (double)d);
      for (int64_t e = 0; e < d; ++e) {
        const bool neg = v[e] < (R)0;
        q[e] = neg ? -c : c;
        if (codes) codes[e] = neg ? -1 : 1;
      }
      if (scal) { scal[0] = l1; scal[1] = (double)c; }
      break;
    }
    case Q_QSGD: {
      // gsgd_b(v) = ||v||_2 / tau * sig(v) * (1/s) * floor(s |v| / ||v||_2 + u),
      // s = 2^(b-1), tau = 1 + min(d / s^2, sqrt(d) / s) in the biased version
      // and tau = 1 in the unbiased one (Appendix C, gsgd_b); sig(0) = +1.
      // u is 24 random bits scaled into [0, 1).  A zero vector maps to zero.
      const double l2sq = canonical_sum(d, [v](int64_t e) { return (double)v[e] * (double)v[e]; });
      const double nrm = std::sqrt(l2sq);
      const double s = (double)P.levels;
      double tau = 1.0;
      if (P.qsgd_biased) tau = 1.0 + std::min((double)d / (s * s), std::sqrt((double)d) / s);
      R r = (R)0, step = (R)0;
      if (nrm > 0.0) {
        r = (R)(s / nrm);
        step = (R)(nrm / (tau * s));
      }
      for (int64_t e = 0; e < d; ++e) {
        const bool neg = v[e] < (R)0;
        int32_t level = 0;
        if (nrm > 0.0) {
          const uint32_t word = random_word(P.seed, t, worker, e0 + e, STREAM_DITHER);
          const R u = (R)(word >> 8) * (R)(1.0 / 16777216.0);
          const R a = std::fabs(v[e]) * r;
          level = (int32_t)std::floor(a + u);
        }
        const R mag = (R)level * step;
        q[e] = neg ? -mag : mag;
        if (codes) codes[e] = neg ? -level : level;
      }
      if (scal) { scal[0] = l2sq; scal[1] = nrm; scal[2] = (double)r; scal[3] = (double)step; }
      break;
    }
  }
}

// ---------------------------------------------------------------------------
// One CHOCO-Gossip step for all n workers (Algorithm 1 without its gradient step).
//   X, Xhat, S: n x d row-major.  S_i = sum_j w_ij xhat_j is the third vector
//   a node keeps (Section 3, remark after Algorithm 1); it is only read and
//   written when mix_form == MIX_INCREMENTAL_S.
//   W: CSR with the self-loop stored explicitly, columns ascending in a row.
// Order of the two halves:
//   ORDER_MIX_THEN_COMPRESS  Algorithm 1 as printed: the mixing step, then compression and exchange.
//   ORDER_COMPRESS_THEN_MIX  compression and exchange first, then the mixing step with the new xhat.
// Mix forms (same mathematics, different fp rounding):
//   MIX_DIRECT         acc = sum_p w_p (xhat_j - xhat_i) in CSR order from 0;
//                      x_i += gamma * acc                       (the mixing step as printed)
//   MIX_INCREMENTAL_S  s_i += w_p q_j in CSR order (only kept entries of q_j
//                      for the sparsifying operators); x_i += gamma (s_i - xhat_i),
//                      valid because rows of W sum to one (Assumption 1).
// Every product and every sum is rounded on its own (no fused multiply-add).
// ---------------------------------------------------------------------------
template <class R>
void mix_half(int n, int64_t d, const int32_t* row_ptr, const int32_t* col_idx, const R* w,
              R gamma, int mix_form, R* X, const R* Xhat, const R* S) {
  for (int i = 0; i < n; ++i) {
    R* x = X + (int64_t)i * d;
    const R* xh = Xhat + (int64_t)i * d;
    if (mix_form == MIX_INCREMENTAL_S) {
      const R* s = S + (int64_t)i * d;
      for (int64_t e = 0; e < d; ++e) {
        const R diff = s[e] - xh[e];
        const R upd = gamma * diff;
        x[e] = x[e] + upd;
      }
    } else {
      for (int64_t e = 0; e < d; ++e) {
        R acc = (R)0;
        for (int32_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
          const R diff = Xhat[(int64_t)col_idx[p] * d + e] - xh[e];
          const R prod = w[p] * diff;
          acc = acc + prod;
        }
        const R upd = gamma * acc;
        x[e] = x[e] + upd;
      }
    }
  }
}

// Layers.  The experiments apply the operator to every layer of the network on its
// own (Section 5, set-up of the ResNet-20 runs): layer l is the slice
// [start[l], start[l] + len[l]) of a worker's vector and is compressed as a vector of
// its own, with len[l] in the place of d (norms, tau, d/k) and k[l] in the place of k.
// Slices are disjoint and ascending; entries that lie in no slice are never sent
// (q = 0 there).  k[l] = 0 sends nothing of layer l.  nseg = 0: the whole vector is
// the only layer.
struct Segments {
  int32_t nseg;
  const int64_t* start;
  const int64_t* len;
  const int64_t* k;   // used by top_a / random_a only
};

template <class R>
void compress_half(const QParams& P, const Segments& G, int n, int64_t d, const int32_t* row_ptr,
                   const int32_t* col_idx, const R* w, int mix_form, uint64_t t, const R* X,
                   R* Xhat, R* S, int32_t* sel_out, int32_t* codes, double* scal) {
  const bool sparse = (P.compressor == Q_TOPK || P.compressor == Q_RANDK);
  const int32_t nseg = G.nseg > 0 ? G.nseg : 1;
  const int64_t whole_start = 0, whole_len = d, whole_k = P.k;
  const int64_t* start = G.nseg > 0 ? G.start : &whole_start;
  const int64_t* len = G.nseg > 0 ? G.len : &whole_len;
  const int64_t* kk = G.nseg > 0 ? G.k : &whole_k;
  int64_t ktot = 0;   // kept entries per worker over all layers
  if (sparse) for (int32_t l = 0; l < nseg; ++l) ktot += kk[l];
  std::vector<R> Qall((size_t)n * (size_t)d, (R)0);
  std::vector<int32_t> sel_all((size_t)n * (size_t)ktot);
  std::vector<R> v((size_t)d);
  for (int i = 0; i < n; ++i) {  // compression: q_i = Q(x_i - xhat_i), layer by layer
    for (int64_t e = 0; e < d; ++e) v[(size_t)e] = X[(int64_t)i * d + e] - Xhat[(int64_t)i * d + e];
    int64_t filled = 0;
    for (int32_t l = 0; l < nseg; ++l) {
      double* sc = scal ? scal + 4 * ((int64_t)i * nseg + l) : nullptr;
      if (sparse && kk[l] == 0) {
        if (sc) sc[0] = sc[1] = sc[2] = sc[3] = 0.0;
        continue;
      }
      QParams Pl = P;
      Pl.k = kk[l];
      int32_t* sel_l = sparse ? sel_all.data() + (int64_t)i * ktot + filled : nullptr;
      compress<R>(Pl, len[l], v.data() + start[l], t, i, Qall.data() + (int64_t)i * d + start[l],
                  sel_l, codes ? codes + (int64_t)i * d + start[l] : nullptr, sc, start[l]);
      if (sparse) {
        for (int64_t m = 0; m < kk[l]; ++m) sel_l[m] += (int32_t)start[l];
        filled += kk[l];
      }
    }
  }
  if (sparse && sel_out && ktot > 0) std::memcpy(sel_out, sel_all.data(), sel_all.size() * sizeof(int32_t));
  for (int j = 0; j < n; ++j) {  // exchange: xhat_j += q_j (one copy stands for all replicas)
    R* xh = Xhat + (int64_t)j * d;
    const R* q = Qall.data() + (int64_t)j * d;
    if (sparse) {
      for (int64_t m = 0; m < ktot; ++m) {
        const int32_t e = sel_all[(size_t)((int64_t)j * ktot + m)];
        xh[e] = xh[e] + q[e];
      }
    } else {
      for (int32_t l = 0; l < nseg; ++l)
        for (int64_t e = start[l]; e < start[l] + len[l]; ++e) xh[e] = xh[e] + q[e];
    }
  }
  if (mix_form == MIX_INCREMENTAL_S) {  // s_i += sum_j w_ij q_j, CSR order
    for (int i = 0; i < n; ++i) {
      R* s = S + (int64_t)i * d;
      for (int32_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
        const int j = col_idx[p];
        const R* q = Qall.data() + (int64_t)j * d;
        if (sparse) {
          for (int64_t m = 0; m < ktot; ++m) {
            const int32_t e = sel_all[(size_t)((int64_t)j * ktot + m)];
            const R prod = w[p] * q[e];
            s[e] = s[e] + prod;
          }
        } else {
          for (int32_t l = 0; l < nseg; ++l)
            for (int64_t e = start[l]; e < start[l] + len[l]; ++e) {
              const R prod = w[p] * q[e];
              s[e] = s[e] + prod;
            }
        }
      }
    }
  }
}

bool segments_ok(const Segments& G, int64_t d, bool sparse) {
  int64_t end = 0;
  for (int32_t l = 0; l < G.nseg; ++l) {
    if (G.start[l] < end || G.len[l] < 1) return false;
    end = G.start[l] + G.len[l];
    if (end > d) return false;
    if (sparse && (G.k[l] < 0 || G.k[l] > G.len[l])) return false;
  }
  return true;
}

template <class R>
int gossip_step(int n, int64_t d, const int32_t* row_ptr, const int32_t* col_idx, const R* w,
                R gamma, const QParams& P, const Segments& G, int order, int mix_form, uint64_t t,
                R* X, R* Xhat, R* S, int32_t* sel_out, int32_t* codes, double* scal) {
  if (n < 1 || d < 1) return -1;
  const bool sparse = (P.compressor == Q_TOPK || P.compressor == Q_RANDK);
  if (G.nseg == 0 && sparse && (P.k < 1 || P.k > d)) return -1;
  if (G.nseg < 0 || (G.nseg > 0 && !segments_ok(G, d, sparse))) return -1;
  if (P.compressor == Q_QSGD && P.levels < 1) return -1;
  if (order == ORDER_MIX_THEN_COMPRESS) {
    mix_half<R>(n, d, row_ptr, col_idx, w, gamma, mix_form, X, Xhat, S);
    compress_half<R>(P, G, n, d, row_ptr, col_idx, w, mix_form, t, X, Xhat, S, sel_out, codes, scal);
  } else {
    compress_half<R>(P, G, n, d, row_ptr, col_idx, w, mix_form, t, X, Xhat, S, sel_out, codes, scal);
    mix_half<R>(n, d, row_ptr, col_idx, w, gamma, mix_form, X, Xhat, S);
  }
  return 0;
}

// ---------------------------------------------------------------------------
// Messages on the wire (Appendix C, the message size stated with each operator;
// entries are float32 there, so this part exists for float only).
//
// paper_message_bits: the sizes as the paper counts them:
//   sign      d + 32           one bit per entry and 32 bits for the norm
//   top_a     2 * 32 * k       values and positions
//   random_a  32 * k           values only, the mask follows from the shared seed
//   gsgd_b    b * d + 32       b = log2(s) + 1 bits per entry (the paper does not
//                              count the norm; 32 bits are added for it here)
//   identity  32 * d
// The byte layout is this build's choice (the paper fixes none); 32-bit
// little-endian words, W = ceil(d / 32):
//   sign      [c as float][W words: bit e%32 of word e/32 set iff the entry is -c]
//   gsgd      [step as float][4 words: ascending indices of entries whose level does
//             not fit the magnitude bits, 0xFFFFFFFF when unused][plane 0: the signs of
//             the entries with a non-zero level (a zero is sent as +0), W words][planes 1..mb: bit p-1 of min(level, 2^mb - 1), W words each],
//             mb = bit length of s - 1 (at least 1).  With s = 2^(b-1) that is b bits
//             per entry as the paper counts; the level s itself, which the formula
//             reaches for the few entries that hold almost the whole norm although
//             the text lists the levels as 0..s-1, goes through the index slots.
//   top_a     k pairs [index][value as float], ascending index
//   random_a  k values as float in ascending order of index; the receiver draws the
//             same mask from (seed, step, sender)
//   identity  d floats
// ---------------------------------------------------------------------------
int magnitude_bits(int levels) {
  int mb = 0;
  for (int x = levels - 1; x > 0; x >>= 1) ++mb;
  return mb < 1 ? 1 : mb;
}

int64_t paper_message_bits(int compressor, int64_t d, int64_t k, int levels) {
  switch (compressor) {
    case Q_IDENTITY: return 32 * d;
    case Q_TOPK: return 64 * k;
    case Q_RANDK: return 32 * k;
    case Q_SIGN: return d + 32;
    case Q_QSGD: {
      int b = 1;
      for (int x = levels; x > 1; x >>= 1) ++b;   // s = 2^(b-1)
      return (int64_t)b * d + 32;
    }
  }
  return -1;
}

constexpr int kOverflowSlots = 4;

int64_t message_words(int compressor, int64_t d, int64_t k, int levels) {
  const int64_t W = (d + 31) / 32;
  switch (compressor) {
    case Q_IDENTITY: return d;
    case Q_TOPK: return 2 * k;
    case Q_RANDK: return k;
    case Q_SIGN: return 1 + W;
    case Q_QSGD: return 1 + kOverflowSlots + (int64_t)(1 + magnitude_bits(levels)) * W;
  }
  return -1;
}

uint32_t float_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, sizeof u);
  return u;
}
float bits_float(uint32_t u) {
  float f;
  std::memcpy(&f, &u, sizeof f);
  return f;
}

// q = Q(v) and its message.  Returns 0, or -2 if more entries than there are slots
// carry a level that does not fit the magnitude bits.
int pack_message(const QParams& P, int64_t d, const float* v, uint64_t t, int worker, float* q,
                 uint32_t* msg, int64_t e0 = 0) {
  std::vector<int32_t> sel((size_t)(P.compressor == Q_TOPK || P.compressor == Q_RANDK ? P.k : 0));
  std::vector<int32_t> codes((size_t)d, 0);
  double scal[4];
  compress<float>(P, d, v, t, worker, q, sel.empty() ? nullptr : sel.data(), codes.data(), scal, e0);
  const int64_t W = (d + 31) / 32;
  const int64_t words = message_words(P.compressor, d, P.k, P.levels);
  for (int64_t j = 0; j < words; ++j) msg[j] = 0;
  switch (P.compressor) {
    case Q_IDENTITY:
      for (int64_t e = 0; e < d; ++e) msg[e] = float_bits(q[e]);
      break;
    case Q_TOPK:
      for (int64_t m = 0; m < P.k; ++m) {
        msg[2 * m] = (uint32_t)sel[(size_t)m];
        msg[2 * m + 1] = float_bits(q[sel[(size_t)m]]);
      }
      break;
    case Q_RANDK:
      for (int64_t m = 0; m < P.k; ++m) msg[m] = float_bits(q[sel[(size_t)m]]);
      break;
    case Q_SIGN:
      msg[0] = float_bits((float)scal[1]);
      for (int64_t e = 0; e < d; ++e)
        if (codes[(size_t)e] < 0) msg[1 + e / 32] |= 1u << (e % 32);
      break;
    case Q_QSGD: {
      const int mb = magnitude_bits(P.levels);
      const int32_t maxmag = (1 << mb) - 1;
      msg[0] = float_bits((float)scal[3]);
      for (int j = 0; j < kOverflowSlots; ++j) msg[1 + j] = 0xFFFFFFFFu;
      int used = 0;
      uint32_t* planes = msg + 1 + kOverflowSlots;
      for (int64_t e = 0; e < d; ++e) {
        const bool neg = codes[(size_t)e] < 0;   // a zero level carries no sign
        int32_t level = std::abs(codes[(size_t)e]);
        if (level > maxmag) {
          if (used == kOverflowSlots) return -2;
          msg[1 + used++] = (uint32_t)e;
          level = maxmag;
        }
        if (neg) planes[e / 32] |= 1u << (e % 32);
        for (int p = 0; p < mb; ++p)
          if ((level >> p) & 1) planes[(int64_t)(1 + p) * W + e / 32] |= 1u << (e % 32);
      }
      break;
    }
  }
  return 0;
}

// The receiver's side: q from the message alone (plus the shared seed, the step and the
// sender for random_a).
void unpack_message(const QParams& P, int64_t d, uint64_t t, int worker, const uint32_t* msg,
                    float* q, int64_t e0 = 0) {
  const int64_t W = (d + 31) / 32;
  for (int64_t e = 0; e < d; ++e) q[e] = 0.0f;
  switch (P.compressor) {
    case Q_IDENTITY:
      for (int64_t e = 0; e < d; ++e) q[e] = bits_float(msg[e]);
      break;
    case Q_TOPK:
      for (int64_t m = 0; m < P.k; ++m) q[msg[2 * m]] = bits_float(msg[2 * m + 1]);
      break;
    case Q_RANDK: {
      std::vector<int32_t> sel;
      select_randk(d, P.k, P.seed, t, worker, sel, e0);
      for (int64_t m = 0; m < P.k; ++m) q[sel[(size_t)m]] = bits_float(msg[m]);
      break;
    }
    case Q_SIGN: {
      const float c = bits_float(msg[0]);
      for (int64_t e = 0; e < d; ++e) q[e] = ((msg[1 + e / 32] >> (e % 32)) & 1u) ? -c : c;
      break;
    }
    case Q_QSGD: {
      const int mb = magnitude_bits(P.levels);
      const float step = bits_float(msg[0]);
      const uint32_t* planes = msg + 1 + kOverflowSlots;
      for (int64_t e = 0; e < d; ++e) {
        int32_t level = 0;
        for (int p = 0; p < mb; ++p)
          level |= (int32_t)((planes[(int64_t)(1 + p) * W + e / 32] >> (e % 32)) & 1u) << p;
        for (int j = 0; j < kOverflowSlots; ++j)
          if (msg[1 + j] == (uint32_t)e) level = P.levels;
        const float mag = (float)level * step;
        q[e] = ((planes[e / 32] >> (e % 32)) & 1u) ? -mag : mag;
      }
      break;
    }
  }
}

// Layer by layer (Section 5): a worker's message is the messages of its layers one after
// the other, each with its own scale / step / index slots and its own word padding;
// positions in top_a pairs count in the whole vector.  A layer with k = 0 sends nothing.
int64_t layer_message_words(const QParams& P, const Segments& G, int32_t l) {
  const bool sparse = (P.compressor == Q_TOPK || P.compressor == Q_RANDK);
  if (sparse && G.k[l] == 0) return 0;
  return message_words(P.compressor, G.len[l], sparse ? G.k[l] : 0, P.levels);
}

int pack_layers(const QParams& P, const Segments& G, int64_t d, const float* v, uint64_t t, int worker,
                float* q, uint32_t* msg) {
  const bool sparse = (P.compressor == Q_TOPK || P.compressor == Q_RANDK);
  for (int64_t e = 0; e < d; ++e) q[e] = 0.0f;
  int64_t off = 0;
  for (int32_t l = 0; l < G.nseg; ++l) {
    const int64_t words = layer_message_words(P, G, l);
    if (words == 0) continue;
    QParams Pl = P;
    Pl.k = sparse ? G.k[l] : 0;
    const int rc = pack_message(Pl, G.len[l], v + G.start[l], t, worker, q + G.start[l], msg + off, G.start[l]);
    if (rc != 0) return rc;
    if (P.compressor == Q_TOPK)
      for (int64_t m = 0; m < Pl.k; ++m) msg[off + 2 * m] += (uint32_t)G.start[l];
    off += words;
  }
  return 0;
}

void unpack_layers(const QParams& P, const Segments& G, int64_t d, uint64_t t, int worker,
                   const uint32_t* msg, float* q) {
  const bool sparse = (P.compressor == Q_TOPK || P.compressor == Q_RANDK);
  for (int64_t e = 0; e < d; ++e) q[e] = 0.0f;
  int64_t off = 0;
  for (int32_t l = 0; l < G.nseg; ++l) {
    const int64_t words = layer_message_words(P, G, l);
    if (words == 0) continue;
    QParams Pl = P;
    Pl.k = sparse ? G.k[l] : 0;
    if (P.compressor == Q_TOPK) {
      for (int64_t m = 0; m < Pl.k; ++m) q[msg[off + 2 * m]] = bits_float(msg[off + 2 * m + 1]);
    } else {
      unpack_message(Pl, G.len[l], t, worker, msg + off, q + G.start[l], G.start[l]);
    }
    off += words;
  }
}

// Algorithm 1, local gradient step: x_i <- x_i - eta g_i  (product rounded, then the difference).
template <class R>
void sgd_step(int n, int64_t d, R* X, const R* G, R lr) {
  for (int64_t a = 0; a < (int64_t)n * d; ++a) {
    const R prod = lr * G[a];
    X[a] = X[a] - prod;
  }
}

// Algorithm 2, momentum and local step: v <- (g + lambda x) + beta v;  x <- x - eta v.
template <class R>
void momentum_step(int n, int64_t d, R* X, R* V, const R* G, R lr, R beta, R lambda) {
  for (int64_t a = 0; a < (int64_t)n * d; ++a) {
    const R wd = lambda * X[a];
    const R gg = G[a] + wd;
    const R bv = beta * V[a];
    V[a] = gg + bv;
    const R prod = lr * V[a];
    X[a] = X[a] - prod;
  }
}

// Consensus distance (1/n) sum_i ||x_i - xbar||^2 (Section 5), ||xbar||_2, and
// Psi = ||X - Xbar||_F^2 + ||X - Xhat||_F^2 (Assumption 3), all in fp64.
template <class R>
void metrics(int n, int64_t d, const R* X, const R* Xhat, double* consensus, double* mean_norm,
             double* psi) {
  double dev = 0.0, mn = 0.0, gap = 0.0;
  for (int64_t e = 0; e < d; ++e) {
    double mean = 0.0;
    for (int i = 0; i < n; ++i) mean += (double)X[(int64_t)i * d + e];
    mean /= (double)n;
    mn += mean * mean;
    for (int i = 0; i < n; ++i) {
      const double a = (double)X[(int64_t)i * d + e] - mean;
      dev += a * a;
      if (Xhat) {
        const double b = (double)X[(int64_t)i * d + e] - (double)Xhat[(int64_t)i * d + e];
        gap += b * b;
      }
    }
  }
  if (consensus) *consensus = dev / (double)n;
  if (mean_norm) *mean_norm = std::sqrt(mn);
  if (psi) *psi = dev + gap;
}

}  // namespace

extern "C" {

void choco_ref_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

uint32_t choco_ref_random_word(uint64_t seed, uint64_t t, int32_t worker, int64_t e,
                               int32_t stream) {
  return random_word(seed, t, worker, e, stream);
}

double choco_ref_canonical_sum(int64_t d, const double* terms) {
  return canonical_sum(d, [terms](int64_t e) { return terms[e]; });
}

#define CHOCO_REF_DEFINE(SUFFIX, R)                                                               \
  int choco_ref_compress_##SUFFIX(int32_t compressor, int64_t d, const R* v, int64_t k,           \
                                  int32_t levels, int32_t qsgd_biased, int32_t randk_rescale,     \
                                  uint64_t seed, uint64_t t, int32_t worker, R* q, int32_t* sel,  \
                                  int32_t* codes, double* scal) {                                 \
    QParams P{compressor, k, levels, qsgd_biased, randk_rescale, seed};                           \
    if (d < 1) return -1;                                                                         \
    if ((compressor == Q_TOPK || compressor == Q_RANDK) && (k < 1 || k > d)) return -1;           \
    if (compressor == Q_QSGD && levels < 1) return -1;                                            \
    compress<R>(P, d, v, t, worker, q, sel, codes, scal);                                         \
    return 0;                                                                                     \
  }                                                                                               \
  int choco_ref_gossip_step_##SUFFIX(                                                             \
      int32_t n, int64_t d, const int32_t* row_ptr, const int32_t* col_idx, const R* w, R gamma,  \
      int32_t compressor, int64_t k, int32_t levels, int32_t qsgd_biased, int32_t randk_rescale,  \
      int32_t order, int32_t mix_form, uint64_t seed, uint64_t t, R* X, R* Xhat, R* S,            \
      int32_t* sel, int32_t* codes, double* scal) {                                               \
    QParams P{compressor, k, levels, qsgd_biased, randk_rescale, seed};                           \
    const Segments G{0, nullptr, nullptr, nullptr};                                               \
    return gossip_step<R>(n, d, row_ptr, col_idx, w, gamma, P, G, order, mix_form, t, X, Xhat, S, \
                          sel, codes, scal);                                                      \
  }                                                                                               \
  /* layer-wise: sel is n x sum(k), scal is n x nseg x 4 */                                       \
  int choco_ref_gossip_step_layers_##SUFFIX(                                                      \
      int32_t n, int64_t d, const int32_t* row_ptr, const int32_t* col_idx, const R* w, R gamma,  \
      int32_t compressor, int32_t nseg, const int64_t* seg_start, const int64_t* seg_len,         \
      const int64_t* seg_k, int32_t levels, int32_t qsgd_biased, int32_t randk_rescale,           \
      int32_t order, int32_t mix_form, uint64_t seed, uint64_t t, R* X, R* Xhat, R* S,            \
      int32_t* sel, int32_t* codes, double* scal) {                                               \
    if (nseg < 1) return -1;                                                                      \
    QParams P{compressor, 0, levels, qsgd_biased, randk_rescale, seed};                           \
    const Segments G{nseg, seg_start, seg_len, seg_k};                                            \
    return gossip_step<R>(n, d, row_ptr, col_idx, w, gamma, P, G, order, mix_form, t, X, Xhat, S, \
                          sel, codes, scal);                                                      \
  }                                                                                               \
  void choco_ref_sgd_step_##SUFFIX(int32_t n, int64_t d, R* X, const R* G, R lr) {                \
    sgd_step<R>(n, d, X, G, lr);                                                                  \
  }                                                                                               \
  void choco_ref_momentum_step_##SUFFIX(int32_t n, int64_t d, R* X, R* V, const R* G, R lr,       \
                                        R beta, R lambda) {                                       \
    momentum_step<R>(n, d, X, V, G, lr, beta, lambda);                                            \
  }                                                                                               \
  void choco_ref_metrics_##SUFFIX(int32_t n, int64_t d, const R* X, const R* Xhat,                \
                                  double* consensus, double* mean_norm, double* psi) {            \
    metrics<R>(n, d, X, Xhat, consensus, mean_norm, psi);                                         \
  }

int64_t choco_ref_paper_message_bits(int32_t compressor, int64_t d, int64_t k, int32_t levels) {
  return paper_message_bits(compressor, d, k, levels);
}

int64_t choco_ref_message_words(int32_t compressor, int64_t d, int64_t k, int32_t levels) {
  return message_words(compressor, d, k, levels);
}

int choco_ref_pack_message(int32_t compressor, int64_t d, const float* v, int64_t k, int32_t levels,
                           int32_t qsgd_biased, int32_t randk_rescale, uint64_t seed, uint64_t t,
                           int32_t worker, float* q, uint32_t* msg) {
  QParams P{compressor, k, levels, qsgd_biased, randk_rescale, seed};
  if (d < 1) return -1;
  if ((compressor == Q_TOPK || compressor == Q_RANDK) && (k < 1 || k > d)) return -1;
  if (compressor == Q_QSGD && levels < 1) return -1;
  return pack_message(P, d, v, t, worker, q, msg);
}

int choco_ref_unpack_message(int32_t compressor, int64_t d, int64_t k, int32_t levels,
                             int32_t qsgd_biased, int32_t randk_rescale, uint64_t seed, uint64_t t,
                             int32_t worker, const uint32_t* msg, float* q) {
  QParams P{compressor, k, levels, qsgd_biased, randk_rescale, seed};
  if (d < 1) return -1;
  unpack_message(P, d, t, worker, msg, q);
  return 0;
}

int64_t choco_ref_layers_message_words(int32_t compressor, int32_t nseg, const int64_t* seg_len,
                                       const int64_t* seg_k, int32_t levels) {
  QParams P{compressor, 0, levels, 1, 0, 0};
  const Segments G{nseg, nullptr, seg_len, seg_k};
  int64_t words = 0;
  for (int32_t l = 0; l < nseg; ++l) words += layer_message_words(P, G, l);
  return words;
}

int choco_ref_pack_layers(int32_t compressor, int64_t d, const float* v, int32_t nseg,
                          const int64_t* seg_start, const int64_t* seg_len, const int64_t* seg_k,
                          int32_t levels, int32_t qsgd_biased, int32_t randk_rescale, uint64_t seed,
                          uint64_t t, int32_t worker, float* q, uint32_t* msg) {
  QParams P{compressor, 0, levels, qsgd_biased, randk_rescale, seed};
  const Segments G{nseg, seg_start, seg_len, seg_k};
  const bool sparse = (compressor == Q_TOPK || compressor == Q_RANDK);
  if (nseg < 1 || !segments_ok(G, d, sparse)) return -1;
  return pack_layers(P, G, d, v, t, worker, q, msg);
}

int choco_ref_unpack_layers(int32_t compressor, int64_t d, int32_t nseg, const int64_t* seg_start,
                            const int64_t* seg_len, const int64_t* seg_k, int32_t levels,
                            int32_t qsgd_biased, int32_t randk_rescale, uint64_t seed, uint64_t t,
                            int32_t worker, const uint32_t* msg, float* q) {
  QParams P{compressor, 0, levels, qsgd_biased, randk_rescale, seed};
  const Segments G{nseg, seg_start, seg_len, seg_k};
  const bool sparse = (compressor == Q_TOPK || compressor == Q_RANDK);
  if (nseg < 1 || !segments_ok(G, d, sparse)) return -1;
  unpack_layers(P, G, d, t, worker, msg, q);
  return 0;
}

CHOCO_REF_DEFINE(f32, float)
CHOCO_REF_DEFINE(f64, double)

}  // extern "C"
