/*
 * choco.h - C ABI of the MI355X (gfx950) CHOCO-Gossip / CHOCO-SGD step.
 *
 * One context holds the state of all n simulated workers on one GPU:
 *   X     n x ld fp32, row i = private iterate x_i          (caller's buffer)
 *   Xhat  n x ld fp32, row i = public copy  xhat_i           (in the workspace)
 *   S     n x ld fp32, row i = sum_j w_ij xhat_j             (in the workspace)
 * following Algorithm 1 (CHOCO-SGD) of the paper and the remark after it that a
 * node needs three vectors.  "send q_i / receive q_j" (the exchange of Algorithm 1)
 * is plain device-memory traffic here because all replicas of xhat_j are equal.
 *
 * Conventions
 *   - every function returns CHOCO_OK (0) or a negative error code; nothing is
 *     printed, nothing aborts, no exception crosses the boundary;
 *   - pointers named *_dev are device pointers, *_host are host pointers;
 *   - device buffers are owned by the caller (allocated e.g. with torch); the
 *     library allocates no device memory, it only carves up the workspace;
 *   - work is enqueued on the caller's stream (one documented exception: the look-ahead
 *     selection of RANDK, see choco_set_lookahead) and the calls return without
 *     synchronising, except choco_metrics, choco_last_scalars, choco_layer_scalars,
 *     choco_profile_report, choco_sync and choco_last_message (when it returns a scale);
 *   - inputs must be finite; NaN/Inf give unspecified selections.
 */
#ifndef CHOCO_H
#define CHOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct choco_ctx choco_ctx; /* opaque, host memory, freed by choco_destroy */

enum {
  CHOCO_OK = 0,
  CHOCO_E_INVAL = -1,       /* bad argument (see choco_init)                        */
  CHOCO_E_NOMEM = -2,       /* workspace too small / host allocation failed         */
  CHOCO_E_HIP = -3,         /* HIP runtime error; see choco_last_hip_error          */
  CHOCO_E_UNSUPPORTED = -4  /* valid request this build does not implement          */
};

/* Compression operators Q of Appendix C ("Compression Schemes"). */
enum {
  CHOCO_Q_IDENTITY = 0, /* Q(v) = v: exact averaging (Appendix A, first example)    */
  CHOCO_Q_TOPK = 1,     /* top_a: keep the k entries of largest |v|; ties -> lower index */
  CHOCO_Q_RANDK = 2,    /* random_a: keep k entries chosen uniformly (Philox, k smallest words) */
  CHOCO_Q_SIGN = 3,     /* sign: (||v||_1 / d) * sgn(v), sgn = -1 iff v < 0          */
  CHOCO_Q_QSGD = 4      /* gsgd_b with s = 2^(b-1) levels and random dithering      */
};

/* Order of the two halves of one gossip step. */
enum {
  CHOCO_ORDER_COMPRESS_THEN_MIX = 0, /* compression and exchange, then the mixing step with the new xhat */
  CHOCO_ORDER_MIX_THEN_COMPRESS = 1  /* Algorithm 1 as printed: mixing step, then compression and exchange */
};

/* How the mixing step of Algorithm 1, x_i += gamma * sum_j w_ij (xhat_j - xhat_i), is evaluated. */
enum {
  CHOCO_MIX_AUTO = 0,          /* DIRECT for sign / gsgd / identity and, up to 64 workers, for
                                  top_a / random_a; INCREMENTAL_S for top_a / random_a with more
                                  workers, for top_a in the printed order and for layer tables in
                                  the printed order (choco_get_mix_form tells which)           */
  CHOCO_MIX_INCREMENTAL_S = 1, /* S_i += sum_j w_ij q_j (CSR order); x_i += gamma (S_i - xhat_i) */
  CHOCO_MIX_DIRECT = 2         /* acc = sum_j w_ij (xhat_j - xhat_i) in CSR order from 0    */
};

typedef struct {
  int32_t n;          /* number of workers, >= 1                                         */
  int64_t d;          /* coordinates per worker, 1 <= d <= CHOCO_MAX_D                   */
  int64_t ld;         /* row stride of X, G and the internal arrays in floats; 0 means d
                         rounded up to a multiple of 4.  Must be >= d and a multiple of 4;
                         a multiple of 64 (rows on 256-byte boundaries) streams fastest.
                         Columns d..ld-1 are never compressed, selected or sent         */
  /* Mixing matrix W of Assumption 1 as CSR.  HOST pointers, copied during choco_init.
     Row i lists the neighbours of i INCLUDING i itself (the exchange of Algorithm 1), columns
     strictly ascending.  W must be symmetric with non-negative entries and rows summing
     to 1, each to within 1e-6.  The values are used as given (never renormalised).      */
  const int32_t *row_ptr_host; /* n + 1 entries */
  const int32_t *col_idx_host; /* nnz entries   */
  const float *w_host;         /* nnz entries   */
  float gamma;           /* consensus stepsize of Algorithm 1, finite and > 0             */
  int32_t compressor;    /* CHOCO_Q_*                                                     */
  int64_t k;             /* TOPK / RANDK: kept coordinates floor(a d), 1 <= k <= d        */
  int32_t levels;        /* QSGD: s = 2^(b-1) >= 1                                        */
  int32_t qsgd_biased;   /* 1: scale by 1/tau (biased gsgd_b); 0: unbiased gsgd_b         */
  int32_t randk_rescale; /* 0: x .* u (biased random_a); 1: (d/k) x .* u (unbiased)       */
  int32_t order;         /* CHOCO_ORDER_*                                                 */
  int32_t mix_form;      /* CHOCO_MIX_*                                                   */
  uint64_t seed;         /* shared seed of the random operators (Appendix C, random_a)    */
  void *stream;          /* hipStream_t owned by the caller; NULL = the null stream       */
  /* Layer-wise compression (Section 5, set-up of the deep-learning experiments: the
     operator is applied to every layer of the network on its own).  nlayers = 0: the whole
     vector is one layer and the three pointers are ignored.  Otherwise HOST arrays of
     nlayers entries, copied during choco_init: layer l is the slice
     [layer_start[l], layer_start[l] + layer_len[l]) of every worker's vector and is
     compressed as a vector of its own - its own norm and its own length in the scales of
     SIGN and QSGD, layer_k[l] kept entries (0 <= layer_k[l] <= layer_len[l], at least one
     entry kept over all layers) for TOPK and RANDK, the field k above is then ignored.
     The layers are any disjoint slices in ascending order (layer_start[l] >= layer_start[l-1] +
     layer_len[l-1], layer_len[l] >= 1, the last one ends at or before d): a flat parameter
     vector can be handed over as it is.  Entries that lie in no layer (gaps, padding) are never
     compressed or transmitted - q is zero there whatever X and G hold - but they are part of x:
     the local update and the mix apply to them like to any entry.  Fastest is a table whose
     layers each start on a multiple of 4 and follow one another with only that padding between
     them, from entry 0 to d: its layer passes use 16-byte accesses throughout and carry the
     fused local update; any other table takes per-entry layer look-ups and the local update as a
     pass of its own (same results).  Layers may have any length; for
     TOPK and RANDK one workgroup selects a layer of up to CHOCO_MAX_LAYER_LEN entries out
     of its registers and longer layers take the whole-vector select, in launches that they
     share (they cost workspace for its candidate lists, a set per such layer).  With
     layers, IDENTITY is CHOCO_E_UNSUPPORTED, SIGN and QSGD take CHOCO_MIX_AUTO only, and
     TOPK / RANDK take CHOCO_MIX_DIRECT in the default order and up to 64 workers only.
     layer_k_host may be NULL for SIGN and QSGD.     */
  int32_t nlayers;
  const int64_t *layer_start_host;
  const int64_t *layer_len_host;
  const int64_t *layer_k_host;
} choco_config;

#define CHOCO_MAX_LAYER_LEN 10240
#define CHOCO_MAX_D (((int64_t)1 << 31) - ((int64_t)1 << 19)) /* rows are indexed in 32 bits with some headroom */

/* Bytes of device workspace choco_init needs for this configuration (Xhat, S, the CSR
   copy and scratch for the operators).  Validates the scalar fields of cfg only. */
int choco_workspace_bytes(const choco_config *cfg, size_t *bytes_host);

/* Algorithm 1, input line: takes X = x^(-1/2) as it stands in x_dev (n*ld floats, 16-byte
   aligned, caller-owned, updated in place by every step), sets xhat_i^(0) = 0, S = 0,
   t = 0.  workspace_dev must be 256-byte aligned.  CHOCO_E_INVAL for n < 1, d out of
   range (above CHOCO_MAX_D), bad ld, k outside [1, d], levels < 1, gamma <= 0 or not finite, null pointers,
   malformed CSR, or a W that violates Assumption 1; CHOCO_E_NOMEM if the workspace is
   too small.  On error *out is NULL.
   Reads one environment variable, CHOCO_FALLBACK_SPIN_LIMIT (decimal; default 65536): TOPK /
   RANDK on rows above 2^21 entries repair a failed threshold guess in one launch whose
   workgroups wait for one of their number in a bounded poll; this is the bound.  A workgroup
   that reaches it leaves and the exact select scans the row instead: same result, slower.  0
   forces that path (a test of it); there is no reason to set it otherwise. */
int choco_init(const choco_config *cfg, float *x_dev, void *workspace_dev, size_t workspace_bytes,
               choco_ctx **out);

/* One CHOCO-Gossip round for all workers (Algorithm 1 without its gradient step; matrix form in
   Appendix A, "Example: CHOCO-SGD"): v_i = x_i - xhat_i, q_i = Q(v_i), xhat_j += q_j,
   x_i += gamma sum_j w_ij (xhat_j - xhat_i), in the configured order.  Asynchronous;
   advances the step counter t used to key the random operators. */
int choco_gossip_step(choco_ctx *ctx);

/* The local gradient step of Algorithm 1: x_i <- x_i - lr * g_i.  g_dev: n*ld floats, 16-byte aligned. */
int choco_sgd_step(choco_ctx *ctx, const float *g_dev, float lr);

/* One whole iteration in the order of Algorithm 3 (Appendix A): its stochastic gradient
   update (the local gradient step of Algorithm 1) with (g, lr), then the gossip step.  The
   result is bit for bit that of choco_sgd_step followed by choco_gossip_step; where the
   configured operator starts with a dense pass over X (sign, gsgd, top_a; or the mix of the
   printed order) the local update is folded into that pass, which saves one read and one
   write of X.  g_dev: n*ld floats, 16-byte aligned.  Asynchronous; advances t. */
int choco_step(choco_ctx *ctx, const float *g_dev, float lr);

/* The momentum and gradient steps of Algorithm 2 (momentum with weight decay):
   m_i <- (g_i + lambda x_i) + beta m_i;  x_i <- x_i - lr m_i.
   m_dev: n*ld floats of caller-owned momentum memory, zero before the first call. */
int choco_momentum_step(choco_ctx *ctx, const float *g_dev, float *m_dev, float lr, float beta,
                        float lambda);

/* One whole iteration of the momentum variant (Algorithm 2): its local update, then the
   gossip step; bit for bit choco_momentum_step followed by choco_gossip_step, with the
   local update folded into a dense pass over X like choco_step.  m_dev as above. */
int choco_step_momentum(choco_ctx *ctx, const float *g_dev, float *m_dev, float lr, float beta,
                        float lambda);

/* Consensus distance (1/n) sum_i ||x_i - xbar||^2 (Section 5), ||xbar||_2 and the Lyapunov
   function Psi = ||X - Xbar||_F^2 + ||X - Xhat||_F^2 (Assumption 3), accumulated in fp64.
   Any output pointer may be NULL.  Synchronises the stream. */
int choco_metrics(choco_ctx *ctx, double *consensus_host, double *mean_norm_host,
                  double *psi_host);

/* For callers that cannot allocate or wait: code under HIP graph capture, tight serving loops,
   harnesses that forbid hipMalloc.  The figures of choco_metrics, finished on the device and
   written to out_dev (3 doubles, 8-byte aligned, caller-owned device memory): {consensus
   distance, ||xbar||_2, Psi}.  Same kernels as choco_metrics, but their partial sums go to an
   array that is part of the loaded library (CHOCO_NOALLOC_SCRATCH_BYTES of device memory on
   every GPU the library runs on, held until the process ends) instead of the workspace, the
   result is not copied to the host and nothing is waited for: the call enqueues two kernels on
   the context's stream and calls no allocating routine.  The address of the array on the
   context's GPU is looked up once, by choco_init.  CHOCO_E_UNSUPPORTED for d above
   CHOCO_NOALLOC_MAX_D (or a GPU number above 63); CHOCO_E_INVAL if the GPU current at the call
   is not the one that was current in choco_init.  All contexts on one GPU share the array:
   calls that overlap on one GPU (different streams) race; calls on one stream do not.  The
   array keeps the last call's partial sums; a call overwrites every slot it reads. */
#define CHOCO_NOALLOC_MAX_D (1 << 28)
#define CHOCO_NOALLOC_SCRATCH_BYTES (1024 * 3 * 8)
int choco_metrics_noalloc(choco_ctx *ctx, double *out_dev);

/* Device pointers to Xhat and S (n*ld floats each, inside the workspace). */
int choco_xhat(choco_ctx *ctx, float **xhat_dev);
int choco_nsum(choco_ctx *ctx, float **s_dev);

/* Message read-back for parity checks.
   choco_last_selection: TOPK/RANDK only; copies the k (index, value) pairs each worker
   sent in the last gossip step into idx_dev / val_dev (n*k entries each, either may be
   NULL), in unspecified order within a worker.  Asynchronous.
   choco_set_capture: SIGN/QSGD only; while codes_dev is non-NULL every gossip step also
   writes the transmitted code of each entry there (n*ld int32: sign -> +1/-1, gsgd ->
   sig(v)*level).  NULL switches it off.
   choco_last_scalars: 6 doubles per worker from the last step, sign: {||v||_1, scale, 0...},
   gsgd: {sum v^2, ||v||_2, s/||v||_2, ||v||_2/(tau s), 0, 0} (the scales as rounded to fp32);
   TOPK/RANDK: {threshold key, tie cut-off index, kept count, select mode of the last step
   (0 = guessed threshold held, 1 = list rebuilt from the histogram, 2 = row scan), number of
   steps so far that needed mode 1 or 2, length of the last candidate list}; for RANDK with the
   look-ahead on (choco_set_lookahead) these are the figures of the selection made last, which
   is a LATER step's (up to seven steps on).  Synchronises. */
int choco_last_selection(choco_ctx *ctx, int32_t *idx_dev, float *val_dev);
int choco_set_capture(choco_ctx *ctx, int32_t *codes_dev);
int choco_last_scalars(choco_ctx *ctx, double *scalars_host);
/* Layer-wise configurations only (else CHOCO_E_INVAL): 4 doubles per worker and layer
   (n * nlayers * 4, worker-major) from the last step.  SIGN: {||v_l||_1, scale, 0, 0};
   QSGD: {sum v_l^2, ||v_l||_2, s/||v_l||_2, ||v_l||_2/(tau_l s)}; TOPK/RANDK: {threshold
   key, entries kept at the threshold key, entries holding that key, 1 if the guessed
   bracket held the threshold and 0 if the whole layer was searched}; for a layer above
   CHOCO_MAX_LAYER_LEN {threshold key, 0, 0, 0 if the select had to scan the layer itself
   and 1 otherwise}.  With
   layers, choco_last_selection returns sum(layer_k) pairs per worker, layer after layer,
   and choco_last_scalars is CHOCO_E_UNSUPPORTED.  Synchronises the stream. */
int choco_layer_scalars(choco_ctx *ctx, double *scalars_host);

/* What one worker sent in the last gossip step (the q_i of Algorithm 1's exchange), in one call:
   TOPK / RANDK: its k kept (index, value) pairs to idx_dev / val_dev (k entries each, order
   unspecified; with layers sum(layer_k) pairs, layer after layer);
   SIGN / QSGD: its bit planes to bits_dev, W = ceil(d/32) words each, bit e%32 of word e/32:
   plane 0 = the entry was sent negative (QSGD: and its level is not zero), then for QSGD mb
   planes with the bits of min(level, 2^mb - 1), lowest first (mb as in choco_pack_messages);
   scale_host: SIGN the scale ||v||_1/d, QSGD the step ||v||_2/(tau s), 0 for the others; with
   layers these differ per layer (choco_layer_scalars) and scale_host must be NULL, and the
   planes count bits from the start of the whole vector.
   Pointers that do not apply to the operator, or that are NULL, are skipped.  The copies are
   asynchronous on the context's stream; a non-NULL scale_host synchronises it.
   CHOCO_E_INVAL for a worker outside [0, n) and for IDENTITY. */
int choco_last_message(choco_ctx *ctx, int32_t worker, int32_t *idx_dev, float *val_dev,
                       uint32_t *bits_dev, float *scale_host);

/* Messages on the wire (Appendix C states a size with each operator).
   choco_paper_message_bits: that size in bits, host arithmetic only: SIGN d + 32, TOPK
   2*32*k, RANDK 32*k, QSGD b*d + 32 with b = log2(levels) + 1, IDENTITY 32*d.
   choco_pack_messages encodes what every worker sent in the LAST gossip step into
   msgs_dev (n messages of choco_message_bytes each, back to back, 4-byte aligned), in
   32-bit words, W = ceil(d/32):
     SIGN   [scale as float][W words: bit e%32 of word e/32 set iff the entry is -scale]
     QSGD   [step as float][4 words: ascending indices of the entries at level `levels`
            when that exceeds the magnitude bits, 0xFFFFFFFF if unused][W words: signs of
            the non-zero levels][mb planes of W words: bit p of min(level, 2^mb - 1)],
            mb = bit length of levels - 1 (at least 1): b bits per entry for levels = 2^(b-1)
     TOPK   k pairs [index][value as float], order of the pairs unspecified
     RANDK  k values as float, ascending index (the receiver repeats the draw of the mask)
   For SIGN and QSGD the bits of the message are written by the gossip step itself (the pass
   that encodes q also writes one sign bit, resp. b bits, per entry into bit planes in the
   workspace); packing copies them behind the header and needs no capture buffer.  Four index
   slots always suffice: an entry reaches level `levels` only if it holds more than half of the
   vector's norm (up to rounding), and the squares of four such shares add up to the whole.
   Asynchronous for every operator.  choco_unpack_messages is the receiver's
   side: it writes the dense q of every worker (n*ld floats, 16-byte aligned, zero where
   nothing was sent); for RANDK the mask is the one the library drew in the last step.
   Layer-wise configurations: a worker's message is the messages of its layers one after
   the other, each with its own scale / step / index slots (these count inside the layer)
   and its own padding to whole words; TOPK pairs carry positions in the whole vector.
   RANDK layer by layer: the kept values in ascending position in the whole vector (which
   is layer after layer).  IDENTITY has no message format (CHOCO_E_UNSUPPORTED).  These
   calls are not part of the timed path. */
int choco_paper_message_bits(int32_t compressor, int64_t d, int64_t k, int32_t levels,
                             int64_t *bits_host);
int choco_message_bytes(choco_ctx *ctx, size_t *bytes_host);
int choco_pack_messages(choco_ctx *ctx, void *msgs_dev);
int choco_unpack_messages(choco_ctx *ctx, const void *msgs_dev, float *q_dev);



/* The evaluation of the mixing step this context uses, CHOCO_MIX_INCREMENTAL_S or CHOCO_MIX_DIRECT:
   what CHOCO_MIX_AUTO was resolved to by choco_init (see the enumeration above). */
int choco_get_mix_form(choco_ctx *ctx, int32_t *mix_form_host);

/* Step counter t (keys the random operators; set it to resume a run exactly). */
int choco_get_step(choco_ctx *ctx, uint64_t *t_host);
int choco_set_step(choco_ctx *ctx, uint64_t t);

/* Per-kernel timing for measurement (off by default).  While enabled, every kernel the
   library launches is bracketed by two HIP events recorded on the context's stream (at
   most 16384 launches are kept; enabling clears earlier records).  choco_profile_report
   synchronises, writes one text line "kernel_name launches total_milliseconds" per kernel
   into buf_host (NUL-terminated; CHOCO_E_NOMEM if it does not fit) and clears the records.
   The events themselves are host-side objects; no device memory is allocated. */
int choco_set_profiling(choco_ctx *ctx, int enable);
int choco_profile_report(choco_ctx *ctx, char *buf_host, size_t buf_bytes);

/* RANDK: the mask of a step depends on (seed, step, worker) only (Appendix C, random_a: the
   receiver can recover it from the seed), so while the messages and mixes of four steps run on
   the caller's stream the library already selects the masks of the NEXT four steps on a stream
   of its own (created by choco_init, default priority, joined with two events per four steps;
   the kept lists and maps of eight steps are part of the workspace, no device memory is
   allocated; rows above 2^21 entries: one step at a time, two copies; with a layer table a
   second such stream takes half of the selection's launches, forked from and joined to the
   first).  Results do not
   change, whatever the calls in between (a moved step counter drops what was selected for
   other steps).  On by default
   where it applies; switch it off (enable = 0) if every call must leave all of its work
   on the caller's stream, e.g. under stream capture.  A no-op for other configurations. */
int choco_set_lookahead(choco_ctx *ctx, int enable);

/* Waits for everything the library has enqueued: the context's stream and, where RANDK
   selects ahead, the library's own stream (that selection writes the workspace). */
int choco_sync(choco_ctx *ctx);
/* Frees the context (host memory, its profiling events, its own stream after waiting for
   it) without waiting for the caller's stream: call choco_sync first if X or the workspace
   are to be freed or reused right away.  The handle is invalid afterwards.  NULL is
   allowed. */
int choco_destroy(choco_ctx *ctx);
const char *choco_strerror(int code);
int choco_last_hip_error(choco_ctx *ctx); /* raw hipError_t of the last CHOCO_E_HIP */

#ifdef __cplusplus
}
#endif
#endif /* CHOCO_H */
