/*
 * csgs -- one partition's sampled GCN layer step with communication-efficient
 * (locality-skewed) layer-wise neighbor sampling, for AMD MI355X (gfx950).
 *
 * The five operations follow the paper's statement of the method:
 *   csgs_build_probs   importance weights ||w_*j||^2 over the neighbors of S_l (Section 4.1),
 *                      skewed linear weighted sampling distribution (Section 4.2, Eq. 10;
 *                      Eq. 7 when skew = 1)
 *   csgs_sample_layer  B draws from that distribution, inclusion probability (Eq. 8), sampled
 *                      adjacency with every kept edge divided by it (Eq. 3)
 *   csgs_remote_count  sampled nodes that live on other partitions = communication volume (Eq. 4)
 *   csgs_aggregate     Z = P~ sigma(H_prev)   (Section 3, Eq. 1: gather of rows + sparse x dense)
 *   csgs_layer_gemm    H = Z W                (Section 3, Eq. 1: dense layer weights)
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless the comment says "host".  All buffers are owned by
 *     the caller; the library never allocates, frees or synchronises.  Work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = default stream) and the call returns at once.
 *   - Return value: CSGS_OK or a negative CSGS_E* code found synchronously from host-visible
 *     arguments; in that case nothing was enqueued.
 *   - Failures that depend on device data (capacity overflow, a non-finite edge value, an id
 *     out of range, an empty candidate set) OR the matching CSGS_ST_* bit into the int32 word
 *     `status` (device).  The caller zeroes it and reads it when it next synchronises.  When a
 *     bit is set the outputs of that call are unspecified but every access stayed in bounds.
 *   - Row counts that exist only on the device.  In a multi-layer step the rows of one call are
 *     the node set the previous call sampled, whose size the host does not know without waiting.
 *     Every entry point that takes a row count n (nS, n_rows, M) therefore also takes n_dev, a
 *     nullable DEVICE pointer to an int32.  NULL: n is the count.  Otherwise the kernels use
 *     min(max(*n_dev, 0), n), read when they run, and n is only the capacity: host-side checks,
 *     launch sizes and array extents ("[nS + 1]") refer to it, entries past the device count are
 *     left untouched.  A whole step can so be enqueued without the host ever waiting.
 *   - `ws` describes scratch memory (see csgs_workspace), prepared once with
 *     csgs_workspace_init().  Every call leaves it ready for the next.  Calls that share one
 *     workspace must be ordered on one stream.  Calls on DIFFERENT workspaces may run side by
 *     side on different streams; at most four such call sequences per device at a time (two
 *     kernels hold all their blocks resident while they wait for each other, and four of them
 *     fit a compute unit together; a sequence that processes several instances per call, see
 *     csgs_workspace, counts once: its instances are dispatched one after the other).
 *   - Replay.  Nothing a kernel needs to tell one call from the next is fixed at launch time
 *     (the call counter behind the inter-block flags lives in the workspace and is advanced by
 *     the kernels), and no entry point records a memset.  A sequence of calls captured into a
 *     HIP graph can therefore be replayed; what changes between replays (the batch, the
 *     iteration number) is passed through device memory: see nS_dev / iter_dev.
 */
#ifndef CSGS_H
#define CSGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CSGS_OK = 0,
    CSGS_EINVAL = -1,       /* null pointer, non-positive size, skew < 1, lo > hi, bad alignment */
    CSGS_EWORKSPACE = -2,   /* the workspace is smaller than this call's sizes need */
    CSGS_EUNSUPPORTED = -3, /* dtype or dimension outside what the kernels cover */
    CSGS_ERANGE = -4,       /* fixed-point format would keep fewer than 24 fraction bits */
    CSGS_ELAUNCH = -5       /* the HIP runtime refused a launch */
};

enum {
    CSGS_ST_CAND_OVERFLOW = 1,    /* more candidates than `cap` */
    CSGS_ST_BAD_EDGE_VALUE = 2,   /* a scanned edge value is NaN or infinite */
    CSGS_ST_EMPTY_CANDIDATES = 4, /* the rows of S have no edges at all */
    CSGS_ST_ADJ_OVERFLOW = 8,     /* sampled adjacency needs more than adj_cap entries */
    CSGS_ST_BAD_NODE_ID = 16,     /* an entry of S is outside [0, n_nodes) */
    CSGS_ST_EDGE_OVERFLOW = 32,   /* the rows of S hold more edges than the workspace was sized for */
    CSGS_ST_INTERNAL = 64         /* a bounded wait between blocks ran out (should not happen) */
};

enum { CSGS_F32 = 0, CSGS_BF16 = 1 };

/* Propagation matrix P in CSR (host struct holding device pointers).  Columns ascend within a
 * row.  [local_lo, local_hi) is the id range of the partition this GPU owns (the paper splits
 * nodes evenly by id, Section 5.1).  rownorm2_max bounds max_i sum_j P_ij^2 (1 for the
 * symmetric or row normalisation); it fixes the fixed-point scale of the weights. */
typedef struct csgs_graph {
    int64_t n_nodes;
    int64_t nnz;
    const int64_t *rowptr; /* [n_nodes + 1] */
    const int32_t *colidx; /* [nnz] */
    const float *val;      /* [nnz] */
    int32_t local_lo, local_hi;
    float rownorm2_max;
} csgs_graph;

/* Written by csgs_build_probs (device).  |L|, |R| and the weight sums are over CANDIDATES
 * (Section 4.2 splits N(S_l) into local and remote nodes). */
typedef struct csgs_prob_stats {
    int64_t n_cand;        /* |N(S_l)| */
    int64_t n_local;       /* |L| */
    int64_t n_remote;      /* |R| */
    int64_t edges_scanned; /* sum of deg(i), i in S_l */
    uint64_t w_local;      /* sum_{k in L} ||w_*k||^2, fixed point, unskewed */
    uint64_t w_remote;     /* sum_{k in R} ||w_*k||^2 */
    uint64_t total;        /* denominator of Eq. 10 in fixed point = cdf[n_cand - 1] */
    int32_t shift;         /* fraction bits of the fixed-point weights */
    int32_t skew_fx;       /* multiplier of local weights that was used, in 1/16 units (remote: 16);
                              negative when remote candidates were given weight zero */
} csgs_prob_stats;

/* Scratch memory of the sampling calls: a host descriptor of a caller-owned device buffer.
 * `base` is 256-byte aligned and holds at least csgs_workspace_bytes(n_nodes, nS_max, B_max,
 * edges_max) bytes.  The four sizes fix the layout, so they must not change while the buffer is
 * in use (and the descriptor is used by one host thread at a time): n_nodes = nodes of the graph, nS_max = most rows a call passes, B_max = most draws,
 * edges_max = most edges the rows of one call hold in total (the graph's nnz is always enough). */
typedef struct csgs_workspace {
    void *base;
    size_t bytes;
    int64_t n_nodes;
    int32_t nS_max, B_max;
    int64_t edges_max;
    /* owned by the library (csgs_workspace_init resets them): */
    uint64_t rows_buf;   /* which of the two sets of row offsets belongs to the current rows */
    uint64_t has_draw;   /* a csgs_draw_nodes has been enqueued on this workspace */
    int32_t draw_B;      /* its B */
    int32_t has_next;    /* the latest csgs_sample_layer prepared the offsets of its S_next */
    /* several instances per call, set by the caller (see below); 0 or 1 = one instance */
    int32_t n_inst;
    int32_t scan_mode;   /* how csgs_build_probs adds up the weights of local candidates: 0 = the library
                            chooses (through owner blocks when a launch scans a million edges or more,
                            else with device-scope atomics like the remote ones), 1 = always atomics,
                            2 = owner blocks whenever the local range allows.  Same results. */
    int64_t inst_stride; /* bytes between consecutive instances' arrays; a multiple of 256 */
} csgs_workspace;

/* Several instances per call.  Consecutive training iterations sample independent mini-batches
 * against the same graph (Section 5.1: a new mini-batch, newly sampled, per iteration); at the
 * paper's batch sizes one of them is too little work to fill the device.  With n_inst = K > 1 the
 * buffer holds K workspaces back to back (bytes >= K * csgs_workspace_bytes(...)), and every call
 * that takes this descriptor -- csgs_build_probs, csgs_build_probs_auto, csgs_draw_nodes,
 * csgs_sampled_adjacency, csgs_sample_layer -- processes K independent instances in the same kernel
 * launches.  Instance k reads and writes every device-pointer argument of the call (S, nS_dev, the
 * candidate arrays, stats, S_next, mult, p_incl, n_next, the adjacency arrays, adj_nnz, status, and
 * remote_total / per_part / src_row / remote_ids of csgs_remote_out) at the given address plus
 * k * inst_stride bytes; null arguments are null for all.  Shared by all instances: the graph's
 * arrays, part_bounds, iter_dev, and all scalar arguments, except that instance k's draws use
 * iteration number iter + k (*iter_dev + k).  Results are those of K separate calls.  At most 64. */

/* Bytes needed for a workspace of these sizes; 0 on bad input. */
size_t csgs_workspace_bytes(int64_t n_nodes, int32_t nS_max, int32_t B_max, int64_t edges_max);

/* Size of the leading part of the workspace that is all-zero whenever no call is in flight
 * (accumulators, flags, bitmaps, rank table).  For tests and debugging. */
size_t csgs_workspace_clean_bytes(int64_t n_nodes);

/* Zero-fills the buffer of `ws` (a fill kernel, safe under graph capture).  Call once before the
 * first use, and again after a call was aborted.  Host errors: CSGS_EINVAL, CSGS_EWORKSPACE. */
int csgs_workspace_init(csgs_workspace *ws /*host*/, void *stream);

/* Bounds the polls a block may spend waiting for another block's flag (polls < 0: the built-in
 * limit, large enough for seconds of waiting).  For tests of the timeout path: with a tiny limit a
 * wait that is not satisfied at once gives up, the call sets CSGS_ST_INTERNAL, its outputs are
 * unspecified, and every kernel still ends normally with all accesses in bounds.  Afterwards
 * csgs_workspace_init must be called again.  Host errors: CSGS_EINVAL, CSGS_EWORKSPACE. */
int csgs_workspace_wait_limit(csgs_workspace *ws /*host*/, int64_t polls, void *stream);

/* Host-only helper: the fixed-point parameters csgs_build_probs will use (see there).
 * shift and s_fx are host pointers, nullable.  Returns CSGS_EINVAL for nS <= 0, skew < 1 or
 * > 2^20, rownorm2_max <= 0; CSGS_ERANGE when fewer than 24 fraction bits would remain. */
int csgs_fixed_point(int32_t nS, float skew, float rownorm2_max, int32_t *shift, int64_t *s_fx);

/*
 * Sampling distribution over the candidates N(S_l) = union of the neighbors of the rows in S
 * (Section 4.1; the layer-wise sampler of Section 5.1).
 *
 * Weight of candidate j:  ||w_*j||^2 = sum_{i in S} P_ij^2, held as an exact integer
 *   sum_i max(1, rne(P_ij^2 * 2^shift)),  shift = min(52, 61 - ceil(log2 nS) - ceil(log2 s_fx)
 *   - ceil(log2 rownorm2_max)),  s_fx = round(16 * skew),
 * so that the result does not depend on summation order.  Skewed weight (Eq. 10 numerator):
 * weight * s_fx for local j, weight * 16 for remote j.
 *
 *   S        [nS] distinct node ids, any order.  NULL: the rows are the node set S_next of the latest
 *            csgs_sample_layer on this workspace (which has already prepared their offsets, so
 *            this call is one kernel shorter); nS must be that call's B, nS_dev NULL -- the row
 *            count is its *n_next
 *   skew     s >= 1 (s = 1 is linear weighted sampling, Eq. 7); used in 1/16 steps.  +infinity
 *            selects the "Local" version of Section 5.1: remote candidates keep their place in
 *            the list but get probability zero
 *   cand_id  [cap] out: candidate ids ascending
 *   cand_w   [cap] out: fixed-point ||w_*j||^2 (unskewed)
 *   cdf      [cap] out: inclusive running sum of the skewed weights (cdf[n_cand-1] = total)
 *   q        [cap] out, nullable: Eq. 10 as float = skewed weight / total
 *   stats    out, see above
 * Host errors: CSGS_EINVAL, CSGS_ERANGE (shift < 24 for nS rows), CSGS_EWORKSPACE.
 * Status bits: CAND_OVERFLOW, BAD_EDGE_VALUE, EMPTY_CANDIDATES, BAD_NODE_ID, EDGE_OVERFLOW.
 */
int csgs_build_probs(const csgs_graph *g /*host*/, const int32_t *S, int32_t nS, const int32_t *nS_dev, float skew,
                     int32_t *cand_id, uint64_t *cand_w, uint64_t *cdf, float *q, int64_t cap,
                     csgs_prob_stats *stats, csgs_workspace *ws /*host*/, int32_t *status,
                     void *stream);

/*
 * Same, with the skew chosen by Theorem 1 (Eq. 12) from the candidate counts of this very call:
 *   s = D (|N(S_l)| - B) / |R| + 1/2,  raised to 1 when smaller, 1 when there is no remote
 * candidate, cut at skew_max, rounded to 1/16 (half up); evaluated on the device in double.
 * The fixed-point shift is the one of skew = skew_max, whatever s turns out to be.  The s that
 * was used is reported in stats->skew_fx.  D >= 0 is the constant of the theorem (the paper
 * sweeps 4, 8, 16, 32), B the sampling budget.
 */
int csgs_build_probs_auto(const csgs_graph *g /*host*/, const int32_t *S, int32_t nS, const int32_t *nS_dev,
                          float D, int32_t B,
                          float skew_max, int32_t *cand_id, uint64_t *cand_w, uint64_t *cdf, float *q,
                          int64_t cap, csgs_prob_stats *stats, csgs_workspace *ws /*host*/,
                          int32_t *status, void *stream);

/*
 * B independent draws from q (Section 4.1: the sampling is run B times), deduplicated into
 * the next layer's node set, and the sampled adjacency of Eq. 3.
 *
 * Draw t uses Philox4x32-10 with key (seed_lo, seed_hi) and counter (t, layer, iter_lo, iter_hi)
 * (iter = *iter_dev, a device uint64 read when the kernel runs, if iter_dev is not NULL);
 * r = x0 | x1 << 32;  u = floor(r * total / 2^64);  the draw is the first candidate k with
 * cdf[k] > u.  Inclusion probability p_j = 1 - (1 - q_j)^B (Eq. 8) in double.
 *
 *   cand_id, cdf, stats   as written by csgs_build_probs for the same S (device);
 *            cand_cap = the capacity those arrays were given there.  The call must follow that
 *            csgs_build_probs call on the same workspace: it reuses the row offsets left there,
 *            and with them the row count that call used (so there is no nS_dev here; nS is the
 *            same capacity).  S may be NULL if it was NULL there.  Besides its outputs the call
 *            prepares the row offsets of S_next for a following csgs_build_probs(S = NULL)
 *            (only when B <= nS_max of the workspace; otherwise that call returns CSGS_EINVAL).
 *   S_next   [B] out: distinct sampled ids ascending; *n_next of them
 *   mult     [B] out: how many of the B draws hit each
 *   p_incl   [B] out: p_j as float
 *   adj_rowptr [nS+1], adj_col [adj_cap], adj_val [adj_cap], adj_nnz: out, CSR of P~ with rows in
 *            the order of S, adj_col = position in S_next (ascending within a row),
 *            adj_val = (float)((double)P_ij / p_j)
 *   remote   nullable: also write the remote split of S_next (see csgs_remote_out)
 * Host errors: CSGS_EINVAL, CSGS_EWORKSPACE.  Status bits: ADJ_OVERFLOW, EDGE_OVERFLOW.
 */
/* Optional extra outputs of csgs_sample_layer: what csgs_remote_count (below) computes, produced by
 * spare blocks of the adjacency kernel, so that a layer step is one launch shorter.  Host struct
 * of device pointers; fields as the parameters of csgs_remote_count. */
typedef struct csgs_remote_out {
    int32_t local_lo, local_hi;
    const int32_t *part_bounds; /* nullable */
    int32_t P;
    int64_t *remote_total;
    int64_t *per_part;  /* nullable */
    int32_t *src_row;   /* nullable */
    int32_t *remote_ids; /* nullable */
} csgs_remote_out;

int csgs_sample_layer(const csgs_graph *g /*host*/, const int32_t *S, int32_t nS,
                      const int32_t *cand_id, const uint64_t *cdf, int64_t cand_cap,
                      const csgs_prob_stats *stats, int32_t B, uint64_t seed, uint64_t iter,
                      const uint64_t *iter_dev, uint32_t layer, int32_t *S_next, int32_t *mult, float *p_incl, int32_t *n_next,
                      int32_t *adj_rowptr, int32_t *adj_col, float *adj_val, int64_t adj_cap,
                      int64_t *adj_nnz, const csgs_remote_out *remote /*host, nullable*/,
                      csgs_workspace *ws /*host*/, int32_t *status, void *stream);

/*
 * The two halves of csgs_sample_layer, for samplers that draw once and then need the sampled
 * operator for other rows than the ones the distribution was built from (the subgraph sampler of
 * Section 5.1 takes all training nodes as candidates, draws the subgraph's nodes, and runs the
 * full convolution on the subgraph: rows = the drawn nodes themselves).
 *
 * csgs_draw_nodes: the B draws, S_next / mult / p_incl / n_next as in csgs_sample_layer.  It
 * leaves the node -> position table and the double inclusion probabilities in the workspace.
 * csgs_sampled_adjacency: CSR of P~ (Eq. 3) for `rows` (n_rows node ids, device) against the node
 * set of the latest csgs_draw_nodes on the same workspace; outputs as in csgs_sample_layer.
 * Host errors: CSGS_EINVAL (also: no draw has run), CSGS_EWORKSPACE (n_rows above nS_max).
 * Status bits: ADJ_OVERFLOW, EDGE_OVERFLOW, BAD_NODE_ID.
 */
int csgs_draw_nodes(int64_t n_nodes, const int32_t *cand_id, const uint64_t *cdf, int64_t cand_cap,
                    const csgs_prob_stats *stats, int32_t B, uint64_t seed, uint64_t iter,
                    const uint64_t *iter_dev, uint32_t layer, int32_t *S_next, int32_t *mult, float *p_incl, int32_t *n_next,
                    csgs_workspace *ws /*host*/, int32_t *status, void *stream);
int csgs_sampled_adjacency(const csgs_graph *g /*host*/, const int32_t *rows, int32_t n_rows,
                           const int32_t *n_rows_dev,
                           int32_t *adj_rowptr, int32_t *adj_col, float *adj_val, int64_t adj_cap,
                           int64_t *adj_nnz, csgs_workspace *ws /*host*/, int32_t *status,
                           void *stream);

/*
 * Communication volume of the step (Eq. 4; Section 5.2 reports the number of nodes whose
 * feature vectors are transferred): sampled ids outside [local_lo, local_hi).
 *
 *   S_next [*n_next] ascending (device; the order csgs_sample_layer produces -- the kernel
 *   relies on it), n_next device
 *   part_bounds [P+1] nullable: partition p owns [b[p], b[p+1]); per_part [P] nullable out
 *   remote_total out (device int64)
 *   src_row [*n_next] nullable out: where the aggregation finds the feature row of S_next[k]:
 *            id - local_lo for a local node, -1 - (rank among the sampled remote nodes) otherwise
 *   remote_ids [*n_next] nullable out: the sampled remote ids ascending (the request list whose
 *            rows the caller stages, in this order, for csgs_aggregate)
 */
int csgs_remote_count(const int32_t *S_next, const int32_t *n_next, int32_t local_lo,
                      int32_t local_hi, const int32_t *part_bounds, int32_t P,
                      int64_t *remote_total, int64_t *per_part, int32_t *src_row,
                      int32_t *remote_ids, void *stream);

/*
 * Z = P~ sigma?(X)  (Eq. 1; sigma = ReLU on the INPUT rows, none for the bottom layer).
 *
 *   adj_*     CSR of P~ from csgs_sample_layer; nS rows
 *   n_next    device, nullable: number of columns of P~ (bounds adj_col; NULL = not checked
 *             against it)
 *   X_local   row-major, rows_local rows, leading dimension ld_local elements (NULL allowed
 *             when rows_local = 0); X_remote nullable, rows_remote rows, ld_remote
 *   src_row   nullable.  NULL: column c reads row c of X_local (upper layers: compact input).
 *             Else column c reads row src_row[c] of X_local if >= 0, row -1 - src_row[c] of X_remote.
 *   F         feature width; dtype CSGS_F32 or CSGS_BF16 (bf16 widened exactly, fp32 accumulate)
 *   Z         [nS x F] float out, leading dimension ldz; rows without kept edges are zero
 * Products are accumulated in double in ascending edge order and rounded to float once.  An edge whose column or source row lies
 * outside the tables contributes nothing (no status word here; every load stays in bounds).
 */
int csgs_aggregate(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val,
                   int32_t nS, const int32_t *nS_dev, const int32_t *n_next, const void *X_local, int64_t ld_local,
                   int64_t rows_local, const void *X_remote, int64_t ld_remote, int64_t rows_remote,
                   const int32_t *src_row, int32_t F, int dtype, int relu_on_input, float *Z,
                   int64_t ldz, void *stream);

/*
 * out[k, 0..F) = X[ids[k], 0..F) for k < n: fills the staged buffer of sampled remote feature rows
 * that csgs_aggregate reads (X_remote) from the request list csgs_remote_count wrote (remote_ids).
 * On one GPU that holds the whole feature table this takes the place of the exchange of feature
 * vectors between partitions (Section 3, the paragraph on the transfer of feature vectors).
 *
 *   X [rows x F], leading dimension ld (elements of dtype CSGS_F32 or CSGS_BF16; rows are copied
 *   bit for bit); ids [cap] device; n = min(*n_dev, cap) when n_dev (device int64, e.g.
 *   remote_total) is given, else cap; out [cap x F], leading dimension ldo.  An id outside
 *   [0, rows) yields a zero row.  Rows k >= n are left untouched.
 */
int csgs_gather_rows(const void *X, int64_t ld, int64_t rows, int32_t F, int dtype, const int32_t *ids,
                     int64_t cap, const int64_t *n_dev, void *out, int64_t ldo, void *stream);

/* H [M x Nout] = Z [M x K] W [K x Nout], all row-major fp32 (Eq. 1).  Operands are widened to
 * double, products accumulate in double on the matrix cores, one rounding to float.
 * With M_dev (device) only the first min(*M_dev, M) rows of H are computed and written; Z must
 * still be M rows of readable memory -- rows beyond the count may be read, whatever they hold
 * reaches no row that is written.
 * Host errors: CSGS_EINVAL; CSGS_EUNSUPPORTED when the tile count exceeds 2^30. */
int csgs_layer_gemm(const float *Z, int64_t ldz, int32_t M, const int32_t *M_dev, int32_t K, const float *W,
                    int64_t ldw, int32_t Nout, float *H, int64_t ldh, void *stream);

/*
 * Several instances per launch for the layer compute (the counterpart of n_inst in csgs_workspace:
 * the forward passes of the mini-batches sampled by one group of sampling calls are independent of
 * each other).  The _n forms below take the arguments of csgs_aggregate, csgs_layer_gemm and
 * csgs_gather_rows plus a host struct of strides; instance k of n_inst uses each device pointer at
 * its address + k * the stride of its group, in bytes (multiples of 16; 0 = the same array for all):
 *   adj       what the sampling calls wrote: adj_rowptr, adj_col, adj_val, nS_dev / M_dev, n_next,
 *             src_row (csgs_aggregate); M_dev (csgs_layer_gemm); ids, n_dev (csgs_gather_rows)
 *   x         the input matrix: X_local (csgs_aggregate), Z (csgs_layer_gemm), X (csgs_gather_rows)
 *   x_remote  X_remote (csgs_aggregate)
 *   out       the output matrix: Z (csgs_aggregate), H (csgs_layer_gemm), out (csgs_gather_rows)
 * Everything else (W, all sizes and leading dimensions) is shared.  inst NULL = one instance.
 * Results are those of n_inst separate calls.  Host errors as the plain forms, CSGS_EINVAL also
 * for n_inst outside [1, 64] and negative or misaligned strides.
 */
typedef struct csgs_inst_strides {
    int32_t n_inst;
    int32_t reserved;
    int64_t adj, x, x_remote, out;
} csgs_inst_strides;

int csgs_aggregate_n(const csgs_inst_strides *inst /*host*/, const int32_t *adj_rowptr, const int32_t *adj_col,
                     const float *adj_val, int32_t nS, const int32_t *nS_dev, const int32_t *n_next,
                     const void *X_local, int64_t ld_local, int64_t rows_local, const void *X_remote,
                     int64_t ld_remote, int64_t rows_remote, const int32_t *src_row, int32_t F, int dtype,
                     int relu_on_input, float *Z, int64_t ldz, void *stream);
int csgs_layer_gemm_n(const csgs_inst_strides *inst /*host*/, const float *Z, int64_t ldz, int32_t M,
                      const int32_t *M_dev, int32_t K, const float *W, int64_t ldw, int32_t Nout, float *H,
                      int64_t ldh, void *stream);
int csgs_gather_rows_n(const csgs_inst_strides *inst /*host*/, const void *X, int64_t ld, int64_t rows, int32_t F,
                       int dtype, const int32_t *ids, int64_t cap, const int64_t *n_dev, void *out, int64_t ldo,
                       void *stream);

/*
 * H = (P~ sigma?(X)) W  (Eq. 1, both halves of a sampled layer) in one kernel: csgs_aggregate followed by
 * csgs_layer_gemm without Z passing through memory.  A block aggregates 32 rows of Z into LDS (sums in double in
 * edge order, one rounding to float: the rounding point of csgs_aggregate) and multiplies them by W on the fp64
 * matrix cores from there (the arithmetic of csgs_layer_gemm).  H equals that of the two calls up to the order
 * in which the double sums of a row of Z are formed.
 *
 *   adj_*, nS, nS_dev, n_next, X_local .. relu_on_input   as csgs_aggregate (F_in = its F)
 *   W [F_in x F_out] row-major, leading dimension ldw; H [nS x F_out] float out, leading dimension ldh
 *   Z         nullable: [nS x F_in] float out, leading dimension ldz, also receives P~ sigma?(X) (a training
 *             step needs it for dW = Z^T G); NULL: Z is never written
 *   csgs_layer_forward_n: instances as above (H moves by `out`); z_stride: bytes between the instances' Z
 *             (a multiple of 16)
 * Takes F_in <= 64, even F_in <= 128, and F_in <= 256 that are multiples of 4, with rows of X starting on
 * multiples of 1, 2 and 4 elements: csgs_layer_forward_supported() (host, no device work) returns 1 for a width,
 * type and pair of leading dimensions (0 = no such table) that the kernel takes, else 0; the calls themselves return
 * CSGS_EUNSUPPORTED for the others, and the caller uses csgs_aggregate + csgs_layer_gemm.
 * Host errors: CSGS_EINVAL, CSGS_EUNSUPPORTED.
 */
int csgs_layer_forward_supported(int32_t F_in, int dtype, int64_t ld_local, int64_t ld_remote);
int csgs_layer_forward(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val, int32_t nS,
                       const int32_t *nS_dev, const int32_t *n_next, const void *X_local, int64_t ld_local,
                       int64_t rows_local, const void *X_remote, int64_t ld_remote, int64_t rows_remote,
                       const int32_t *src_row, int32_t F_in, int dtype, int relu_on_input, const float *W,
                       int64_t ldw, int32_t F_out, float *H, int64_t ldh, float *Z, int64_t ldz, void *stream);
int csgs_layer_forward_n(const csgs_inst_strides *inst /*host*/, const int32_t *adj_rowptr, const int32_t *adj_col,
                         const float *adj_val, int32_t nS, const int32_t *nS_dev, const int32_t *n_next,
                         const void *X_local, int64_t ld_local, int64_t rows_local, const void *X_remote,
                         int64_t ld_remote, int64_t rows_remote, const int32_t *src_row, int32_t F_in, int dtype,
                         int relu_on_input, const float *W, int64_t ldw, int32_t F_out, float *H, int64_t ldh,
                         float *Z, int64_t ldz, int64_t z_stride, void *stream);

/*
 * Gradients of one sampled layer.  Every GPU obtains a stochastic gradient of the loss (Section 3,
 * Eq. 2) through its sampled layers (Eq. 1): for H = Z W, Z = P~ sigma(H_prev) and G = dL/dH,
 *     dW      = Z^T G                                  csgs_layer_gemm_grad_w
 *     dZ      = G W^T                                  csgs_layer_gemm_grad_z
 *     dH_prev = (P~^T dZ) .* [H_prev > 0]              csgs_aggregate_grad   (sigma = ReLU)
 * Same conventions as the forward calls: row-major fp32, double accumulation (fp64 matrix cores
 * for the two products), one rounding to float, M / nS / n_cols with nullable *_dev counterparts.
 *
 * csgs_layer_gemm_grad_w: Z [M x K], G [M x Nout] -> dW [K x Nout].  The sum over the M rows is
 *   split into parts that are added in a fixed order; `scratch` (device, 8-byte aligned) holds the
 *   parts: at least csgs_layer_gemm_grad_w_scratch_bytes(M, K, Nout) bytes.
 * csgs_layer_gemm_grad_z: G [M x Nout], W [K x Nout] (as in the forward call) -> dZ [M x K]; as in the
 *   forward call, rows of G beyond a device count may be read and reach no row that is written.
 * csgs_aggregate_grad: P~ as written by csgs_sample_layer (nS rows, n_cols = *n_next columns,
 *   adj_cap = capacity of adj_col / adj_val), dZ [nS x F] -> dH_prev [n_cols x F].  H_prev
 *   [n_cols x F] is the layer's input (NULL: no activation, no mask).  The transpose of P~ is built
 *   in `scratch` (256-byte aligned, csgs_aggregate_grad_scratch_bytes(n_cols, adj_cap) bytes),
 *   every column in ascending row order: the sums are formed in that order, in double, so two calls
 *   on the same input give the same bits.
 * Host errors: CSGS_EINVAL, CSGS_EWORKSPACE (scratch too small), CSGS_EUNSUPPORTED.
 */
size_t csgs_layer_gemm_grad_w_scratch_bytes(int32_t M, int32_t K, int32_t Nout);
int csgs_layer_gemm_grad_w(const float *Z, int64_t ldz, const float *G, int64_t ldg, int32_t M,
                           const int32_t *M_dev, int32_t K, int32_t Nout, float *dW, int64_t lddw,
                           void *scratch, size_t scratch_bytes, void *stream);
int csgs_layer_gemm_grad_z(const float *G, int64_t ldg, int32_t M, const int32_t *M_dev, int32_t Nout,
                           const float *W, int64_t ldw, int32_t K, float *dZ, int64_t lddz, void *stream);
/*
 * csgs_layer_gemm_grad_w for callers that cannot allocate device memory and have no scratch buffer to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same results as csgs_layer_gemm_grad_w, but the partial sums go to a
 * buffer of CSGS_GRAD_W_STATIC_BYTES bytes that is part of the library's device image (every GPU the
 * library runs on holds one until the process ends).  The call allocates and frees nothing.
 *   - Shapes whose csgs_layer_gemm_grad_w_scratch_bytes(M, K, Nout) exceeds CSGS_GRAD_W_STATIC_BYTES
 *     are rejected with CSGS_EWORKSPACE before anything is enqueued (the five named configurations
 *     need at most 16.1 MB).
 *   - All calls on one GPU share that buffer: calls that overlap on one GPU (different streams, or
 *     one stream's call still running when another stream's starts) race.  Order them.
 *   - The first call on a device looks up the buffer's address on that device (no allocation); make
 *     that first call outside graph capture.  CSGS_ELAUNCH if the lookup fails.
 */
#define CSGS_GRAD_W_STATIC_BYTES (32u << 20)
int csgs_layer_gemm_grad_w_static(const float *Z, int64_t ldz, const float *G, int64_t ldg, int32_t M,
                                  const int32_t *M_dev, int32_t K, int32_t Nout, float *dW, int64_t lddw,
                                  void *stream);
size_t csgs_aggregate_grad_scratch_bytes(int32_t n_cols, int64_t adj_cap);
int csgs_aggregate_grad(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val,
                        int64_t adj_cap, int32_t nS, const int32_t *nS_dev, int32_t n_cols,
                        const int32_t *n_cols_dev, const float *dZ, int64_t lddz, int32_t F,
                        const float *H_prev, int64_t ldh, float *dH_prev, int64_t ldd, void *scratch,
                        size_t scratch_bytes, void *stream);

/* Static string for a CSGS_E* code. */
const char *csgs_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CSGS_H */
