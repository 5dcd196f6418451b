/*
 * libsat — one graph partition's SAT (staleness-alleviated training) GCN layer
 * step on one MI355X (gfx950): pull of cached halo embeddings, correction by
 * the embedding predictor, normalised-adjacency aggregation, feature transform,
 * the matching backward pass, and push of fresh embeddings.
 *
 * Plain C ABI. No function takes or returns a framework type.
 *
 * Conventions (all entry points)
 * ------------------------------
 *  - Every function returns a sat_status; SAT_OK is 0, errors are negative.
 *    Arguments are validated on the host BEFORE anything is enqueued: a call
 *    that returns an error has had no effect on device memory.
 *  - "device pointer" = memory of the current HIP device; "host pointer" =
 *    ordinary process memory. The library allocates no device memory, keeps no
 *    pointer past the kernels it enqueues, and owns nothing: every buffer is
 *    the caller's. Scratch comes from a caller-supplied workspace whose size a
 *    *_workspace_bytes() query returns.
 *  - Compute calls take `stream` (a hipStream_t passed as void*, NULL = the
 *    null stream), enqueue their kernels there and return without waiting.
 *  - Dense matrices are row-major with an explicit leading dimension `ld`
 *    counted in ELEMENTS (ld >= number of columns). Padding columns
 *    [d, ld) are never read for arithmetic and never written.
 *  - Node ids are int32_t; row offsets (rowptr, split, colptr) are int64_t.
 *  - Element types (`dtype`): SAT_F32 (float) or SAT_BF16 (bfloat16, the
 *    upper 16 bits of a float). dtype is the STORAGE type of every `void*`
 *    matrix of the call (features, activations, history tables, layer
 *    weights W and the gradients with those shapes). Every sum is carried in
 *    fp32 and rounded to nearest-even once, where the result is stored.
 *    Pointers typed `float*` are fp32 in both modes: the partition view's
 *    values, the predictor's parameters, dW and the loss.
 *  - Alignment of matrices other than gather/push operands: base pointer
 *    16-byte aligned and ld * sizeof(element) a multiple of 16 (ld % 4 == 0
 *    for fp32, ld % 8 == 0 for bf16), else SAT_EALIGN. Gather and push accept
 *    any ld (they fall back to element-wise copies).
 *  - Kernels bound-check every id they read from device memory: an id outside
 *    its table is skipped (gather/push: that row is not copied; aggregation:
 *    that entry contributes nothing). They never fault on bad ids, but the
 *    result is then unspecified for the rows concerned.
 *
 * Notation follows the paper: V_m local (in-subgraph) nodes of partition m,
 * n_local = |V_m|; halo = out-of-subgraph 1-hop neighbours, n_halo of them;
 * n_bar = n_local + n_halo; H_bar^(l) = [H_in^(l) ; H_out_hat^(l)] one buffer
 * of n_bar rows, local rows first; P = A_hat = D~^-1/2 (A + I) D~^-1/2 with
 * GLOBAL degrees, P = P_in + P_out.
 */
#ifndef SAT_H_
#define SAT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t sat_status;

enum {
  SAT_OK = 0,
  SAT_EINVAL = -1,       /* null pointer, negative size, ld < d, inconsistent sizes */
  SAT_EUNSUPPORTED = -2, /* element type or a dimension outside what is compiled in */
  SAT_EALIGN = -3,       /* a pointer or ld breaks a stated alignment requirement */
  SAT_EWORKSPACE = -4,   /* workspace pointer null or smaller than the query says */
  SAT_EHIP = -5          /* a HIP call or launch failed; see sat_last_hip_error() */
};

enum { SAT_F32 = 0, SAT_BF16 = 1 };
enum { SAT_ACT_IDENTITY = 0, SAT_ACT_RELU = 1 };

/*
 * Local view of partition m (Eq. 2: in-subgraph vs out-of-subgraph neighbours;
 * appendix: P = P_in + P_out; Sec. "Temporal graphs": the partition plus its
 * 1-hop neighbourhood). Canonical form, one valid encoding only:
 *   rows    = local nodes in ascending global id;
 *   columns = relabelled ids: local node -> its rank in V_m, halo node ->
 *             n_local + its rank among halo nodes (ascending global id);
 *   each row holds its self-loop and all neighbours, sorted ascending by
 *   relabelled id, hence every local column precedes every halo column;
 *   split[i] is the offset (into col/val) of row i's first halo column
 *   (= rowptr[i+1] if it has none);
 *   val[k] = A_hat entry, stored as ONE fp32 product isd[i] * isd[j] where
 *   isd[v] = fp32(1 / sqrt(1 + deg(v))) rounded once from fp64.
 * The halo block P_out is also stored transposed (CSR of P_out^T): for halo
 * node u, h_row[h_colptr[u] .. h_colptr[u+1]) are its local neighbours in
 * ascending order with values h_val; h_self[u] = A_hat[u,u] = isd[u]^2.
 * All pointers are device pointers for the compute calls below and host
 * pointers for sat_partition_view_build().
 */
typedef struct sat_part_view {
  int64_t n_local, n_halo, nnz, nnz_halo;
  const int64_t* rowptr;   /* [n_local + 1] */
  const int64_t* split;    /* [n_local]     */
  const int32_t* col;      /* [nnz], values in [0, n_local + n_halo) */
  const float* val;        /* [nnz]         */
  const int64_t* h_colptr; /* [n_halo + 1]  */
  const int32_t* h_row;    /* [nnz_halo], values in [0, n_local) */
  const float* h_val;      /* [nnz_halo]    */
  const float* h_self;     /* [n_halo]      */
} sat_part_view;

/*
 * Parameters omega of one hidden layer's embedding predictor g_omega
 * (Sec. "Embedding Predictor": an RNN-GNN made of an LSTM and a GCN). Device
 * pointers, fp32, row-major, dense (no padding):
 *   Wx [4*d_s, d], Wh [4*d_s, d_s], b [4*d_s]  LSTM, gate blocks stacked i,f,g,o
 *   Wg [d_s, d]                                weight of the GCN hop
 */
typedef struct sat_predictor {
  const float* Wx;
  const float* Wh;
  const float* b;
  const float* Wg;
  int32_t d;    /* embedding width of the layer */
  int32_t d_s;  /* LSTM hidden size: 32, 64 or 128 (bf16 embeddings: 32 or 64) */
  int32_t tau;  /* window length, 1 <= tau <= 8 */
  int32_t bypass; /* nonzero: plain historical embeddings, no correction */
} sat_predictor;

/* ---------------------------------------------------------------- utilities */
const char* sat_status_string(sat_status s); /* static string, never NULL */
int32_t sat_last_hip_error(void); /* hipError_t of this thread's last SAT_EHIP, else 0 */
int32_t sat_version(void);        /* major*10000 + minor*100 + patch */

/* ------------------------------------------------- setup: partition view
 * (Eq. 2; appendix P = P_in + P_out). HOST pointers, runs on the CPU, once
 * per partition. Input: a simple undirected graph as symmetric CSR without
 * self-loops (g_rowptr [N+1], g_col ascending inside a row, ids in [0,N)),
 * the partition vector part[N] and the partition m to view. g_deg (nullable)
 * overrides the neighbour count of every node used for normalisation; NULL
 * means the row lengths of the CSR. (Rows of nodes outside partition m are
 * never read, so a caller that only holds partition m's rows passes them
 * plus g_deg for everybody.)
 * _sizes() reports the four counts; the caller allocates and calls _build(),
 * which fills arrays of exactly those sizes (layout: see sat_part_view;
 * local_ids [n_local] and halo_ids [n_halo] are ascending GLOBAL ids).
 * Errors: SAT_EINVAL on null pointers, N < 0, ids out of range, a
 * non-monotone rowptr, or a self-loop / unsorted row inside partition m.
 */
sat_status sat_partition_view_sizes(int64_t N, const int64_t* g_rowptr, const int32_t* g_col,
                                    const int32_t* part, int32_t m, int64_t* n_local,
                                    int64_t* n_halo, int64_t* nnz, int64_t* nnz_halo);
sat_status sat_partition_view_build(int64_t N, const int64_t* g_rowptr, const int32_t* g_col,
                                    const int32_t* g_deg, const int32_t* part, int32_t m,
                                    int32_t* local_ids, int32_t* halo_ids, int64_t* rowptr,
                                    int64_t* split, int32_t* col, float* val, int64_t* h_colptr,
                                    int32_t* h_row, float* h_val, float* h_self);

/* ------------------------------------------------- pull (Alg. 1 "Pull H_out")
 * out[k, 0:d) = table[ids[k], 0:d) for k in [0, n). A bit-exact copy.
 * table: device, [n_rows, ld_table]; ids: device int32 [n] (repeats allowed);
 * out: device, [n, ld_out]; must not overlap table. Used for the halo rows of
 * the static input features (layer 0), for plain historical embeddings, and
 * to assemble the predictor's window.
 */
sat_status sat_history_gather(const void* table, int64_t n_rows, int64_t ld_table,
                              const int32_t* ids, int64_t n, int32_t d, void* out,
                              int64_t ld_out, int32_t dtype, void* stream);

/* ------------------------------------- push (Alg. 1 "Push computed embeddings")
 * table[ids[k], 0:d) = H[k, 0:d) for k in [0, n). Bit-exact copy; ids must be
 * distinct (otherwise which copy survives is unspecified). Other rows and the
 * columns [d, ld_table) are untouched.
 */
sat_status sat_history_push(void* table, int64_t n_rows, int64_t ld_table, const int32_t* ids,
                            int64_t n, int32_t d, const void* H, int64_t ld_h, int32_t dtype,
                            void* stream);

/* ------ pull of the stale-gradient term (appendix, SAT backward: the second term
 * P_out^T D~^(t-1) W^T of G_H). A partition's local nodes are halo nodes of other
 * partitions; each of those computes P_out^T dAGG for them (sat_spmm_bwd's dH_halo),
 * pushes it into a gradient table with sat_history_push, and one step later the
 * owner adds its rows to its own gradient:
 *   out[k, 0:d) += table[ids[k], 0:d) for k in [0, n), added in fp32 (bf16: one
 * rounding of the sum). ids with repeats are allowed (each k is its own row of
 * out); an id outside [0, n_rows) adds nothing. out must not overlap table.
 * Unlike gather and push this call needs 16-byte aligned rows (SAT_EALIGN).
 */
sat_status sat_history_gather_add(const void* table, int64_t n_rows, int64_t ld_table,
                                  const int32_t* ids, int64_t n, int32_t d, void* out,
                                  int64_t ld_out, int32_t dtype, void* stream);

/* -------------------- embedding predictor g_omega (Eq. 7; Sec. "Embedding Predictor")
 * Writes the predicted halo embeddings H_out_hat into rows [n_local, n_bar)
 * of Hbar [n_bar, ld]:
 *   1. per node u of the partition and its halo, S_u = last hidden state of a
 *      one-layer LSTM (zero initial state) run over u's tau cached embeddings,
 *      oldest first;
 *   2. per halo node u, Delta_u = (A_hat[u,u] S_u + sum over local neighbours v
 *      of A_hat[u,v] S_v) Wg   (one GCN propagation, no activation);
 *   3. H_out_hat[u] = newest cached embedding of u + Delta_u.
 * With w->bypass set, step 3 alone with Delta = 0 (a copy of the newest rows).
 * slots: HOST array of tau DEVICE pointers, oldest first; slot s is a matrix
 * [*, ld_slot]. Row of node k (k in [0, n_bar), local nodes first) inside a
 * slot is ids[k] if ids != NULL (device int32 [n_bar]; lets the call read the
 * history table in place), else k. n_rows_slot bounds the row index.
 * Local rows of Hbar are not touched. Hbar must not overlap any slot.
 * dtype is the element type of the slots and of Hbar; the parameters in *w are
 * fp32. d must be a multiple of 4 (fp32) or 8 (bf16), else SAT_EUNSUPPORTED.
 * Workspace: sat_predict_workspace_bytes(); 256-byte aligned device memory.
 */
int64_t sat_predict_workspace_bytes(int64_t n_local, int64_t n_halo, int32_t d, int32_t d_s,
                                    int32_t tau);
sat_status sat_predict(const sat_part_view* pv, const sat_predictor* w, const void* const* slots,
                       int64_t n_rows_slot, int64_t ld_slot, const int32_t* ids, void* Hbar,
                       int64_t ld, int32_t dtype, void* workspace, int64_t workspace_bytes,
                       void* stream);

/* The two halves of sat_predict as calls of their own (Sec. "Embedding Predictor", Eq. (7)),
 * for callers that cannot hold the whole window dense at once (a coded ring that is decoded a
 * range of rows at a time): the LSTM is row-wise, only the hop needs every node's state.
 *
 * sat_predict_states: step 1 of sat_predict for n_nodes rows: S[k, 0:d_s) (device, fp32,
 * dense [n_nodes, d_s], 16-byte aligned) = last LSTM state over the tau slots of node k, whose
 * row inside a slot is ids[k] if ids != NULL, else k. For a range of nodes the caller passes
 * ids + begin (or slots that hold just that range) and S + begin * d_s. Same restrictions on
 * d, d_s and dtype as sat_predict; w->bypass set is SAT_EINVAL.
 * Workspace: sat_predict_states_workspace_bytes(d, d_s), 256-byte aligned device memory (the
 * re-laid weights; calls on one stream may share it).
 *
 * sat_predict_hop: steps 2 and 3 of sat_predict from S [n_local + n_halo, d_s] (local nodes
 * first): Hbar[n_local + u, 0:d) = newest[row(u), 0:d) + Delta_u, row(u) = halo_ids[u] if
 * halo_ids != NULL (device int32 [n_halo]) else u; rows outside [0, n_rows_newest) leave the
 * output row untouched. `newest` [*, ld_newest] holds the newest cached embedding of the HALO
 * nodes and may be the halo rows of Hbar themselves (newest == Hbar + n_local * ld elements,
 * ld_newest == ld, halo_ids == NULL; d_s <= 64 only): the sum is then formed in place. Any
 * other overlap of the two is SAT_EINVAL.
 * Workspace: sat_predict_hop_workspace_bytes(n_halo, d_s), 256-byte aligned device memory.
 */
int64_t sat_predict_states_workspace_bytes(int32_t d, int32_t d_s);
sat_status sat_predict_states(const sat_predictor* w, const void* const* slots,
                              int64_t n_rows_slot, int64_t ld_slot, const int32_t* ids,
                              int64_t n_nodes, int32_t dtype, float* S, void* workspace,
                              int64_t workspace_bytes, void* stream);
int64_t sat_predict_hop_workspace_bytes(int64_t n_halo, int32_t d_s);
sat_status sat_predict_hop(const sat_part_view* pv, const sat_predictor* w, const float* S,
                           const void* newest, int64_t n_rows_newest, int64_t ld_newest,
                           const int32_t* halo_ids, void* Hbar, int64_t ld, int32_t dtype,
                           void* workspace, int64_t workspace_bytes, void* stream);

/* sat_predict with the LSTM's input projections kept between calls. Consecutive windows of
 * the sliding window of Sec. "Embedding Predictor" share all but their newest slot, and
 * x_s Wx^T of a slot does not depend on the slot's position in the window; so the caller
 * keeps, per ring slot, a matrix proj [n_bar, 4 d_s] fp32 (row k = node k in local-then-
 * halo order, gate blocks i, f, g, o; no padding) that this call reads or writes:
 *   proj: HOST array of tau DEVICE pointers, oldest slot first (entries may be NULL:
 *         nothing is kept for that slot);
 *   n_proj_valid: the first n_proj_valid slots of the window are taken from proj (their
 *         cached rows and the Wx tiles are not read at all); every later slot except the
 *         window's first is multiplied out and, if its pointer is not NULL, written.
 *         0 <= n_proj_valid < tau (the newest slot is always new).
 * A cached matrix is valid as long as the slot's rows, the id list and Wx are unchanged:
 * the caller invalidates it (passes a smaller n_proj_valid) after a push into the slot or
 * an update of the predictor. The result is bit-identical to sat_predict's: the cached
 * value is the same fp32 sum in the same order. d_s = 32 or 64 (else SAT_EUNSUPPORTED);
 * with w->bypass the cache is ignored. Everything else as sat_predict. */
sat_status sat_predict_cached(const sat_part_view* pv, const sat_predictor* w,
                              const void* const* slots, int64_t n_rows_slot, int64_t ld_slot,
                              const int32_t* ids, void* Hbar, int64_t ld, int32_t dtype,
                              float* const* proj, int32_t n_proj_valid, void* workspace,
                              int64_t workspace_bytes, void* stream);

/* ------- compression of stored embeddings (Sec. "Data Compression for Historical
 * Embedding Storage"). Every value v is rounded to `precision` decimal places,
 * q = floor(v * 10^precision + 1/2) (three fp32 operations, each correctly rounded),
 * and q is written in the Encoded Polyline Algorithm Format's character coding:
 * shift left one bit and invert if negative, 5-bit groups from the low end, 0x20 set
 * on every group but the last, plus 63 (bytes 63..126). Values are coded one by one,
 * a row is the concatenation of its d codes, row k occupies bytes
 * [row_off[k], row_off[k+1]) of `codes`. |q| saturates at 2^30 (the largest magnitude
 * whose shifted code fits 32 bits for either sign; +-inf land there), NaN codes as 0.
 * Lossy: |decoded - v| <= 10^-precision / 2 (plus fp32 rounding) for |v| 10^precision < 2^30.
 *   _plan    row_off[0..n] (device int64) from the dense rows H [n, ld_h]: code sizes,
 *            then an exclusive scan; row_off[n] is the total number of bytes. The caller
 *            reads it back to size `codes`.
 *   _encode  writes the codes of the same H; rows that would end beyond `capacity`
 *            bytes are not written.
 *   sat_history_decompress  out[k, 0:d) = decoded row ids[k] (ids == NULL: row k) of a
 *            coded table of n_rows rows, value = float(q) / 10^precision (one correctly
 *            rounded division; bf16: rounded again to nearest-even). The pull of a coded
 *            table: gather and decode in one pass. d <= 2340.
 * precision in [0, 9]. Workspace (_plan only): sat_history_compress_workspace_bytes(n),
 * 8-byte aligned.
 */
int64_t sat_history_compress_workspace_bytes(int64_t n);
sat_status sat_history_compress_plan(const void* H, int64_t ld_h, int64_t n, int32_t d,
                                     int32_t precision, int32_t dtype, int64_t* row_off,
                                     void* workspace, int64_t workspace_bytes, void* stream);
sat_status sat_history_compress_encode(const void* H, int64_t ld_h, int64_t n, int32_t d,
                                       int32_t precision, int32_t dtype, const int64_t* row_off,
                                       uint8_t* codes, int64_t capacity, void* stream);
sat_status sat_history_decompress(const uint8_t* codes, const int64_t* row_off, int64_t n_rows,
                                  const int32_t* ids, int64_t n, int32_t d, int32_t precision,
                                  int32_t dtype, void* out, int64_t ld_out, void* stream);

/* ------- training of the embedding predictor (Eq. 11; mini-batches of Eq. 12; Alg. 1
 * "embedding predictor update"). One hidden layer's predictor, one partition.
 * The partition knows this step's fresh embeddings of its LOCAL nodes, so the
 * predictor is supervised there: for local node v
 *   pred[v] = newest cached embedding of v + (sum_u A_hat[v,u] S_u) Wg,
 * the sum over row v of [P_in | P_out] (self-loop, local and halo neighbours), S as
 * in sat_predict;
 *   loss = sum_v weight[v] |pred[v] - target[v]|^2 / (d * sum_v weight[v]).
 * slots / n_rows_slot / ld_slot / ids: as for sat_predict (the window the prediction
 * was made from, i.e. the ring before this step's push). target: device
 * [n_local, ld_target], the fresh embeddings (a constant of this call). weight:
 * device float [n_local] or NULL (all ones); a 0/1 vector selects a mini-batch.
 * Outputs (device, fp32, dense): dWx [4 d_s, d], dWh [4 d_s, d_s], db [4 d_s],
 * dWg [d_s, d], loss [1]; all overwritten. Reductions run in a fixed order.
 * dtype: element type of the slots and of target (SAT_BF16: bfloat16 tables; everything
 * computed here, the parameters and the outputs stay fp32). d_s = 32, 64 or 128 (SAT_BF16:
 * 32 or 64) and d % 4 == 0 (SAT_BF16: d % 8 == 0), else SAT_EUNSUPPORTED.
 * Workspace: sat_predictor_train_workspace_bytes(); 256-byte aligned.
 */
int64_t sat_predictor_train_workspace_bytes(int64_t n_local, int64_t n_halo, int32_t d,
                                            int32_t d_s, int32_t tau);
sat_status sat_predictor_grad(const sat_part_view* pv, const sat_predictor* w,
                              const void* const* slots, int64_t n_rows_slot, int64_t ld_slot,
                              const int32_t* ids, const void* target, int64_t ld_target,
                              const float* weight, int32_t dtype, float* dWx, float* dWh, float* db,
                              float* dWg, float* loss, void* workspace, int64_t workspace_bytes,
                              void* stream);
/* param[i] -= lr * grad[i] for i in [0, n): the plain gradient step of Alg. 1
 * (theta with eta_1, omega with eta_2). Device pointers, fp32. */
sat_status sat_sgd_update(float* param, const float* grad, int64_t n, float lr, void* stream);

/* --------------- aggregation (appendix, SAT forward: P_in H_in + P_out H_out_hat)
 * AGG [n_local, ld_out] = [P_in | P_out] * Hbar [n_bar, ld_in], d columns.
 * AGG must not overlap Hbar.
 */
int64_t sat_spmm_workspace_bytes(const sat_part_view* pv_sizes_only, int32_t d);
sat_status sat_spmm_fwd(const sat_part_view* pv, const void* Hbar, int64_t ld_in, int32_t d,
                        int32_t dtype, void* AGG, int64_t ld_out, void* workspace,
                        int64_t workspace_bytes, void* stream);

/* ---------------- transpose aggregation (appendix, SAT backward: P_in^T D W^T)
 * dH_local [n_local, ld_out] = P_in^T * dAGG [n_local, ld_in]. P_in is
 * symmetric (A_hat is, and local ids label rows and columns alike), so this
 * walks the local-column prefix [rowptr[i], split[i]) of every row.
 * If dH_halo != NULL also dH_halo [n_halo, ld_halo] = P_out^T * dAGG through
 * the transposed halo block. The SAT step itself never uses dH_halo: predicted
 * halo embeddings are constants of the step.
 */
sat_status sat_spmm_bwd(const sat_part_view* pv, const void* dAGG, int64_t ld_in, int32_t d,
                        int32_t dtype, void* dH_local, int64_t ld_out, void* dH_halo,
                        int64_t ld_halo, void* workspace, int64_t workspace_bytes, void* stream);

/* --------------------- feature transform (appendix: Z = (P H) W, H' = sigma(Z))
 * H [n, ld_h] = act(AGG [n, ld_a] * W [d_in, ld_w]) with d_out columns;
 * act = SAT_ACT_RELU on hidden layers, SAT_ACT_IDENTITY on the last. No bias.
 */
sat_status sat_dense_fwd(const void* AGG, int64_t ld_a, int64_t n, int32_t d_in, int32_t d_out,
                         const void* W, int64_t ld_w, int32_t act, int32_t dtype, void* H,
                         int64_t ld_h, void* stream);

/* ------ backward of the feature transform (appendix: D = G o sigma'(Z),
 * G_W = (P H)^T D, gradient to the aggregate D W^T)
 *   dZ   = dH o [Hout > 0]     (act = RELU; Hout is the forward's output, and
 *                               Hout > 0 exactly where Z > 0) or dH (IDENTITY,
 *                               Hout may be NULL);
 *   dW   [d_in, ld_dw] = AGG^T dZ   (fp32; reduced over all n rows in a fixed
 *                               order, so results are run-to-run identical);
 *   dAGG [n, ld_da]    = dZ W^T     (skipped if dAGG == NULL, e.g. layer 0).
 * dW == NULL skips the weight gradient (AGG may then be NULL and no workspace
 * is needed): only dAGG is computed.
 * Workspace: sat_dense_bwd_workspace_bytes(); 256-byte aligned device memory.
 * The first call with dW != NULL on a device raises that device's limit on dynamic
 * LDS for the weight-gradient kernel (a HIP runtime setting, no allocation; failure is
 * SAT_EHIP): make one such call per device before capturing the call into a HIP graph.
 */
int64_t sat_dense_bwd_workspace_bytes(int64_t n, int32_t d_in, int32_t d_out);
sat_status sat_dense_bwd(const void* dH, int64_t ld_dh, const void* Hout, int64_t ld_ho,
                         const void* AGG, int64_t ld_a, const void* W, int64_t ld_w, int64_t n,
                         int32_t d_in, int32_t d_out, int32_t act, int32_t dtype, float* dW,
                         int64_t ld_dw, void* dAGG, int64_t ld_da, void* workspace,
                         int64_t workspace_bytes, void* stream);

/* ---------------- local loss gradient (Eq. 4 with softmax cross-entropy)
 * dH [n, ld_dh] = (softmax(HL[n, ld_hl], over n_classes columns) - onehot(y)) / n;
 * y: device int32 [n] in [0, n_classes). If loss != NULL (device float[1]) the
 * mean cross-entropy is written there (summed in a fixed order).
 * Workspace: sat_loss_workspace_bytes(n) bytes, 256-byte aligned (only
 * needed when loss != NULL).
 */
int64_t sat_loss_workspace_bytes(int64_t n);
sat_status sat_loss_grad(const void* HL, int64_t ld_hl, int64_t n, int32_t n_classes,
                         const int32_t* y, int32_t dtype, void* dH, int64_t ld_dh, float* loss,
                         void* workspace, int64_t workspace_bytes, void* stream);

/* sat_loss_grad for callers that cannot allocate device memory or carry a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same kernels and results, with the per-block partial sums of the loss in an
 * array the library holds statically on every GPU it runs on (1 MiB per GPU, kept until
 * the process ends) instead of a workspace. Calls no hipMalloc / hipFree. Limit:
 * n <= sat_loss_grad_static_max_rows() (33,554,432), beyond it SAT_EUNSUPPORTED and
 * nothing is enqueued. Every call on one GPU shares that GPU's array: two calls that may
 * overlap in time on one GPU (different streams) race on it; calls on one stream do not.
 * Nothing in the array has to be cleared between calls (each call overwrites the part it
 * reads). The first call on a device looks the array's address up (a HIP runtime query,
 * no allocation); make one call per device before capturing a graph. */
int64_t sat_loss_grad_static_max_rows(void);
sat_status sat_loss_grad_static(const void* HL, int64_t ld_hl, int64_t n, int32_t n_classes,
                                const int32_t* y, int32_t dtype, void* dH, int64_t ld_dh,
                                float* loss, void* stream);

/* =================== graph attention backbone (second backbone of the paper's
 * experiments; the layer is Eq. 1 / Eq. 2 with attention as the aggregation
 * function, defined as in Velickovic et al., "Graph Attention Networks",
 * Eq. 1-4). One layer on a partition, Hbar = [local rows ; halo rows]:
 *   Z = Hbar W                        sat_dense_fwd over all n_local + n_halo rows
 *   el, er                            sat_gat_scores
 *   H' = act(sum_j alpha_ij Z_j)      sat_gat_aggregate_fwd
 * and backwards sat_gat_aggregate_bwd (dZ, gradients of the attention
 * vectors), then sat_dense_bwd (dW over all rows, dHbar = dZ W^T over the local
 * rows). The neighbourhood of local node i is row i of the view's CSR
 * (self-loop included); the stored values A_hat are not used.
 *
 * Shapes: d = heads * d_head columns, head k owning columns [k d_head, (k+1) d_head).
 * Supported: heads in {1, 2, 4, 8}; d <= 256; for heads > 1, d_head / 4 a power of
 * two (else SAT_EUNSUPPORTED). Scores, statistics and attention vectors are fp32
 * whatever the storage type; sums are fp32. All pointers are device pointers;
 * el, er, stats 16-byte aligned; matrices as everywhere (16-byte aligned rows).
 */

/* Attention scores: er[r, k] = <a_src[k], Z[r, head k]> for r < n and
 * el[r, k] = <a_dst[k], Z[r, head k]> for r < n_dst (n_dst <= n: the local rows).
 * a_dst, a_src: [heads * d_head] fp32. el: [n_dst, heads], er: [n, heads]. */
sat_status sat_gat_scores(const void* Z, int64_t ld_z, int64_t n, int64_t n_dst, int32_t heads,
                          int32_t d_head, const float* a_dst, const float* a_src, int32_t dtype,
                          float* el, float* er, void* stream);

/* Edge softmax and aggregation for the n_local rows of the view:
 *   e_ij = LeakyReLU(el[i] + er[j]; slope), alpha_ij = softmax over row i's entries,
 *   H[i] = act(sum_j alpha_ij Z[j]) per head (act as in sat_dense_fwd).
 * Z: [n_local + n_halo, ld_z]; H: [n_local, ld_h]; stats: [n_local, heads, 2] fp32
 * receives (max_j e_ij, 1 / sum_j exp(e_ij - max)) for the backward. A row without
 * entries gives H[i] = 0, stats (0, 0). */
sat_status sat_gat_aggregate_fwd(const sat_part_view* pv, const void* Z, int64_t ld_z,
                                 int32_t heads, int32_t d_head, int32_t dtype, const float* el,
                                 const float* er, float slope, int32_t act, void* H, int64_t ld_h,
                                 float* stats, void* stream);

/* Backward of scores + aggregation. With dOUT = dH o [H > 0] (act = RELU; H is the
 * forward's output) or dH (IDENTITY; H may be NULL):
 *   dalpha_ij = <dOUT_i, Z_j>, ds_ij = alpha_ij (dalpha_ij - sum_k alpha_ik dalpha_ik)
 *               LeakyReLU'(el_i + er_j), d_el_i = sum_j ds_ij, d_er_j = sum_i ds_ij,
 *   dZ[j]  = sum_i alpha_ij dOUT_i + d_er_j a_src + d_el_j a_dst  (last term: local j),
 *   da_dst = sum_i d_el_i Z_i, da_src = sum_j d_er_j Z_j          ([heads * d_head] fp32).
 * dZ: [n_local + n_halo, ld_dz], every row written. Needs the view's transposed halo
 * block (h_colptr, h_row) and relies on the local block's pattern being symmetric.
 * Sums run in a fixed order (run-to-run identical results).
 * Workspace: sat_gat_aggregate_bwd_workspace_bytes(); 256-byte aligned. */
int64_t sat_gat_aggregate_bwd_workspace_bytes(int64_t n_local, int64_t n_halo, int32_t heads,
                                              int32_t d_head, int32_t dtype);
sat_status sat_gat_aggregate_bwd(const sat_part_view* pv, const void* Z, int64_t ld_z,
                                 int32_t heads, int32_t d_head, int32_t dtype, const float* el,
                                 const float* er, const float* stats, float slope, int32_t act,
                                 const void* dH, int64_t ld_dh, const void* H, int64_t ld_h,
                                 const float* a_dst, const float* a_src, void* dZ, int64_t ld_dz,
                                 float* da_dst, float* da_src, void* workspace,
                                 int64_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SAT_H_ */
