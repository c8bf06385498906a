/*
 * lcrwmd - Linear-Complexity Relaxed Word Mover's Distance on one AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of arXiv:1711.07227.  Notation is the paper's
 * (Tables I and II): v vocabulary size, m embedding dimension, E the v x m embedding
 * matrix, X1 the resident ("database") histograms, X2 the transient ("query")
 * histograms, Z the per-word minimum distances, D the distance matrix, R the top-k
 * result.  n = rows of X1, q = rows of X2.
 *
 * Conventions that hold for every call
 *   - Pointers named in lcrwmd_csr / lcrwmd_emb and every Z, D, R, workspace pointer
 *     are DEVICE pointers on the context's device, unless a comment says "host".
 *   - The caller owns every buffer.  The library allocates no device memory and frees
 *     nothing it is given; temporary storage comes from the caller's workspace
 *     (size from lcrwmd_workspace_bytes).  The workspace must be 256-byte aligned.
 *   - Work is enqueued on the hipStream_t passed as `hip_stream` (NULL = the default
 *     stream) and is asynchronous with respect to the host, except where a call's
 *     comment lists a synchronisation.
 *   - Every function returns an lcrwmd_status.  Argument errors are detected before
 *     anything is launched.  The library never aborts, throws or prints; the text
 *     for the last failure of a context is available from lcrwmd_last_error.
 *   - A context is not thread safe; use one per host thread.  Calls on the same
 *     stream may share a workspace; calls on different streams must not.
 *   - Histograms: CSR with int64 row_ptr (row_ptr[0] == 0), int32 col_idx strictly
 *     increasing inside a row and < cols, fp32 val > 0 summing to 1 per row
 *     (Sec. II: L1-normalised histograms; Sec. III: rows of X store the weights of the
 *     unique words).  Every row must hold at least one word: the minimum over an empty
 *     word set is undefined.  The library does not renormalise weights.
 */
#ifndef LCRWMD_H
#define LCRWMD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lcrwmd_ctx lcrwmd_ctx;   /* opaque */

typedef enum {
    LCRWMD_OK = 0,
    LCRWMD_EINVAL = 1,        /* null pointer, negative size, bad leading dimension, bad option      */
    LCRWMD_EBADCSR = 2,       /* validation on: row_ptr not monotone, column out of range/unsorted   */
    LCRWMD_EEMPTYDOC = 3,     /* a histogram without words                                           */
    LCRWMD_EWORKSPACE = 4,    /* workspace missing, misaligned or too small                          */
    LCRWMD_EUNSUPPORTED = 5,  /* e.g. k larger than the supported maximum                            */
    LCRWMD_EHIP = 6,          /* a HIP runtime call failed; see lcrwmd_last_error                    */
    LCRWMD_ENOCONVERGE = 7    /* a transport problem used up its augmentation budget (lcrwmd_wmd_*)  */
} lcrwmd_status;

/* Storage type of embedding values.  Accumulation is always fp32. */
typedef enum { LCRWMD_F32 = 0, LCRWMD_BF16 = 1,
               LCRWMD_BF16X3 = 2   /* only as lcrwmd_options.compute, never as a storage type */
} lcrwmd_dtype;

/* A set of histograms X (Sec. III, Fig. 2): one sparse row per document. */
typedef struct {
    int64_t rows, cols, nnz;        /* cols == v                                                     */
    const int64_t* row_ptr;         /* device, [rows + 1]                                            */
    const int32_t* col_idx;         /* device, [nnz]                                                 */
    const float* val;               /* device, [nnz]                                                 */
    const int64_t* row_ptr_host;    /* HOST copy of row_ptr, or NULL.  When NULL, calls that plan
                                       batches from the row lengths (lcrwmd_rwmd, lcrwmd_rwmd_topk)
                                       copy row_ptr back themselves, which synchronises the stream. */
} lcrwmd_csr;

/* The embedding matrix E (Sec. III): row w holds the m-vector of word w, row-major. */
typedef struct {
    const void* data;               /* device, v rows of m values, consecutive rows `ld` values apart */
    int64_t v, m, ld;               /* ld >= m                                                       */
    lcrwmd_dtype dtype;             /* LCRWMD_F32: float; LCRWMD_BF16: 16-bit bfloat16               */
} lcrwmd_emb;

typedef struct {
    int validate;                   /* 1: check every CSR on the device before use (one extra stream
                                       synchronisation per call); 0 (default): trust the caller       */
    int compute;                    /* lcrwmd_dtype the first-phase contraction multiplies in.
                                       LCRWMD_F32 (default for fp32 E): fp32 MFMA.  LCRWMD_BF16: E is
                                       rounded to bf16 (round-to-nearest-even) unless already bf16,
                                       products accumulate in fp32.  bf16 E always computes in bf16.
                                       The bf16 kernels take m <= 300; wider embeddings are computed in
                                       fp32 on an fp32 copy of the bf16 values (same results, workspace
                                       4 v m bytes more).
                                       LCRWMD_BF16X3 (fp32 E, m <= 300; otherwise it means
                                       LCRWMD_F32): every fp32 value x is split into hi = bf16(x) and
                                       lo = bf16(x - hi) and a product is taken as hi*hi + hi*lo + lo*hi
                                       on the bf16 matrix units with fp32 accumulation; norms stay fp32.
                                       The dropped lo*lo term is 2^-16 relative: distances agree with
                                       fp32 arithmetic to about 1e-6 relative for unit-norm rows.      */
    int64_t max_query_batch;        /* upper limit on histograms of X2 per pass (Sec. IV, many-to-many:
                                       X2 is divided into batches); 0 = chosen from the workspace     */
    int64_t max_db_batch;           /* same for the database rows handled per pass of the swapped
                                       direction; 0 = chosen from the workspace                      */
    int dedup;                      /* 0 (default): the per-entry form - distances are recomputed per stored
                                       entry, as the paper's two phases do.
                                       1: the table form where it can run - the Euclidean distances between
                                       the distinct words of the database and the distinct words of a range
                                       of queries are computed once, as one table (the operator of Sec. III
                                       on the two reduced vocabularies), and both directions take their
                                       minima from it.  Same result up to fp32 summation order.  The table
                                       lives in the workspace (4 bytes x distinct database words x distinct
                                       query words); when it does not fit, or for fp32 E with m < 208 or
                                       m > 300, the per-entry form runs instead.
                                       2: the library picks, per range of queries, the form its cost model
                                       expects to be faster (contraction flops of the per-entry form against
                                       the table's build and its two bandwidth-bound passes; Sec. III-B
                                       discusses this trade-off); more than 4,096 queries in one call always
                                       take the per-entry form.
                                       lcrwmd_forms_ran tells which form(s) the last call used.        */
} lcrwmd_options;

/* Create a context bound to HIP device `device`.  No device memory is allocated. */
lcrwmd_status lcrwmd_create(lcrwmd_ctx** out, int device);
void lcrwmd_destroy(lcrwmd_ctx* ctx);

/* Text for the last non-OK status returned on this context (owned by the context; "" if none). */
const char* lcrwmd_last_error(const lcrwmd_ctx* ctx);

/* Forms used by the last lcrwmd_rwmd / lcrwmd_rwmd_topk / lcrwmd_rwmd_reduce call on this context: bit 0 set when a
   range of queries ran the per-entry form, bit 1 when one ran the table form (see lcrwmd_options.dedup). */
int lcrwmd_forms_ran(const lcrwmd_ctx* ctx);

/* Copy the options in / out.  Defaults: validate 0, compute LCRWMD_F32, batches 0, dedup 0. */
lcrwmd_status lcrwmd_set_options(lcrwmd_ctx* ctx, const lcrwmd_options* opt);
lcrwmd_status lcrwmd_get_options(const lcrwmd_ctx* ctx, lcrwmd_options* opt);

/*
 * Workspace, in bytes, that lets every entry point below run the given problem with its
 * preferred batch sizes.  lcrwmd_rwmd and lcrwmd_rwmd_topk also run with less, in smaller
 * batches, down to a floor below which they return LCRWMD_EWORKSPACE.
 * nnz_db / nnz_q are the stored entries of X1 / X2; k = 0 when no top-k is wanted.
 * With dedup = 1 the figure includes the word-pair table at its upper bound (distinct words <=
 * stored entries); with dedup = 2 it does so where the cost model picks the table form at those
 * bounds and the table then fits three quarters of the device's memory, and is the per-entry
 * form's figure otherwise.  Any size that suffices without the
 * option still works: a range of queries whose table does not fit runs the per-entry form.
 */
lcrwmd_status lcrwmd_workspace_bytes(lcrwmd_ctx* ctx, int64_t v, int64_t m, int64_t n, int64_t nnz_db,
                                     int64_t q, int64_t nnz_q, lcrwmd_dtype emb_dtype, int k,
                                     size_t* out_bytes);

/*
 * First phase of LC-RWMD in its many-to-many form (Sec. IV, Fig. 6, and the paragraph
 * "Many-to-many LC-RWMD"): for every vocabulary word w and every histogram j of `queries`
 *
 *     Z[w * ldz + j] = min over the words a of queries[j] of || E[w] - E[a] ||_2
 *
 * i.e. the row-wise minima of E o T2 taken separately for each j.  Z is v x queries->rows
 * fp32, row-major, ldz >= queries->rows.  queries->val is not read.  The distance is
 * evaluated as sqrt(max(|x|^2 + |y|^2 - 2 x.y, 0)) with the x.y contraction on the matrix
 * cores, and is exactly 0 where w itself occurs in queries[j].
 * No host synchronisation (unless validation is on).
 */
lcrwmd_status lcrwmd_phase1_mindist(lcrwmd_ctx* ctx, const lcrwmd_emb* E, const lcrwmd_csr* queries,
                                    float* Z, int64_t ldz, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Second phase (Sec. IV, Fig. 7): the sparse histogram matrix times the dense minima,
 *
 *     S[i][j] = sum over stored p of X[i] of  X.val[p] * Z[X.col_idx[p] * ldz + j],   j < ncols
 *
 * combine == 0:  D[i * ldd + j]  = S[i][j]                       (D is X->rows x ncols)
 * combine == 1:  D[i * ldd + j]  = max(D[i * ldd + j], S[i][j])
 * combine == 2:  D[j * ldd + i]  = max(D[j * ldd + i], S[i][j])  (D is ncols x X->rows: the
 *                transposed maximum D = max(D1, D2^T) of Sec. IV, used after swapping the sets)
 * Z is X->cols x ncols fp32 row-major.  Needs no workspace.  No host synchronisation.
 */
lcrwmd_status lcrwmd_phase2_spmm(lcrwmd_ctx* ctx, const lcrwmd_csr* X, const float* Z, int64_t ldz,
                                 int64_t ncols, float* D, int64_t ldd, int combine, void* hip_stream);

/*
 * The full bound (Sec. III "Solving the RWMD problem", Sec. IV): for database doc i and query j
 *
 *     D[i * ldd + j] = max( sum_p X1[i][p] * min_{a in X2[j]} ||E[p]-E[a]|| ,
 *                           sum_a X2[j][a] * min_{p in X1[i]} ||E[p]-E[a]|| )
 *
 * D is n x q fp32 row-major (n = database->rows, q = queries->rows, ldd >= q).  Both directions
 * run the two phases, the second one with the sets swapped; words that do not occur in the
 * set that plays X1 are dropped from the vocabulary of that pass (Sec. IV, vocabulary
 * reduction).  The first-phase minima of all queries are kept in the workspace (in ranges of
 * queries when it is smaller than lcrwmd_workspace_bytes asks for, each range then repeating the
 * swapped pass), and the database rows are handled in blocks: forward second phase, swapped
 * first and second phase and the maximum, block by block.  Results do not depend on the
 * batch sizes.
 * Synchronises the stream to read back the two vocabulary sizes, which decide grids and batch
 * sizes (and before that once more when it has to fetch the row pointers because no host
 * copies were given); everything else is asynchronous.
 */
lcrwmd_status lcrwmd_rwmd(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                          const lcrwmd_emb* E, float* D, int64_t ldd, void* ws, size_t ws_bytes,
                          void* hip_stream);

/*
 * The same bound by the quadratic-complexity method the paper starts from (Sec. III "Solving the RWMD problem";
 * Sec. V, first GPU mapping): for every pair, C = T1,i o T2,j, its row minima dotted with F1,i, its column minima
 * dotted with F2,j, the larger of the two.  The T1,i of a block of database histograms are stacked into one matrix
 * and multiplied with the stacked T2,j of all queries, as in Sec. V - but nothing is shared between histograms:
 * a word is paired with a query (a database histogram) once per histogram it occurs in, 2 nnz(X1) nnz(X2) m flops
 * per evaluation of all C.  C is evaluated twice, once per kind of minimum: the minima are taken inside the
 * contraction along one dimension, and C itself (nnz(X1) x nnz(X2) values) is never stored.  Same D as lcrwmd_rwmd
 * up to fp32 summation order; it exists as the comparison the paper draws (Sec. VI: LC-RWMD is faster by about the
 * average histogram size).  Arithmetic follows the compute option.  Synchronises only to fetch row pointers.
 */
lcrwmd_status lcrwmd_rwmd_quadratic_workspace_bytes(lcrwmd_ctx* ctx, int64_t v, int64_t m, int64_t n, int64_t nnz_db,
                                                    int64_t q, int64_t nnz_q, lcrwmd_dtype emb_dtype, size_t* out_bytes);
lcrwmd_status lcrwmd_rwmd_quadratic(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                                    const lcrwmd_emb* E, float* D, int64_t ldd, void* ws, size_t ws_bytes,
                                    void* hip_stream);

/*
 * Top-k on the same bound (Sec. III: the k smallest distances of a query and the positions of
 * the respective database histograms, stored in an n2 x k matrix R): for each query j,
 * R_idx[j * k + r] / R_dist[j * k + r], r < k, are the database rows with the r-th smallest
 * D[.][j] and those distances, ordered by (distance, row index) ascending.  D is never formed:
 * the bound of one block of database rows (at most 16,384, option max_db_batch) lives in a tile
 * of the workspace just long enough to receive both directions and to be merged into the running
 * lists.  1 <= k <= min(n, 64).  Same synchronisation as lcrwmd_rwmd, once per range of queries.
 */
lcrwmd_status lcrwmd_rwmd_topk(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                               const lcrwmd_emb* E, int k, int32_t* R_idx, float* R_dist,
                               void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The all-pairs job within one set of histograms (Sec. IV, "Many-to-many LC-RWMD", with X2 = X1: the set is
 * compared with itself, `batch` histograms at a time): for every histogram i of `docs`
 *
 *     R_idx[i*k .. i*k + k-1], R_dist[...]  its k nearest histograms of the set by the bound D of lcrwmd_rwmd,
 *                                           ascending by (distance, index); itself included, at distance 0
 *     dist_sum[i]                           the sum of D(i, j) over all j of the set, accumulated in fp64
 *
 * (k = 0: sums only; dist_sum = NULL: lists only).  The n x n matrix is never formed.  The bound is the
 * maximum of the two one-sided bounds and therefore symmetric, D(i, j) = D(j, i): a batch is compared only
 * with the histograms from its own first one on, and every tile of distances updates the lists and sums of
 * its columns (the batch) and of its rows (the later histograms) - half the work of n / batch calls of
 * lcrwmd_rwmd_reduce.  D(i, j) is evaluated once, with the histogram of the smaller batch as the query: a
 * list can differ from lcrwmd_rwmd_reduce's in the order of distances that agree to fp32 rounding.
 * batch: histograms per pass (at most 4,096 with dedup = 1); 0 = the largest power of two up to 65,536 whose
 * workspace figure fits ws_bytes (larger batches share more of their words and cost less in total: the
 * 1,000,000-document job of the benchmark set takes 39 s in batches of 4,096, 30 s in batches of 16,384 and
 * 24.5 s in batches of 65,536, for which the workspace figure is 171 GB).  Workspace:
 * lcrwmd_workspace_bytes with q = batch and nnz_q = the most stored entries of `batch` consecutive rows;
 * LCRWMD_EWORKSPACE if it does not suffice (nothing useful is in the outputs then).  docs as for lcrwmd_rwmd;
 * R_idx, R_dist: n x k; dist_sum: n doubles.  Results do not depend on timing; they do depend on `batch`
 * and on the database-block option in the last bits of sums and in the order of near-ties.
 */
lcrwmd_status lcrwmd_rwmd_self(lcrwmd_ctx* ctx, const lcrwmd_csr* docs, const lcrwmd_emb* E, int64_t batch, int k,
                               int32_t* R_idx, float* R_dist, double* dist_sum, void* ws, size_t ws_bytes,
                               void* hip_stream);

/*
 * The bound reduced on the device, for jobs whose n x q matrix is too large to keep (Sec. IV, many-to-many
 * LC-RWMD in batches; Sec. III, top-k): lcrwmd_rwmd_topk's lists (when k > 0; R_idx / R_dist may be NULL when
 * k == 0) and / or, when col_sum is not NULL, the column sums
 *     col_sum[j] = sum over all database rows i of D[i][j]         (device, q doubles, fp64 accumulation
 *                                                                   of the fp32 distances in a fixed order)
 * - a checksum of everything the call computed.  Blocks of database rows as in lcrwmd_rwmd_topk.
 */
lcrwmd_status lcrwmd_rwmd_reduce(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                                 const lcrwmd_emb* E, int k, int32_t* R_idx, float* R_dist, double* col_sum,
                                 void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Top-k of an existing distance matrix: D is n x q fp32 row-major (ldd >= q); outputs as in
 * lcrwmd_rwmd_topk.  The workspace is optional (ws may be NULL): with it the rows of D are
 * split over more workgroups and the partial lists merged.  No host synchronisation.
 */
lcrwmd_status lcrwmd_topk(lcrwmd_ctx* ctx, const float* D, int64_t n, int64_t q, int64_t ldd, int k,
                          int32_t* R_idx, float* R_dist, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * lcrwmd_topk for callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same results bit for
 * bit.  The partial lists of the row splits live in a file-scope device array of 8 MiB that every GPU the library runs
 * on holds until the process ends; its address on the context's device is looked up once, in lcrwmd_create.  The call
 * allocates and frees nothing.  Problems whose partial lists (what lcrwmd_topk would take from its workspace:
 * 8 q k bytes per row split, at most 64 splits) exceed the array return LCRWMD_EWORKSPACE and launch nothing.
 * All calls on one GPU share that GPU's array, whatever their context or stream: calls that overlap in time on one GPU
 * race; calls ordered on one stream do not.  Nothing in the array has to start at zero (every slot that is read is
 * written by the same call first).  No host synchronisation.
 */
lcrwmd_status lcrwmd_topk_noalloc(lcrwmd_ctx* ctx, const float* D, int64_t n, int64_t q, int64_t ldd, int k,
                                  int32_t* R_idx, float* R_dist, void* hip_stream);

/*
 * Per-kernel timing for benchmarks (not part of the method).  Between lcrwmd_profile_begin and
 * lcrwmd_profile_end every launch of the first-phase contraction kernel and of the second-phase
 * SpMM kernel made through this context is bracketed by HIP events on the stream it is launched
 * on.  lcrwmd_profile_end synchronises the device, sums the event times and stops recording.
 * Work figures are algorithmic: first-phase flops = 2 * vocabulary rows * stored tokens * m per
 * launch (padding, norms and the epilogue earn nothing); second-phase bytes = the CSR arrays,
 * the rows of Z and the output, each counted once per launch; gather bytes = 4 * stored
 * entries * columns (what the lanes actually load from Z through the caches).
 */
typedef struct {
    double phase1_ms;  int64_t phase1_launches;  double phase1_flops;
    double phase2_ms;  int64_t phase2_launches;  double phase2_bytes;  double phase2_gather_bytes;
    /* dedup option: the table build counts as first-phase work (2 * distinct database words * distinct query
       words * m flops); the two table passes are timed here, bytes = table rows streamed + outputs. */
    double table_fwd_ms;  int64_t table_fwd_launches;  double table_fwd_bytes;
    double table_rev_ms;  int64_t table_rev_launches;  double table_rev_bytes;
    /* lcrwmd_wmd_pairs / lcrwmd_wmd_topk: the transport solver (it also forms its cost matrices) */
    double emd_ms;  int64_t emd_launches;  double emd_pairs;
    /* lcrwmd_wmd_topk: survivors whose solve stopped early because a lower bound passed the cut-off */
    double emd_abandoned;
    /* the part of phase1_ms / phase1_flops spent in the pass with the two sets swapped (Sec. IV) */
    double phase1_swapped_ms;  double phase1_swapped_flops;
} lcrwmd_profile;
lcrwmd_status lcrwmd_profile_begin(lcrwmd_ctx* ctx);
lcrwmd_status lcrwmd_profile_end(lcrwmd_ctx* ctx, lcrwmd_profile* out);

/*
 * Diagnostic for benchmarks (not part of the method): the rate the matrix cores sustain for the first phase's MFMA
 * shape on this device - v_mfma_f32_32x32x16_bf16 (LCRWMD_BF16) or v_mfma_f32_32x32x2_f32 (LCRWMD_F32) - in a loop
 * of nothing but MFMAs running for about `seconds` on every CU.  random_data: operands are random values of
 * magnitude 0.5 .. 1 (1) or all zero (0): under sustained load on data that toggles, the part lowers its shader
 * clock.  a_from_lds: the A operand is re-read from LDS once per two MFMAs, as the first-phase kernel does (1), or
 * both operands stay in registers (0).  Outputs (HOST): achieved TFLOP/s and the average shader clock in MHz.
 * Workspace: 1 MiB is enough.  Synchronises the stream.
 */
lcrwmd_status lcrwmd_probe_mfma(lcrwmd_ctx* ctx, lcrwmd_dtype dtype, int random_data, int a_from_lds, double seconds,
                                void* ws, size_t ws_bytes, double* tflops, double* shader_mhz, void* hip_stream);

/*
 * Diagnostic for benchmarks (not part of the method): the rate at which wavefronts gather row segments the way the
 * second phase does (Sec. IV, Fig. 7: every stored entry reads a row of Z) - 64 * floats_per_lane consecutive floats
 * of a pseudo-random row per load, eight loads in flight per wavefront, eight workgroups per CU - from a table of
 * `segments` rows (a power of two, at most 2^24) with a pitch of 16 KiB.  floats_per_lane 4 is the second phase's own
 * 16-byte load (1 KiB per wavefront and load), 2 and 1 the narrower ones.  The number of distinct segments decides
 * which cache level serves them.  Output (HOST): terabytes per second loaded by the lanes.
 * Workspace: segments * 16 KiB + 256 bytes (cleared by the call).  Synchronises the stream.
 */
lcrwmd_status lcrwmd_probe_gather(lcrwmd_ctx* ctx, int64_t segments, int floats_per_lane, void* ws, size_t ws_bytes,
                                  double* tbytes_per_s, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Exact WMD behind the RWMD bound (Sec. II, Sec. III).  These calls take fp32 or bf16 E of any m and
 * pitch.  Cost matrices are fp32: |a|^2 + |b|^2 - 2 a.b on the matrix cores where the two words lie
 * apart (d^2 >= (|a|^2 + |b|^2) / 4), sums of squared coordinate differences where they lie close,
 * exactly 0 for equal word ids.  The transport problems are solved in fp64, results returned as fp32.
 * ------------------------------------------------------------------------------------------- */

/*
 * Word Centroid Distance (Sec. III, "Word Centroid Distance"): with the centroids C1 = X1 E and
 * C2 = X2 E (weights as stored),  D[i * ldd + j] = || C1[i] - C2[j] ||_2.   D is n x q fp32.
 * Workspace: (n + q) * round_up(m, 4) * 4 bytes + 512.  No host synchronisation.
 */
lcrwmd_status lcrwmd_wcd(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                         const lcrwmd_emb* E, float* D, int64_t ldd, void* ws, size_t ws_bytes,
                         void* hip_stream);

/*
 * Workspace of lcrwmd_wmd_pairs for `pairs_in_flight` transport problems at a time, and the part of
 * lcrwmd_wmd_topk's workspace that holds them: per problem max_h_db * max_h_q * 12 bytes (fp32 costs,
 * fp64 flows), where max_h_* are the largest stored-entry counts of a database / query histogram.
 * pairs_in_flight <= 0 asks for as many as the device keeps resident at once (one wavefront each);
 * more than that is never used.
 */
lcrwmd_status lcrwmd_wmd_pairs_workspace_bytes(lcrwmd_ctx* ctx, int64_t max_h_db, int64_t max_h_q,
                                               int64_t pairs_in_flight, size_t* out_bytes);

/*
 * WMD of listed pairs (Sec. II: EMD(x1, x2) = min sum y[p,q] c[p,q] over y >= 0 with row sums x1
 * and column sums x2; Sec. III, "Solving the WMD problem": x1 = F1,i, x2 = F2,j, c = T1,i o T2,j):
 *
 *     out[t] = EMD( X1[pair_db[t]], X2[pair_q[t]],  C[p,u] = || E[word p] - E[word u] ||_2 ),  t < npairs
 *
 * pair_db / pair_q / out (and flags, when not NULL) are device arrays of npairs entries; pair_db[t]
 * in [0, n), pair_q[t] in [0, q) (checked on the device when the validate option is set).  Both
 * histograms' weights are divided by their fp64 sums before the solve (stored fp32 weights add up
 * to 1 only up to rounding, and the two masses must agree).  One wavefront solves one problem by
 * successive shortest paths; flags[t] = 1 where it ran out of its augmentation budget
 * (8 (h1 + h2) + 64 paths), in which case out[t] is the cost of a partial flow - none has been
 * seen to; the call then also returns LCRWMD_ENOCONVERGE when flags is NULL.
 * As many wavefronts as the workspace has room for (at least one) take the problems off a queue.
 * Synchronises the stream when it has to fetch row pointers, when validating, and (flags NULL) at
 * the end to read the failure count.  Histograms of more than 2,048 words
 * are LCRWMD_EUNSUPPORTED (per-word solver state is kept in LDS and registers).
 */
lcrwmd_status lcrwmd_wmd_pairs(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                               const lcrwmd_emb* E, const int32_t* pair_db, const int32_t* pair_q,
                               int64_t npairs, float* out, int32_t* flags, void* ws, size_t ws_bytes,
                               void* hip_stream);

/*
 * Workspace that lets lcrwmd_wmd_topk run with its preferred batch sizes: the RWMD top-k workspace
 * (lcrwmd_workspace_bytes with k) plus candidate lists and transport problems in flight.
 */
lcrwmd_status lcrwmd_wmd_topk_workspace_bytes(lcrwmd_ctx* ctx, int64_t v, int64_t m, int64_t n,
                                              int64_t nnz_db, int64_t q, int64_t nnz_q,
                                              lcrwmd_dtype emb_dtype, int k, int64_t max_h_db,
                                              int64_t max_h_q, size_t* out_bytes);

/*
 * The k nearest database histograms of every query by exact WMD, found with the RWMD cut-off
 * (Sec. III, "Speeding-up WMD using RWMD"): per query, RWMD to every database histogram
 * (lcrwmd_rwmd), the k nearest by RWMD, WMD to those, the largest of these k values as cut-off L,
 * WMD to every other histogram whose RWMD is below L, and the k smallest of all WMDs evaluated.
 * RWMD <= WMD, so nothing that belongs to the result is cut.  While k transport problems per query
 * of the batch do not fill the device, the first round takes the k1 > k (at most 64) nearest by
 * RWMD instead and L is the k-th smallest of their k1 WMDs: the same wall time, a lower cut-off,
 * fewer survivors (any k evaluated distances bound the k-th best from above).  A survivor's solve
 * stops as soon as a lower bound on its distance (the value of the solver's dual variables, which
 * starts at the one-sided RWMD and ends at the WMD) exceeds L: it cannot be among the k nearest.
 * Where k per query does fill the device, the next nearest by RWMD up to 64 per query are evaluated
 * against that L in the same way before the survivors are listed, and L becomes the k-th smallest of
 * all 64.  The device compares fp32 RWMD values against fp32 WMD values, so the test is
 * RWMD < L (1 + 1e-5): rounding can only add candidates.
 * R_idx / R_dist: q x k, ordered by (distance, row index) ascending, as in lcrwmd_rwmd_topk.
 * evaluated (HOST, q entries, or NULL): WMD evaluations started for each query (first round +
 * survivors, including those that stopped early).
 * fp32 E with the LCRWMD_BF16 compute option is refused (LCRWMD_EUNSUPPORTED): a bound rounded to
 * bf16 may exceed the WMD it is meant to bound.  1 <= k <= min(n, 64).
 * Synchronises the stream several times per query batch (RWMD vocabulary sizes, survivor counts).
 * Returns LCRWMD_ENOCONVERGE if any transport problem ran out of budget (results are still written).
 */
lcrwmd_status lcrwmd_wmd_topk(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                              const lcrwmd_emb* E, int k, int32_t* R_idx, float* R_dist,
                              int64_t* evaluated, void* ws, size_t ws_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LCRWMD_H */
