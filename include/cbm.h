/*
 * libcbm -- Compressed Binary Matrix (CBM) products on one AMD MI355X (gfx950).
 *
 * C ABI.  A binary m x n matrix A, given as CSR without values (each row a
 * sorted list of column indices: the paper's adjacency-list input, Section 2),
 * is compressed once into a CBM handle; the handle then multiplies any number
 * of dense fp32 matrices (the "compressed once, multiplied many times" use of
 * Section 1.2).  All dense operands are row-major fp32 in DEVICE memory; all
 * index arrays passed to cbm_build are in HOST memory.
 *
 * Every function returns a cbm_status; nothing throws or aborts across this
 * boundary, and output arguments are left untouched on failure.
 */
#ifndef CBM_H
#define CBM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cbm_handle cbm_handle; /* opaque; owns its host and device arrays */

typedef enum {
    CBM_OK = 0,
    CBM_ERR_INVALID_ARG = 1, /* null pointer, k <= 0, ld < k, bad option value      */
    CBM_ERR_INVALID_CSR = 2, /* row offsets not monotone, columns unsorted, repeated
                                or out of [0, n)                                     */
    CBM_ERR_ALLOC = 3,       /* host or device allocation failed                     */
    CBM_ERR_HIP = 4,         /* a HIP runtime call failed                            */
    CBM_ERR_UNSUPPORTED = 5, /* size beyond what the index types can hold            */
    CBM_ERR_STATE = 6        /* handle cannot do this (host-only handle, normalised
                                product on a handle built without self-loops, ...)   */
} cbm_status;

/* cbm_build_opts.flags */
#define CBM_FLAG_HOST_ONLY 1u /* build the format but upload nothing to a GPU:
                                 cbm_stats / cbm_get_tree / cbm_decompress work,
                                 products return CBM_ERR_STATE                      */
#define CBM_FLAG_EXACT_TREE 2u /* the chain of compression is a minimum-cost arborescence
                                  of the pruned candidate digraph rooted at the virtual
                                  vertex (Section 2.2, "Edge Pruning"), found exactly by
                                  Edmonds' algorithm; max_depth and seed_roots are
                                  ignored.  With hub_cap = max_candidates = -1 the
                                  candidate digraph is the whole pruned distance graph. */

#define CBM_FLAG_DEVICE_BUILD 4u /* run the builder's candidate search (which rows share columns
                                    with which, the pattern of A A^T) on the GPU instead of the
                                    host threads; the chain of compression is the same.  Needs
                                    1 <= max_candidates <= 16 (the default qualifies); not with
                                    CBM_FLAG_HOST_ONLY or CBM_FLAG_HOST_SEARCH.  Without this
                                    flag a matrix of 65536 rows or more is searched on the GPU
                                    too when those conditions hold, and on the host threads if
                                    the GPU cannot take it (the search needs up to 24 GB of
                                    device memory while it runs); with it, that is an error.   */
#define CBM_FLAG_HOST_SEARCH 16u /* keep the candidate search on the host threads              */

#define CBM_FLAG_TRANSPOSE 8u /* compress the transpose: the handle holds A^T (n x m; (A v I)^T with
                                 add_self_loops) and every product and query works on that matrix.
                                 The normalised product keeps D = the row sums of A v I as given, so
                                 it computes (D^-1/2 (A + I) D^-1/2)^T X: the backward pass of the
                                 normalised product for a directed graph (for a symmetric one the
                                 transpose is the matrix itself and this flag changes nothing).   */

/*
 * Build options.  A NULL pointer means all zeros, i.e. the defaults below.
 *
 * alpha          Edge-pruning threshold of Section 2.2 ("Edge Pruning"): row x may
 *                be compressed against row y only if that saves at least alpha
 *                scalar operations, w(y,x) <= nnz(a_x) - alpha.  alpha = 0 keeps
 *                every compression that strictly beats storing the row in full
 *                (draws go to the virtual vertex, Section 2.2 after Eq. (5)).
 * add_self_loops Compress A v I instead of A (needs m == n).  Required by
 *                cbm_spmm_normalized, whose matrix is D^-1/2 (A + I) D^-1/2.
 * max_depth      Cap on the depth of the compression tree (a row stored in full
 *                has depth 1).  -1 = unlimited.  0 = automatic: cap 16, and a
 *                cost model of the kernels (launch overhead, latency of the
 *                longest work item, bandwidth) decides whether the tree pays
 *                for its extra dependent launches at all; on small graphs it
 *                does not, and every row is then stored in full (the paper's
 *                own finding for its small citation graphs, Section 3.3); the
 *                same model drops a trailing round of dependent work when
 *                storing its rows in full is cheaper than its launch, and on a
 *                matrix of 65536 rows or more the candidate search first looks
 *                at every 64th row: if their best candidates would save under
 *                2 % of their entries, the search stops there and every row is
 *                stored in full.  The
 *                tree is cut into vertical paths, one work item each;
 *                dependent kernel launches per product = rounds of paths
 *                (cbm_stats), at most the depth.  Any value yields a valid CBM
 *                (exact product).
 * hub_cap        Candidate search: columns with more than hub_cap entries are
 *                not expanded when counting shared columns (their rows are still
 *                compared exactly once they are candidates).  0 = default (512);
 *                -1 = expand everything (exact shared-column search).
 * max_candidates Candidate parents kept per row.  0 = default (8); -1 = keep all
 *                (with hub_cap = -1, max_depth = -1 and alpha = 0 the tree is then
 *                a true minimum spanning tree of the extended distance graph).
 * seed_roots     Rows forced to be stored in full before the tree is grown, spread
 *                evenly over the row range.  With a depth cap, growing from many
 *                seeds at once gives wider levels (more parallel work per dependent
 *                launch) and often fewer deltas.  0 = automatic (the cost model
 *                picks among 0, m/128, m/32, m/8); -1 = none; > 0 = that many.
 * num_threads    Host threads for the build.  0 = all hardware threads.
 * device         HIP device that will own the arrays.  -1 = current device.
 * flags          CBM_FLAG_* bits.
 * column_blocks  0 or 1 = the format of the paper: one tree over whole rows.  B > 1 = column-blocked CBM (the
 *                column-splitting idea that Section 1.1 credits to a related format): the columns are cut
 *                into B equal ranges, the part of every row inside a range is a row of its own, and the
 *                compression tree is grown over all B m part-rows, so two rows that are alike only inside one
 *                range can still share; a product sums the B partial rows of each row in a last launch.  Costs B
 *                partial rows (written, then read) per matrix row and product.  Not with CBM_FLAG_TRANSPOSE.
 */
typedef struct {
    int32_t alpha;
    int32_t add_self_loops;
    int32_t max_depth;
    int32_t hub_cap;
    int32_t max_candidates;
    int32_t seed_roots;
    int32_t num_threads;
    int32_t device;
    uint32_t flags;
    int32_t column_blocks;
} cbm_build_opts;

typedef struct {
    int64_t m, n;
    int64_t nnz;             /* nonzeros of the compressed matrix (A, or A v I)      */
    int64_t num_delta_plus;  /* sum over rows of |Delta+|                            */
    int64_t num_delta_minus; /* sum over rows of |Delta-|                            */
    int64_t num_roots;       /* rows compressed against the virtual null row         */
    int64_t num_internal;    /* rows that some other row is compressed against       */
    int64_t scalar_ops;      /* Section 2.2: nnz(a_x) for a root, 1+|D+|+|D-| else   */
    int64_t num_tasks;       /* GPU work items (rows, plus segments of split rows)   */
    int64_t num_split_rows;  /* rows whose delta list is cut into several segments   */
    int64_t bytes_csr;       /* int64 row offsets + int32 columns, no values         */
    int64_t bytes_cbm;       /* packed device arrays of this handle                  */
    int32_t depth;           /* number of tree levels                                */
    int32_t alpha;
    int32_t add_self_loops;
    int32_t rounds;          /* dependent kernel launches per product (<= depth)      */
    double build_seconds;
    int32_t column_blocks;   /* 1, or B for a column-blocked handle: the tree then spans
                                B m part-rows; num_roots, num_internal, depth and the
                                delta counts are those of the part-rows, and scalar_ops
                                includes the (B - 1) m additions of the block sum        */
    int32_t bundled_rounds;  /* rounds whose paths are gathered in one sweep per path
                                (long work items of more than one row)                 */
} cbm_stats_t;

/*
 * cbm_build -- compress a binary CSR matrix (Section 2).
 *   m, n      matrix shape; 0 <= m, n < 2^29.
 *   rowptr    host, m + 1 entries, rowptr[0] = 0, non-decreasing.
 *   colidx    host, rowptr[m] entries; within a row strictly increasing, in [0, n).
 *   opts      host, or NULL for defaults.
 *   out       receives the handle.
 * The CSR arrays are only read during the call (copied, not retained).
 * Builder = extended distance graph restricted to row pairs that share a column
 * (only those can beat the virtual edge), Prim growth from the virtual vertex
 * with the draw rule and the alpha rule, delta lists by list merge (Eq. (2)).
 */
cbm_status cbm_build(int64_t m, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                     const cbm_build_opts* opts, cbm_handle** out);

/*
 * cbm_spmm -- Y = A . X  (Eq. (5), Algorithm 1).
 *   X   device, n x k row-major fp32, leading dimension ldx >= k (in floats).
 *   Y   device, m x k row-major fp32, leading dimension ldy >= k.  Fully
 *       overwritten (it need not be zeroed).  The byte ranges spanned by X and
 *       Y must be disjoint (CBM_ERR_INVALID_ARG otherwise, also for column
 *       slices interleaved in one buffer).  The tree update runs in place in Y
 *       (Property 3).
 *   hip_stream  a hipStream_t (NULL = default stream).  The call only enqueues
 *       kernels and returns; the caller synchronises.
 * If the handle was built with add_self_loops the product is (A v I) . X.
 * k not a multiple of 4, or pointers / leading dimensions that are not 16-byte
 * multiples, select a variant of the same kernel that moves 32 bits per lane
 * and access instead of 128, not an error; it takes about 1.7x the time per
 * byte on a large graph, so pad the feature dimension to a multiple of 4 where
 * speed matters.
 * Rows with very long delta lists are summed in pieces through a scratch array owned
 * by the handle (cbm_stats.num_split_rows > 0 says the handle has such rows).  Hence:
 *  - one product at a time per handle: two products of one handle that run at the same
 *    time (two host threads, or two streams) would share that scratch and race;
 *  - the scratch is sized for the widest k seen so far.  A product with a wider k than
 *    any before it frees and reallocates it (the free waits for the device), which is
 *    not allowed under HIP-graph capture: call cbm_reserve(h, widest k) once beforehand;
 *    after that, products with k <= that width only launch kernels and can be captured.
 * Per-launch profiling (cbm_profile_enable) records events and must be off during capture.
 */
cbm_status cbm_spmm(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                    void* hip_stream);

/*
 * cbm_spmm_noalloc -- cbm_spmm for callers that cannot allocate device memory: code under HIP-graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the
 * same result as cbm_spmm, but the partial sums of split rows go to a 64 MiB array that is part of the
 * library's device code instead of a scratch the handle allocates; the call makes no hipMalloc / hipFree
 * and no other allocating call.
 *   Limit: (segments the handle's split rows are cut into -- one scratch row each, at most
 *   cbm_stats.num_tasks) x (k rounded up to a multiple of 4) floats must fit 64 MiB = 16,777,216 floats,
 *   else CBM_ERR_UNSUPPORTED (cbm_last_error_detail gives the numbers); a handle without split rows
 *   (cbm_stats.num_split_rows == 0) always fits.
 *   CBM_ERR_STATE while per-launch profiling is on (it creates events).
 * Every GPU the library runs on holds one such array until the process ends, and every call on that GPU
 * shares it, whatever the handle: calls that overlap in time on one GPU (two streams, two host threads)
 * race on it -- run them one after the other.  Nothing in it has to be cleared between calls: a product
 * writes every scratch row it later reads.
 */
cbm_status cbm_spmm_noalloc(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                            void* hip_stream);

/*
 * cbm_reserve -- size the handle's split-row scratch for products of up to max_k columns now, so
 * that no later product with k <= max_k allocates (see cbm_spmm).  The handle's device must be
 * current.  A handle without split rows needs no scratch: the call then does nothing.
 */
cbm_status cbm_reserve(cbm_handle* h, int32_t max_k);

/*
 * cbm_spmm_normalized -- Y = D^-1/2 (A + I) D^-1/2 . X  (Eq. (1); Section 2.2,
 * "Extending SpMM with CBM to normalized adjacency matrices"), D = row sums of
 * A v I.  Same arguments as cbm_spmm.  Needs a square handle built with
 * add_self_loops, else CBM_ERR_STATE.  The column scale d_j^-1/2 is applied to
 * each gathered row of X, the row scale d_x^-1/2 when a row is written.
 */
cbm_status cbm_spmm_normalized(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y,
                               int64_t ldy, void* hip_stream);

/* Same as cbm_spmm_normalized followed by an element-wise max(., 0): the
 * sigma(A_hat . Z) step of Eq. (1) with sigma = ReLU, fused into the row write. */
cbm_status cbm_spmm_normalized_relu(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y,
                                    int64_t ldy, void* hip_stream);

/*
 * Two more aggregators of the GNN layers the paper names as targets (Section 1: GraphSAGE, GIN), as
 * epilogues of the same kernels; M is the compressed matrix (A, or A v I if built with add_self_loops).
 *   cbm_spmm_mean  Y = D^-1 M X, D = row sums of M: the mean of each row's entries (GraphSAGE's mean
 *                  aggregator); a row of M with no entry gives a zero row.
 *   cbm_spmm_gin   Y = M X + (1 + eps) X (GIN's aggregator); needs m == n.
 * Arguments as for cbm_spmm.  For a symmetric M the backward pass of all products here is the
 * same product applied to the output gradient (M^T = M).
 */
cbm_status cbm_spmm_mean(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                         void* hip_stream);
cbm_status cbm_spmm_gin(const cbm_handle* h, float eps, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                        void* hip_stream);

/*
 * cbm_dense_matmul -- C = A . B for dense row-major fp32 device matrices
 * (the X . W products of Eq. (1)); fp32 MFMA, fp32 accumulation.
 *   A  M x K (lda >= K),  B  K x N (ldb >= N),  C  M x N (ldc >= N), no overlap.
 */
cbm_status cbm_dense_matmul(int64_t M, int32_t N, int32_t K, const float* A, int64_t lda, const float* B,
                            int64_t ldb, float* C, int64_t ldc, void* hip_stream);

/*
 * cbm_gcn2_forward -- two-layer GCN inference, Eq. (1):
 *   out = A_hat . relu(A_hat . (X . W0)) . W1
 * evaluated as Z0 = X W0, H = relu(A_hat Z0), Z1 = H W1, out = A_hat Z1.
 *   X n x f_in, W0 f_in x hidden, W1 hidden x f_out, out n x f_out: device,
 *   row-major, densely packed (leading dimension = number of columns).
 *   workspace  device scratch of at least cbm_gcn2_workspace_bytes() bytes,
 *              caller-owned, 16-byte aligned.
 * X, W0, W1, the workspace and out must not overlap one another where one is written
 * (CBM_ERR_INVALID_ARG).  The handle's split-row scratch is sized for max(hidden, f_out)
 * before the first kernel is enqueued (as cbm_reserve does).
 */
cbm_status cbm_gcn2_forward(const cbm_handle* h, const float* X, int32_t f_in, const float* W0, int32_t hidden,
                            const float* W1, int32_t f_out, float* out, void* workspace, size_t workspace_bytes,
                            void* hip_stream);
size_t cbm_gcn2_workspace_bytes(const cbm_handle* h, int32_t f_in, int32_t hidden, int32_t f_out);

/* Counters of the built format (Properties 1 and 2, Lemma 2.2). */
cbm_status cbm_stats(const cbm_handle* h, cbm_stats_t* out);

/*
 * cbm_get_tree -- the chain of compression, host arrays of m entries each (any
 * may be NULL): parent[x] = row that x is compressed against, -1 for the virtual
 * null row; nplus / nminus = |Delta+|, |Delta-| of the edge (parent[x], x);
 * level[x] = depth of x, 1 for rows stored in full.  For a column-blocked handle (column_blocks = B > 1)
 * every array has B m entries: entry b m + i is the part of row i inside column range b, and parents are
 * part-row indices.
 */
cbm_status cbm_get_tree(const cbm_handle* h, int32_t* parent, int32_t* nplus, int32_t* nminus, int32_t* level);

/*
 * cbm_decompress -- rebuild the compressed matrix from the tree and the delta
 * lists alone, a_x = (a_y u Delta+) \ Delta- (Eq. (2)).  Host outputs: rowptr
 * (m + 1) and colidx (stats.nnz entries, sorted within rows).  Returns A v I
 * when the handle was built with add_self_loops.
 */
cbm_status cbm_decompress(const cbm_handle* h, int64_t* rowptr, int32_t* colidx);

/*
 * Per-launch timing of the product kernels.  With profiling on, every kernel a
 * product call enqueues is bracketed by HIP events on the caller's stream.
 * After synchronising the stream, cbm_profile_read returns, for the most
 * recent product call, up to `cap` records and the total count in *count.
 */
typedef struct {
    int32_t kind;           /* 0 = gather/update round, 1 = segments of split rows,
                               2 = split-row combine, 3 = deferred finish of rows that
                               other work items read (row weight, self term, ReLU),
                               4 = sum of the partial rows of a column-blocked handle    */
    int32_t level;          /* round for kinds 0 and 2, else 0                         */
    int64_t tasks;          /* work items in the launch                               */
    int64_t deltas;         /* delta entries gathered by the launch                   */
    int64_t algorithmic_bytes; /* bytes the method itself must move in this launch    */
    float milliseconds;
    int32_t per_xcd;        /* 1 = the launch hands every XCD a work list of its own (segments
                               by column range; a round in graph-locality order), else 0     */
} cbm_launch_record;
cbm_status cbm_profile_enable(cbm_handle* h, int32_t on);
cbm_status cbm_profile_read(cbm_handle* h, cbm_launch_record* records, int32_t cap, int32_t* count);

void cbm_free(cbm_handle* h); /* NULL-safe; releases everything the handle owns */
const char* cbm_status_string(cbm_status s);
/* Text naming the HIP call and runtime error behind the calling thread's most recent
 * CBM_ERR_HIP / CBM_ERR_ALLOC ("" if none).  Valid until that thread's next failing call. */
const char* cbm_last_error_detail(void);

#ifdef __cplusplus
}
#endif
#endif /* CBM_H */
