/*
 * libgnnagg - message-passing Aggregation by feature slices on one AMD MI355X
 * (CDNA4 / gfx950).
 *
 * The library computes the Aggregation phase of GNN inference as the paper
 * states it in Algorithm 1 (Section II-B): the feature vector of every vertex
 * is split into chunks along its last dimension, each chunk is aggregated over
 * the in-neighbours of every vertex, and the chunk results sit side by side in
 * the output.  Aggregation is element-wise over features (Section I), so the
 * chunked result equals the unchunked one.
 *
 * Conventions common to all calls
 *  - Messages flow src -> dst.  The CSR is indexed by DESTINATION: row i lists,
 *    in colidx[rowptr[i] .. rowptr[i+1]), the SOURCE vertices of the edges that
 *    end in i (Section II-C: the input is the COO edge set and the vertex
 *    feature matrix).
 *  - Unless a parameter says "host", every pointer is a DEVICE pointer owned by
 *    the caller.  The library allocates no device memory; scratch is passed in
 *    as `workspace`.  Inputs and outputs must not overlap.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    gnnagg_aggregate, gnnagg_aggregate_ws, gnnagg_aggregate_update,
 *    gnnagg_aggregate_noalloc, gnnagg_aggregate_blocked, gnnagg_gat_attention,
 *    gnnagg_combine, gnnagg_combine_scaled, gnnagg_rank_sources, gnnagg_gcn_factors and gnnagg_scale_rows only enqueue kernels on
 *    it and return (no allocation
 *    on the host or the device, no synchronisation, no memset: they can be
 *    captured in a HIP graph); gnnagg_build_csr, gnnagg_check_csr,
 *    gnnagg_plan_rows, gnnagg_plan_source_blocks, gnnagg_tune_f_chunk and
 *    gnnagg_tune_blocked also wait for it, because they hand results back to the host.
 *  - Every call returns a gnnagg_status.  Invalid arguments are detected on the
 *    host before anything is launched and leave all outputs untouched.  Index
 *    values outside [0, N) inside colidx are a contract violation that the
 *    aggregation calls do not check; gnnagg_build_csr does check src/dst.
 *  - Workspace protocol: call once with workspace == NULL to receive the
 *    required size in *workspace_bytes (nothing is launched); then call with a
 *    buffer of at least that size, 256-byte aligned, and *workspace_bytes set
 *    to its size.
 */
#ifndef GNNAGG_H
#define GNNAGG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GNNAGG_API __attribute__((visibility("default")))

typedef enum {
  GNNAGG_OK = 0,
  GNNAGG_EINVAL = -1,       /* an argument is out of range or inconsistent */
  GNNAGG_ENULL = -2,        /* a required pointer is NULL */
  GNNAGG_EUNSUPPORTED = -3, /* valid request the library does not implement */
  GNNAGG_EWORKSPACE = -4,   /* workspace missing, too small or misaligned */
  GNNAGG_EDEVICE = -5       /* a HIP call failed */
} gnnagg_status;

typedef enum {
  GNNAGG_SUM = 0,  /* out[i,f] = sum_j X[j,f] */
  GNNAGG_WSUM = 1, /* out[i,f] = sum_j edge_w[e] * X[j,f]   (GCN with the weights of NORM_SYM) */
  GNNAGG_MEAN = 2, /* out[i,f] = (sum_j X[j,f]) / deg(i), 0 for an empty row (GraphSAGE mean) */
  GNNAGG_MAX = 3,  /* out[i,f] = max_j X[j,f], +0.0 for an empty row; -0 orders below +0 */
  /* out[i,f] = row_scale[i] * sum_j X[j,f]: a weighted sum whose weights factor into a per-destination
   * and a per-source part, w_ij = a_i b_j, with the sources' part already in X (gnnagg_scale_rows).  GCN's
   * weights do (a = b = d^-1/2, gnnagg_gcn_factors), and the stream of per-edge weights then goes unread.
   * row_scale ([N] fp32) is passed in the edge_w argument. */
  GNNAGG_SUM_SCALED = 4
} gnnagg_op;

typedef enum { GNNAGG_F32 = 0, GNNAGG_BF16 = 1 } gnnagg_dtype;

enum {
  GNNAGG_SELF_LOOPS = 1, /* append the edges i -> i, i = 0..N-1, after the E input edges */
  GNNAGG_NORM_SYM = 2    /* edge_w = 1/sqrt(d_i d_j), d = row length after self-loops */
};

/* f_chunk value that lets the library pick the chunk width (see gnnagg_aggregate). */
#define GNNAGG_F_CHUNK_AUTO (-1)

/* Number of degree classes in a row plan (class 0: empty rows; class c >= 1:
 * rows with 2^(c-1) <= degree < 2^c). */
#define GNNAGG_PLAN_CLASSES 33

GNNAGG_API int gnnagg_version(void);
GNNAGG_API const char* gnnagg_strerror(int status);

/*
 * COO -> destination-indexed CSR (Section II-C: forward takes the COO edge
 * set; Section III discusses the cost of converting it to CSR).
 *
 *   src, dst   [E] int32, edge k is src[k] -> dst[k]; values must lie in [0,N)
 *   flags      GNNAGG_SELF_LOOPS | GNNAGG_NORM_SYM
 *   rowptr     [N+1] int64 out
 *   colidx     [nnz] int32 out, nnz = E (+ N with SELF_LOOPS).  Inside a row the
 *              entries are ordered by (source ascending, input position
 *              ascending); duplicate edges are kept.
 *   edge_w     [nnz] fp32 out, may be NULL.  With NORM_SYM: the fp64 value
 *              1/sqrt(d_i*d_j) rounded once to fp32; otherwise 1.0f.
 *   perm       [nnz] int64 out, may be NULL: input position of the edge held in
 *              each CSR slot (self-loop i has position E+i).
 *
 * The result is unique, so it can be compared bit for bit.  Returns
 * GNNAGG_EINVAL (outputs undefined) if a src/dst value is out of range,
 * GNNAGG_EUNSUPPORTED if nnz >= 2^32 or N >= 2^31.  Waits for `stream`.
 */
GNNAGG_API int gnnagg_build_csr(int64_t N, int64_t E, const int32_t* src, const int32_t* dst, uint32_t flags,
                     int64_t* rowptr, int32_t* colidx, float* edge_w, int64_t* perm, void* workspace,
                     size_t* workspace_bytes, void* stream);

/*
 * Checks a CSR that did not come from gnnagg_build_csr before it is handed to the aggregation calls,
 * which trust it: rowptr[0] == 0, rowptr non-decreasing, rowptr[N] == nnz, every colidx value in [0, N).
 * Returns GNNAGG_EINVAL if any of that fails.  Waits for `stream`; the usual workspace protocol.
 */
GNNAGG_API int gnnagg_check_csr(int64_t N, int64_t nnz, const int64_t* rowptr, const int32_t* colidx, void* workspace,
                     size_t* workspace_bytes, void* stream);

/*
 * Degree-sorted row schedule for the aggregation kernels (per graph, reusable
 * by every later aggregation call on the same CSR).  Power-law degree
 * distributions (Section III, Table II: average degree 4.5 to 597) need rows of
 * similar length to share a wavefront and hub rows to get a whole workgroup.
 *
 *   row_order  [N] int32 out: row ids by degree descending, ties by row id
 *   class_off  HOST pointer, [GNNAGG_PLAN_CLASSES+1] int64 out: rows of degree
 *              class c occupy row_order[class_off[32-c] .. class_off[33-c])
 *
 * Waits for `stream`.
 */
GNNAGG_API int gnnagg_plan_rows(int64_t N, const int64_t* rowptr, int32_t* row_order, int64_t* class_off,
                     void* workspace, size_t* workspace_bytes, void* stream);

/*
 * Aggregation, one feature chunk after another (Algorithm 1, the Message /
 * Aggregate / Concat steps).
 *
 *   X        [N,F] row-major, x_dtype GNNAGG_F32 or GNNAGG_BF16 (bf16 is widened
 *            exactly; sums accumulate in fp64)
 *   out      [N,F] row-major, out_dtype GNNAGG_F32, or GNNAGG_BF16 (the fp32 result rounded to
 *            nearest even: halves the write stream)
 *   edge_w   [nnz] fp32, required for GNNAGG_WSUM; for GNNAGG_SUM_SCALED the [N] fp32 factors of the
 *            destinations, required; ignored otherwise
 *   f_chunk  chunk WIDTH (the width of one decomposition layer,
 *            Section III): chunk c covers columns [c*f_chunk, min(F,(c+1)*f_chunk)).
 *            Chunks run one after another over all rows (the chunk-outer,
 *            vertex-inner order of Algorithm 1), each written in place into its
 *            columns of `out` (no separate concat).  0 or >= F: one chunk.
 *            GNNAGG_F_CHUNK_AUTO: the library picks (Section II-B ties the number of layers to the
 *            memory capacity of the device and the character of the dataset): row pieces of 1, 2, 4
 *            or 8 cache lines when the rows of X start on 128-byte lines (see gnnagg_aggregate_ws)
 *            and the plan shows a graph whose longest rows hold a large share of the edges - the
 *            fewer rows and the shorter they are, the wider the piece; a power-of-two width whose
 *            column slice of X is a few hundred MB once X is beyond 1 GiB (never narrower than 128
 *            bytes per row); otherwise one chunk.  gnnagg_auto_f_chunk returns that choice;
 *            gnnagg_tune_f_chunk finds the width by measurement instead.
 *   row_order, class_off   a plan from gnnagg_plan_rows for this rowptr, or both
 *            NULL (rows then run in natural order, one wavefront per row slice:
 *            correct for any graph, slow on hub rows).  class_off is a HOST
 *            pointer and is read before the call returns.
 *
 * Sums accumulate in fp64 and are rounded to fp32 once, so every element is
 * the correctly rounded sum up to fp64 reordering effects, whatever the degree;
 * max is exact.  No atomics are
 * used: results are bit-reproducible from run to run.
 */
GNNAGG_API int gnnagg_aggregate(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                     const void* X, int x_dtype, void* out, int out_dtype, int32_t F, int32_t f_chunk,
                     const int32_t* row_order, const int64_t* class_off, void* stream);

/*
 * gnnagg_aggregate with row pitches and a workspace (same operation, same result up to the order
 * of the fp64 additions; max is bit-identical).
 *
 *   x_pitch, out_pitch   elements between the starts of consecutive rows of X / out (>= F; 0 = F; a row
 *            pitch of X of 2^32 bytes or more is GNNAGG_EUNSUPPORTED).
 *            A gather moves whole 128-byte lines: a 200-byte row (100 bf16 columns) at a 200-byte
 *            pitch straddles 2.55 lines on average, at a 256-byte pitch exactly 2.  gnnagg_row_pitch
 *            returns the pitch that puts every row on line boundaries.  Columns [F, pitch) are never
 *            read or written.
 *
 *   workspace, workspace_bytes   Power-law graphs (Section III, Table II) can hold rows with millions
 *            of in-edges.  gnnagg_aggregate gives such a row to one workgroup, whose serial walk then
 *            sets the run time of the whole call.  With a plan and a workspace, every row of 2^15 edges
 *            or more is cut into pieces of 2^13 consecutive edges; one workgroup per piece leaves an
 *            fp64 partial result in the workspace and a second kernel folds the pieces of a row in
 *            order (no atomics: results stay bit-reproducible).  The usual protocol: workspace == NULL
 *            returns the size in *workspace_bytes and launches nothing.  The size depends on
 *            (N, F, class_off) only and is 0 when the plan holds no such row or there is no plan; then
 *            pass any non-NULL 256-byte-aligned pointer.  The workspace may be reused by the next call
 *            on the same stream; calls on different streams need workspaces of their own.
 */
GNNAGG_API int gnnagg_aggregate_ws(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                        const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                        int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk, const int32_t* row_order,
                        const int64_t* class_off, void* workspace, size_t* workspace_bytes, void* stream);

/*
 * Aggregation followed by the Update step of Algorithm 1 in the same kernels (Section I: Combination is
 * the per-vertex dense update; Section III orders it before or after Aggregation):
 *
 *   W2 == NULL:  out[N,F]  = act( aggregate(X) + bias[F] )          any F, any f_chunk
 *   W2 != NULL:  out[N,H2] = act( aggregate(X) W2[F,H2] + bias[H2] )  F <= GNNAGG_FUSED_MAX_ROW
 *
 * so that a layer act(A (X W) + b) is gnnagg_combine followed by this call with no further pass over the
 * result, and a layer act((A X) W2 + b) at a hidden width is this call alone: the aggregated row is
 * multiplied while it is still in the workgroup's LDS.  aggregate(X) is the value gnnagg_aggregate_ws
 * returns (rounded to fp32 once).  With W2 the F products and the bias are summed in fp64 and rounded
 * once, as in gnnagg_combine; without W2 the bias is added in fp32.  act is max(0, .) for relu == 1 and
 * the identity for relu == 0.
 *
 *   W2     [F,H2] row-major fp32, or NULL (then H2 must be 0); H2 <= GNNAGG_FUSED_MAX_COLS
 *   bias   fp32, as long as a row of out, or NULL
 *   out    [N,F] or [N,H2], out_dtype GNNAGG_F32 or GNNAGG_BF16 (rounded to nearest even after act)
 *   f_chunk  as in gnnagg_aggregate; with W2 the row is contracted whole, so 0, >= F or
 *          GNNAGG_F_CHUNK_AUTO only (anything else is GNNAGG_EINVAL)
 *
 * Everything else (pitches, plan, workspace protocol, splitting of very long rows) as in
 * gnnagg_aggregate_ws.  GNNAGG_EUNSUPPORTED for W2 with F > GNNAGG_FUSED_MAX_ROW.
 */
#define GNNAGG_FUSED_MAX_ROW 64
#define GNNAGG_FUSED_MAX_COLS 4096
GNNAGG_API int gnnagg_aggregate_update(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                            const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, int32_t F,
                            int32_t f_chunk, const float* W2, int32_t H2, const float* bias, int relu, void* out,
                            int out_dtype, int64_t out_pitch, const int32_t* row_order, const int64_t* class_off,
                            void* workspace, size_t* workspace_bytes, void* stream);

/*
 * gnnagg_aggregate_ws for callers that cannot allocate device memory and have no workspace to hand over
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * without the workspace pair, same kernels, same result bit for bit.  The partial results of split rows
 * (rows of 2^15 edges or more in the plan) go to a fixed array of GNNAGG_NOALLOC_SCRATCH_BYTES that is
 * part of the library's code object: every GPU the library runs on holds one copy until the process
 * ends.  The call allocates nothing, on the host or on the device.
 *
 *   - GNNAGG_EWORKSPACE if the plan needs more than GNNAGG_NOALLOC_SCRATCH_BYTES (the size
 *     gnnagg_aggregate_ws reports for the same (N, F, class_off)): use gnnagg_aggregate_ws then.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (different
 *     streams, or graphs replayed concurrently) race on it.  Calls on one stream are ordered and safe.
 *     Nothing in the array has to start at zero: every slot is written in full before it is read.
 *   - The device of `stream` must be current.  The first call on a device that splits a row looks the
 *     array's address up (hipGetSymbolAddress); make that call outside stream capture.
 */
#define GNNAGG_NOALLOC_SCRATCH_BYTES (8u << 20)
GNNAGG_API int gnnagg_aggregate_noalloc(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                             const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                             int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk,
                             const int32_t* row_order, const int64_t* class_off, void* stream);

/* Row pitch (in elements) that starts every row of an [N,F] matrix of the given type on a 128-byte line
 * boundary, or on a power-of-two fraction of a line for rows shorter than one (host arithmetic only;
 * 0 for invalid arguments). */
GNNAGG_API int64_t gnnagg_row_pitch(int32_t F, int dtype);

/* The chunk width the aggregation calls use for GNNAGG_F_CHUNK_AUTO (host-side arithmetic only) for an
 * X of row pitch x_pitch (0 = F) whose first row starts on a 128-byte line, and the plan's class_off
 * (HOST pointer, or NULL for no plan).  0 for invalid arguments. */
GNNAGG_API int32_t gnnagg_auto_f_chunk(int64_t N, int32_t F, int x_dtype, int64_t x_pitch, const int64_t* class_off);

/*
 * The chunk width by measurement instead of by rule (Section II-B: the number of layers is to be
 * determined per device and dataset; the paper does so by hand).  Runs gnnagg_aggregate_ws on the caller's
 * own arrays at a handful of widths - one chunk, the width GNNAGG_F_CHUNK_AUTO would take, and row pieces
 * of 1, 2, 4 and 8 cache lines - a warm-up and three timed calls each, and returns the fastest in
 * *best_f_chunk (its time per call in *best_ms, which may be NULL).  A per-graph step like the plan: pass
 * the result as f_chunk from then on.  `out` holds a valid aggregation afterwards.  Same arguments and
 * workspace protocol as gnnagg_aggregate_ws; waits for `stream`.
 */
GNNAGG_API int gnnagg_tune_f_chunk(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                        const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out, int out_dtype,
                        int64_t out_pitch, int32_t F, const int32_t* row_order, const int64_t* class_off,
                        void* workspace, size_t* workspace_bytes, void* stream, int32_t* best_f_chunk,
                        float* best_ms);

/*
 * Source blocks: the trade of Section II-B (better reuse of the feature rows against more passes over
 * the graph) taken along the vertex dimension as well.  The vertices are cut into B blocks of
 * ceil(N/B) consecutive ids; a blocked aggregation gathers from one block's rows of X at a time, over all
 * destinations and all feature chunks, so that the rows it re-reads are B times fewer and stay in the
 * caches, and carries every destination's unfinished state from block to block.
 *
 * gnnagg_plan_source_blocks is the per-graph step (like gnnagg_plan_rows, which it replaces for the
 * blocked call).  Every row of the CSR must list its sources in ascending order, as gnnagg_build_csr
 * writes them, so that a block's edges are one run of the row: GNNAGG_EINVAL otherwise (checked).
 *
 *   B          number of blocks, 1 .. GNNAGG_MAX_SOURCE_BLOCKS
 *   block_ptr  [(B+1) * N] int64 out: the edges of row r with sources in block b are
 *              colidx[block_ptr[b*N + r] .. block_ptr[(b+1)*N + r])
 *   row_order  [B * N] int32 out: per block, the rows by the number of their edges in it, descending
 *   class_off  HOST pointer, [B * (GNNAGG_PLAN_CLASSES+1)] int64 out: per block, as in gnnagg_plan_rows
 *
 * Waits for `stream`.
 */
#define GNNAGG_MAX_SOURCE_BLOCKS 64
GNNAGG_API int gnnagg_plan_source_blocks(int64_t N, const int64_t* rowptr, const int32_t* colidx, int32_t B,
                              int64_t* block_ptr, int32_t* row_order, int64_t* class_off, void* workspace,
                              size_t* workspace_bytes, void* stream);

/*
 * gnnagg_aggregate_ws over source blocks: same operators, same layout arguments, the result of the same
 * arithmetic contract (fp64 accumulation, one rounding; max exact).  Block b runs as one pass of the
 * aggregation kernels over the edges block_ptr selects, with that block's row order; between blocks a
 * destination's state waits in the workspace as doubles (max: its integer key), so the sum of a row is
 * still taken in the row's edge order up to the grouping by lanes, and the row is rounded once, after the
 * last block.  Mean divides by the row's whole degree.
 *
 *   B, block_ptr, row_order, class_off   from gnnagg_plan_source_blocks for this CSR (class_off HOST)
 *   f_chunk    as in gnnagg_aggregate; GNNAGG_F_CHUNK_AUTO here means row pieces of two 128-byte lines
 *              when the rows of X start on lines and are at least two pieces long, else one chunk
 *   workspace  min(B-1, 2) arrays of N rows of F doubles (rows padded to 128-byte lines) for the states
 *              in transit, used in turn, plus what the split rows of the longest block need; size query
 *              as usual
 *
 * Only enqueues kernels.  GNNAGG_EINVAL for B outside 1 .. GNNAGG_MAX_SOURCE_BLOCKS.
 */
GNNAGG_API int gnnagg_aggregate_blocked(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                             const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                             int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk, int32_t B,
                             const int64_t* block_ptr, const int32_t* row_order, const int64_t* class_off,
                             void* workspace, size_t* workspace_bytes, void* stream);

/*
 * gnnagg_tune_f_chunk for the blocked call: times gnnagg_aggregate_blocked on the caller's own arrays, with
 * the tables of B blocks, at its own chunk width and at row pieces of 1, 2 and 4 cache lines (a warm-up and
 * three timed calls each) and returns the fastest width in *best_f_chunk and its time per call in *best_ms
 * (may be NULL).  Comparing *best_ms over a few block counts, and with gnnagg_tune_f_chunk's for the plain
 * call, settles by measurement what gnnagg_auto_source_blocks settles by rule.  Same arguments and workspace
 * protocol as gnnagg_aggregate_blocked; `out` holds a valid aggregation afterwards; waits for `stream`.
 */
GNNAGG_API int gnnagg_tune_blocked(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                        const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out, int out_dtype,
                        int64_t out_pitch, int32_t F, int32_t B, const int64_t* block_ptr,
                        const int32_t* row_order, const int64_t* class_off, void* workspace,
                        size_t* workspace_bytes, void* stream, int32_t* best_f_chunk, float* best_ms);

/* Number of source blocks worth using for operator `op` on a graph with the row plan class_off (HOST
 * pointer, the plan of gnnagg_plan_rows; NULL: 1) and an X of row pitch x_pitch (0 = F) whose first row
 * starts on a 128-byte line; 1 means the plain calls are the faster ones (host arithmetic only; 0 for
 * invalid arguments).  Blocks pay on dense graphs only: the states in transit cost 16 bytes per output
 * element and block. */
GNNAGG_API int32_t gnnagg_auto_source_blocks(int op, int64_t N, int32_t F, int x_dtype, int64_t x_pitch,
                                  const int64_t* class_off);

/*
 * Graph-attention aggregation (the GAT operator the paper evaluates in
 * Section III, with chunk width 8 = one head at 8 channels per head).
 *
 *   H          [N, heads, C] fp32
 *   a_src,a_dst [heads, C] fp32
 *   score      s_src[j,h] = sum_c a_src[h,c] H[j,h,c], s_dst likewise, computed
 *              once from whole head vectors (so every chunk sees the same
 *              weights); e_ij,h = LeakyReLU(s_src[j,h] + s_dst[i,h])
 *   alpha      [nnz, heads] fp32 out, may be NULL: softmax of e over the in-edges
 *              of each destination, per head
 *   out        [N, heads, C] fp32 out, may be NULL: sum_j alpha_ij,h H[j,h,:];
 *              empty rows give 0
 *   f_chunk    0, or a multiple of C (chunks are whole heads); anything else is
 *              GNNAGG_EINVAL
 *   workspace  holds the two score arrays (2*N*heads fp32) and, when the plan holds rows of 2^15 edges
 *              or more, the partial softmax states of their pieces (such rows are split over
 *              workgroups as in gnnagg_aggregate_ws and finished by two small kernels).  Its size
 *              therefore depends on class_off: query it with the plan the call will use.
 *              With alpha == NULL and 4, 8 or 16 channels per head both scores of an edge are recomputed
 *              in registers from the feature rows: the call is then a single kernel launch and leaves
 *              the score arrays untouched.
 *
 * Precision.  Scores are summed in fp64 and rounded to fp32, the logit s_src + s_dst and the LeakyReLU are
 * fp32 operations, and exp(logit - reference) uses the hardware exponential (relative error about
 * 1e-7 * |argument| + 2e-7), while denominators and weighted sums are carried in fp64.  The result is
 * within 1e-6 + 1e-5 |r| of the fp64 definition as long as the logits of a row stay within about +-16
 * (scores of a few units, as attention vectors of standard deviation 0.1 give); the error grows in
 * proportion to the largest |logit| (ulp of the fp32 logit), about 1e-5 relative at |logit| = 100.
 */
GNNAGG_API int gnnagg_gat_attention(int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* H,
                         const float* a_src, const float* a_dst, int32_t heads, int32_t C,
                         float negative_slope, float* alpha, float* out, int32_t f_chunk,
                         const int32_t* row_order, const int64_t* class_off, void* workspace,
                         size_t* workspace_bytes, void* stream);

/*
 * Combination (Section I: the per-vertex MLP update; Algorithm 1, Update) as one dense layer, so
 * that it can run ahead of Aggregation and Aggregation works at the hidden width (Section III):
 *
 *     out[N,H] = act( X[N,F] * W[F,H] + bias[H] )
 *
 *   X      [N,F] row-major, GNNAGG_F32 or GNNAGG_BF16
 *   W      [F,H] row-major fp32; bias [H] fp32 or NULL
 *   relu   1: act = max(0, .), 0: identity
 *   out    [N,H] row-major fp32; must not overlap X
 *   out_rows  [N] int32 or NULL: row i of the result is stored as row out_rows[i] of out (a
 *          permutation of 0..N-1, e.g. the rank array of gnnagg_rank_sources, so that the
 *          aggregation that follows gathers from rows stored in popularity order)
 *
 * Products and sums are carried in fp64 on the matrix cores and rounded to fp32 once.
 * Asynchronous on `stream`.
 */
GNNAGG_API int gnnagg_combine(int64_t N, const void* X, int x_dtype, int32_t F, const float* W, const float* bias,
                              int32_t H, int relu, float* out, const int32_t* out_rows, void* stream);

/*
 * gnnagg_combine with the rows of the result scaled on their way out:
 *
 *     out[i, :] = row_scale[i] * act( X[i, :] W + bias )
 *
 * the product formed in fp32 on the rounded result, so that the call equals gnnagg_combine followed by
 * gnnagg_scale_rows bit for bit.  With row_scale = the factors of gnnagg_gcn_factors this is the input of a
 * GCN aggregation in factored form (GNNAGG_SUM_SCALED; Section III: Combination ahead of Aggregation)
 * without a scaling pass of its own.  row_scale [N] fp32, required; everything else as in gnnagg_combine.
 */
GNNAGG_API int gnnagg_combine_scaled(int64_t N, const void* X, int x_dtype, int32_t F, const float* W,
                                     const float* bias, int32_t H, int relu, const float* row_scale, float* out,
                                     const int32_t* out_rows, void* stream);

/*
 * Popularity order of the source vertices, for feature rows narrower than a 128-byte line
 * (Aggregation at the hidden widths of Section III).  A gather fetches whole lines; when the rows that
 * are gathered most often sit next to each other, the hot part of X occupies a fraction of the lines
 * it would otherwise and stays in L2.
 *
 *   rank           [N] int32 out: position of vertex j when the vertices are ordered by how often they
 *                  occur in colidx, most frequent first, ties by vertex id
 *   colidx_ranked  [nnz] int32 out: rank[colidx[e]]
 *
 * Aggregating with (colidx_ranked, Xr), where Xr[rank[j]] = X[j] - e.g. the output of gnnagg_combine
 * with out_rows = rank - gives bit for bit the result of (colidx, X): the order of the edges inside a
 * row does not change.  (Not for gnnagg_gat_attention, which also reads H at the destination.)
 * Asynchronous on `stream`; the usual workspace protocol.
 */
GNNAGG_API int gnnagg_rank_sources(int64_t N, int64_t nnz, const int32_t* colidx, int32_t* rank,
                        int32_t* colidx_ranked, void* workspace, size_t* workspace_bytes, void* stream);

/*
 * GCN's aggregation weights in factored form (the GCN operator of Section III: the adjacency matrix with
 * self-loops, normalised by the degrees on both sides): 1/sqrt(d_i d_j) = s_i s_j with
 *
 *     s[i] = (float)(1 / sqrt(d_i)),  d_i = rowptr[i+1] - rowptr[i];  0 for an empty row
 *
 *   s   [N] fp32 out.  Asynchronous on `stream`.
 *
 * out = GNNAGG_SUM_SCALED(rowptr, colidx, s, gnnagg_scale_rows(X, s)) is then the GCN aggregation of X
 * without the [nnz] stream of edge weights; it differs from GNNAGG_WSUM with the weights of
 * GNNAGG_NORM_SYM by how the weights are rounded (here s_j X[j,f] is rounded to fp32 once per source row,
 * there 1/sqrt(d_i d_j) once per edge): a few units of 2^-24 relative to the sum of the terms' magnitudes.
 */
GNNAGG_API int gnnagg_gcn_factors(int64_t N, const int64_t* rowptr, float* s, void* stream);

/*
 * out[j,f] = scale[j] * X[j,f]: the per-source part of factored aggregation weights, applied to the
 * feature rows once instead of to every edge (see GNNAGG_SUM_SCALED).  One fp32 product per element,
 * correctly rounded (a bf16 input is widened first).
 *
 *   X      [N,F] GNNAGG_F32 or GNNAGG_BF16, row pitch x_pitch elements (>= F; 0 = F)
 *   scale  [N] fp32
 *   out    [N,F] fp32, row pitch out_pitch; may be X itself when X is fp32 and the pitches agree, must not
 *          overlap it otherwise.  Columns [F, pitch) are neither read nor written.
 *
 * Asynchronous on `stream`.
 */
GNNAGG_API int gnnagg_scale_rows(int64_t N, int32_t F, const void* X, int x_dtype, int64_t x_pitch,
                                 const float* scale, float* out, int64_t out_pitch, void* stream);

/*
 * Measurement aid, not part of the method: overrides, for every later aggregation call of the process, how
 * many workgroups of the aggregation kernel may share a compute unit (the library normally derives that
 * from the plan's degree classes and the bytes a workgroup keeps in flight).  cap = -1 restores the
 * library's rule, 0 lifts the cap, 2..16 forces that many.  Results do not depend on it.  Used to check
 * the rule against measured optima on graphs it was not derived from.
 */
GNNAGG_API int gnnagg_set_workgroup_cap(int cap);

/*
 * Measurement aid, not part of the method: copies `bytes` bytes (a multiple of
 * 16, both pointers 16-byte aligned, buffers disjoint) from src to dst with a
 * plain streaming kernel on `stream`.  Its HBM traffic is known exactly (bytes
 * read + bytes written), which gives the achievable copy rate of the device and
 * the scale of the profiler's byte counters next to the aggregation kernels.
 */
GNNAGG_API int gnnagg_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Measurement aid, not part of the method: `workgroups` workgroups of four wavefronts each issue
 * 8 * iters v_mfma_f64_16x16x4_f64 instructions (2048 flop each) and nothing else: the fp64 matrix rate
 * the device sustains, next to which gnnagg_combine is set.  sink: 8 bytes of device memory, never
 * written.  Asynchronous on `stream`.
 */
GNNAGG_API int gnnagg_mfma_f64_probe(double* sink, int64_t iters, int32_t workgroups, void* stream);

/*
 * Measurement aid, not part of the method: the access pattern of a one-line gather.  `workgroups`
 * workgroups of 256 lanes; every group of eight lanes reads 8 * rounds 128-byte lines of buf[0 .. bytes)
 * (16 bytes per lane, eight loads in flight per lane).
 *   idx == NULL: the pattern alone - lines chosen by a hash, no index loaded, no sum kept: the rate at which
 *     the memory system serves random lines out of a working set of `bytes` bytes (in L2, in the Infinity
 *     Cache or in HBM, by its size), the ceiling for the aggregation kernels' line requests.
 *   idx != NULL: [workgroups * 32 * 8 * rounds] uint32 line numbers (clamped to the buffer), read the way an
 *     aggregation pass reads colidx (one per lane and round, a round ahead, handed round with swizzles);
 *     the loaded floats pass a bit mask and are summed in fp64: an aggregation pass without its rows, what
 *     the ingredients themselves cost.
 * Lines read per call: workgroups * 32 * 8 * rounds.  buf: 128-byte aligned, bytes a multiple of 128
 * (below 2^38); sink: 4 bytes of device memory, never written.  Asynchronous on `stream`.
 */
GNNAGG_API int gnnagg_line_gather_probe(const void* buf, size_t bytes, const uint32_t* idx, int32_t rounds,
                             int32_t workgroups, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GNNAGG_H */
