/*
 * es_spmm.h -- C ABI of the MI355X (gfx950) edge-sampled SpMM library.
 *
 * The library computes the GNN feature aggregation  Y = sample_W(A) * X  of the
 * ES-SpMM / "CacheSample" method (paper: Section 4, Algorithm 1): A is an N x N
 * sparse matrix in plain 3-array CSR (Section 2.2), X and Y are dense row-major
 * fp32 (Section 4.1); every row of A is capped at W stored entries by an
 * in-kernel sampler (Section 4.2, "cache-first edge sampling") whose picks are
 * staged in on-chip memory (LDS) and then multiplied with the gathered rows of
 * X (Section 4.3).
 *
 * Conventions for every entry point
 *   - All array pointers are DEVICE pointers on the current HIP device, owned by
 *     the caller; the library neither allocates, frees nor retains them.
 *   - The library keeps no state between calls: no process-wide settings, no
 *     hidden workspace.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  Calls return as soon as the launch is queued; they never
 *     synchronise and never read device memory on the host.
 *   - Return value: ES_OK or a negative es_status_t.  Nothing aborts or throws.
 *     On any error no kernel is launched and no output is touched.
 *   - Not checked (caller's contract): rowptr[0] == 0, rowptr non-decreasing,
 *     rowptr[N] == nnz < 2^31, 0 <= colidx[p] < N, X and Y do not overlap.
 */
#ifndef ES_SPMM_H
#define ES_SPMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Sampling strategy (Section 4.4).  FULL keeps every entry: the exact product. */
typedef enum { ES_FULL = 0, ES_BUCKET = 1, ES_FASTRAND = 2 } es_mode_t;

/* Row normalisation folded into the kernel (Section 6.1: sampling changes a
 * row's edge count, so the degree normalisation cannot stay outside the SpMM).
 * The row's sum is multiplied by a factor of its stored count n and its kept
 * count k; rows with k == 0 stay zero. */
typedef enum {
    ES_NORM_NONE = 0,     /* 1                                                     */
    ES_NORM_MEAN = 1,     /* 1 / k        mean over the kept neighbours            */
    ES_NORM_RSQRT = 2,    /* 1 / sqrt(k)  destination side of the symmetric norm   */
    ES_NORM_RESCALE = 3,  /* n / k        estimate of the full row sum             */
    ES_NORM_INV_DEGREE = 4 /* 1 / n       mean aggregation by the original degree:
                                         with vals == NULL no value array is read  */
} es_norm_t;

typedef enum {
    ES_OK = 0,
    ES_ERR_INVALID_ARG = -1,  /* null pointer, negative size, ld < F, W < 1, bad mode */
    ES_ERR_UNSUPPORTED = -2,  /* shape outside what the kernels cover, or N above the
                                 capacity of es_spmm_static_ws                     */
    ES_ERR_LAUNCH = -3        /* the HIP runtime rejected the launch                */
} es_status_t;

/*
 * es_spmm -- Algorithm 1 of the paper, fused sampling + SpMM.
 *
 * For every row r (n = rowptr[r+1] - rowptr[r] stored entries):
 *     k = n                      for ES_FULL
 *     k = min(n, W)              for ES_BUCKET / ES_FASTRAND   (Section 4.2)
 *     slot i in [0, k) reads the row's entry number
 *         i                               ES_FULL, ES_BUCKET, or n <= W
 *                                         (Section 4.2: a row that fits is kept
 *                                         whole; Section 4.4: Bucket = first W)
 *         (off + i * P) mod n             ES_FASTRAND with n > W  (Equation 2)
 *       P   = first of 577, 587, 593, 599 that does not divide n (577 is the
 *             paper's multiplier; the fallbacks keep the k picks distinct)
 *       off = 0 when seed == 0 (exactly Equation 2); otherwise the high 32 bits
 *             of output number r+1 of the SplitMix64 generator seeded with
 *             `seed`, reduced mod n (a per-row rotation; the picks stay distinct)
 *     Y[r, c] = sum over the k slots of vals[p] * X[colidx[p], c],  c in [0, F)
 * Y is overwritten (rows with n == 0 become zeros).  Accumulation is fp32; the
 * summation order is unspecified.  X is meant to hold finite values: a kernel
 * may add zero times a row of X that the output row gathers anyway, so an
 * output element whose exact value is +-Inf may come out as NaN.
 *
 *   rowptr  [N+1] int32          colidx [nnz] int32
 *   vals    [nnz] fp32, or NULL = every stored entry is 1 (unweighted graph)
 *   X       N rows of F fp32, row stride ldx >= F elements
 *   Y       N rows of F fp32, row stride ldy >= F elements
 *   nnz     rowptr[N]; used only to pick a launch shape (mean row length) --
 *           results never depend on it
 *   W       cap per row, >= 1 (ignored for ES_FULL).  Any W is accepted: rows
 *           longer than one LDS tile are staged tile by tile.
 *   seed    see above; ES_BUCKET and ES_FULL ignore it
 * X and Y must be 4-byte aligned.  Rows are read with 128-bit loads for every
 * F >= 4; when F, ldx, ldy are multiples of 4 and X, Y are 16-byte aligned the
 * aligned kernels run, otherwise variants that tolerate 4-byte-aligned rows
 * (F = 41 with ldx = 41, say).
 */
int es_spmm(const int32_t* rowptr, const int32_t* colidx, const float* vals,
            const float* X, float* Y,
            int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy,
            int32_t W, int32_t mode, uint64_t seed, void* stream);

/*
 * es_spmm_norm -- es_spmm with the row factor `norm` (an es_norm_t) applied to
 * every output row before it is stored.  es_spmm is es_spmm_norm with
 * ES_NORM_NONE; every other argument and rule is the same.  The paper gives no
 * formula for its in-kernel normalisation; the factors above are this
 * library's definition of it.
 */
int es_spmm_norm(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                 const float* X, float* Y,
                 int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy,
                 int32_t W, int32_t mode, uint64_t seed, int32_t norm, void* stream);

/*
 * es_spmm_backward -- the transposed product  dX = sample_W(A)^T * dY, i.e. the
 * gradient of es_spmm_norm's output with respect to X for the same W, mode,
 * seed and norm (training is the use Section 6.2 of the paper points to; the
 * per-call seed gives a different edge subset per iteration).
 *     dX[c, :] = sum over rows r and kept slots of r whose column is c
 *                of  factor_r * vals[p] * dY[r, :]
 *   dY  N rows of F fp32, row stride ldy >= F (input)
 *   dX  N rows of F fp32, row stride ldx >= F (output, fully overwritten: the
 *       library zero-fills it with a kernel of its own, then accumulates with
 *       fp32 atomic adds, so the summation order -- and the last bits -- may
 *       differ from launch to launch).  dX must not overlap dY.
 * Every other argument as in es_spmm_norm.
 */
int es_spmm_backward(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                     const float* dY, float* dX,
                     int64_t N, int64_t nnz, int32_t F, int32_t ldy, int32_t ldx,
                     int32_t W, int32_t mode, uint64_t seed, int32_t norm, void* stream);

/*
 * es_spmm_sample_edges -- the sampler of Section 4.2 / 4.4 on its own, for
 * verification.  Runs the same device sampler and slot-to-lane schedule as
 * es_spmm and writes, for row r and slot i < k_r, the CSR position
 * rowptr[r] + (entry number of slot i) into pos[r * W + i]; slots i >= k_r get
 * -1; cnt[r] = k_r = min(n_r, W).  mode must be ES_BUCKET or ES_FASTRAND.
 *   pos [N * W] int32 (device), cnt [N] int32 (device); N * W must be < 2^31.
 *   rows_per_wave: 0 = the library's default schedule, a power of two in
 *   [1, 64] = that many rows share a wavefront, -1 = the long-row schedule (a
 *   whole wavefront per row, the sampler restarted at every 256-slot segment).
 *   Every value must produce the same output; tests sweep it.
 */
int es_spmm_sample_edges(const int32_t* rowptr, int64_t N, int32_t W, int32_t mode,
                         uint64_t seed, int32_t rows_per_wave,
                         int32_t* pos, int32_t* cnt, void* stream);

/*
 * es_spmm_materialize -- write the sampled graph out as a CSR matrix of its
 * own: the "pre-sampled graph" of Section 5.6, which the paper feeds to
 * unsampled SpMM kernels to separate the cost of sampling from the cost of the
 * product.  Row r of the output holds the k_r = min(n_r, W) entries es_spmm
 * would stage, in slot order (mode ES_FULL copies the matrix).
 *   out_rowptr [N+1] int32, written: prefix sums of k_r (out_rowptr[0] = 0)
 *   out_colidx, out_vals: written; capacity at least min(nnz, N*W) entries
 *   vals == NULL writes ones.  nnz: rowptr[N], a launch-shape hint as in es_spmm.
 * es_spmm(out_rowptr, out_colidx, out_vals, ..., ES_FULL) then sums exactly the
 * entries es_spmm(rowptr, colidx, vals, ..., W, mode, seed) sums.
 */
int es_spmm_materialize(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                        int64_t N, int64_t nnz, int32_t W, int32_t mode, uint64_t seed,
                        int32_t* out_rowptr, int32_t* out_colidx, float* out_vals,
                        void* stream);

/*
 * es_spmm_materialize_transposed -- the TRANSPOSE of the sampled graph as a CSR
 * matrix of its own (the sampled graph in CSC form).  Row c of the output lists,
 * for every kept entry of es_spmm_norm(..., W, mode, seed, norm) whose column is
 * c, the row r it came from and the value factor_r * vals[p].  With it the
 * backward pass is a gather instead of an atomic scatter:
 *     es_spmm(out_ptr, out_idx, out_vals, dY, dX, ..., ES_FULL)
 * computes the same dX as es_spmm_backward, and the structure can be reused for
 * every product that shares (W, mode, seed, norm).
 *   out_ptr  [N+1] int32, written: start of each output row (out_ptr[N] = kept total)
 *   out_end  [N]   int32, written: end of each output row (= out_ptr[c+1]); the
 *            build advances it entry by entry, so it is an output, not scratch
 *   out_idx, out_vals: written; capacity at least min(nnz, N*W) entries
 * The order of the entries inside an output row is unspecified (they are placed
 * through an atomic cursor) and may differ from launch to launch.
 */
int es_spmm_materialize_transposed(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                                   int64_t N, int64_t nnz, int32_t W, int32_t mode, uint64_t seed,
                                   int32_t norm, int32_t* out_ptr, int32_t* out_end,
                                   int32_t* out_idx, float* out_vals, void* stream);

/*
 * es_spmm_transpose_graph -- the transposed graph that es_spmm_backward_pull
 * reads: A^T in CSR form, built ONCE per graph (it does not depend on W, mode or
 * seed).  Row c of the result lists every stored entry (r, c) of A as the row r
 * it came from, its entry number idx inside row r, the slot that reads it under
 * Equation 2, and its value.
 *   t_ptr  [N+1] int32, written: start of each row of A^T (t_ptr[N] = nnz)
 *   t_end  [N]   int32, written: end of each row (= t_ptr[c+1]); the build
 *          advances it entry by entry
 *   t_row  [nnz] int32, written: the row r of A the entry belongs to
 *   t_idx  [nnz] int32, written: its entry number inside that row, 0 .. n_r - 1
 *   t_slot [nnz] int32, written: (idx * P^-1) mod n_r, the slot i for which
 *          Equation 2, (i * P) mod n_r, gives idx (P: the row's multiplier)
 *   t_vals [nnz] fp32, written (vals == NULL: ones)
 *   t_pinv [N]   int32, written: P^-1 mod n_r per row (0 for rows of < 2 entries)
 * The order of the entries inside a row of A^T is unspecified (atomic cursor).
 */
int es_spmm_transpose_graph(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                            int64_t N, int64_t nnz, int32_t* t_ptr, int32_t* t_end, int32_t* t_row,
                            int32_t* t_idx, int32_t* t_slot, float* t_vals, int32_t* t_pinv,
                            void* stream);

/*
 * es_spmm_backward_pull -- the same dX = sample_W(A)^T * dY as es_spmm_backward,
 * computed as a gather over the transposed graph instead of an atomic scatter
 * (training is the use Section 6.2 points to; there the graph stays and the seed
 * changes every iteration).  Row c of dX sums factor_r * a_rc * dY[r, :] over the
 * stored entries (r, c) that es_spmm_norm(..., W, mode, seed, norm) keeps for row
 * r; whether it keeps entry idx of a row of n entries follows from inverting
 * the sampling rule of Section 4.4: always for ES_FULL or n <= W; idx < W for
 * ES_BUCKET; for ES_FASTRAND the slot that reads the entry is
 * ((idx - off) * P^-1) mod n = (t_slot - off * P^-1) mod n (Equation 2 solved
 * for the slot), kept iff that slot is < W.  No atomics: every output row is
 * written once, results are bit-reproducible.
 *   rowptr            the ORIGINAL graph's row pointers [N+1]
 *   t_ptr .. t_pinv   as written by es_spmm_transpose_graph for that graph (t_end
 *                     is not needed)
 *   t_rows            [2 * N] int32, 8-byte aligned, scratch: every call
 *                     overwrites it with each row's (length, rotation) for this
 *                     seed; calls that share it must be ordered (same stream)
 *   dY  N rows of F fp32, row stride ldy (input); dX likewise, stride ldx (output,
 *       fully overwritten); they must not overlap
 *   nnz, W, mode, seed, norm as in es_spmm_backward.
 */
int es_spmm_backward_pull(const int32_t* rowptr, const int32_t* t_ptr, const int32_t* t_row,
                          const int32_t* t_idx, const int32_t* t_slot, const float* t_vals,
                          const int32_t* t_pinv, int32_t* t_rows,
                          const float* dY, float* dX,
                          int64_t N, int64_t nnz, int32_t F, int32_t ldy, int32_t ldx,
                          int32_t W, int32_t mode, uint64_t seed, int32_t norm, void* stream);

/*
 * es_spmm_validate_csr -- checks on the device what every other entry point
 * takes on trust (see "Not checked" above); meant to be run once on a graph of
 * unknown origin, since a bad column id makes es_spmm read outside X.
 *   report [4] int32 (device), written:
 *     report[0]  row-pointer faults: pairs with rowptr[r+1] < rowptr[r] or
 *                outside [0, nnz], plus one each if rowptr[0] != 0 or
 *                rowptr[N] != nnz
 *     report[1]  column ids outside [0, N) (only rows with a sound pointer
 *                pair are inspected)
 *     report[2]  rows whose column ids are not strictly increasing -- legal,
 *                but "the first W entries" of ES_BUCKET (Section 4.4) then
 *                means storage order, not the lowest-numbered neighbours
 *     report[3]  length of the longest row
 * The graph is usable when report[0] == 0 and report[1] == 0.
 */
int es_spmm_validate_csr(const int32_t* rowptr, const int32_t* colidx, int64_t N, int64_t nnz,
                         int32_t* report, void* stream);

/*
 * es_launch_opts_t -- per-call launch-shape overrides (Section 4.5 of the paper,
 * "thread management" and "load balancing": how rows map onto thread groups
 * and how skewed rows are balanced).  Passed by pointer to the *_ex entry
 * points and to es_spmm_launch_info; NULL, or a field left 0, means "the
 * library's own choice".  The struct is read during the call and not retained;
 * the library keeps no launch state between calls, so concurrent calls with
 * different options never interact.  No option changes which entries are
 * sampled; Y differs between settings only by fp32 summation order.
 */
typedef struct {
    int32_t rows_per_wave;       /* rows sharing one wavefront: a power of two in
                                    [1, 64], lowered when F needs more lanes per row
                                    (Section 4.2 assigns a thread group per row; the
                                    group is 64 / rows_per_wave lanes)              */
    int32_t lanes_per_row;       /* column slicing: cap the lanes spanning the
                                    feature columns at 4, 8, 16, 32 or 64, so one
                                    workgroup covers 4 * lanes columns and the rows
                                    are swept once per column slice (a smaller piece
                                    of X per sweep; the sampler runs once per slice).
                                    -1 = never slice.  Ignored by the backward pass */
    int32_t long_row_threshold;  /* a row keeping more entries than this is cut into
                                    256-entry segments that several workgroups sum
                                    with atomic adds (load balance for skewed degree
                                    distributions); any positive value             */
    int32_t column_partition;    /* es_spmm_ws only: 1 = run the column-partitioned
                                    product whenever it applies (a workspace is given,
                                    mode is not ES_BUCKET, N >= 512), -1 = never, 0 =
                                    the library decides from N, F, W and nnz / N      */
    int32_t kernel;              /* 1 = the row kernel (a row, or a row per team of
                                    lanes, on a wave at a time); 2 = the flattened
                                    kernel (a wave lays 64 or 128 / lanes_per_row rows
                                    end to end and deals their entries to its edge
                                    slots: for short rows and narrow column slices;
                                    the library picks it by itself where that
                                    measured faster); falls back to 1 where 2 does not
                                    apply (F < 4, the backward pass, FastRand in the
                                    column-partitioned product)                       */
} es_launch_opts_t;

/*
 * es_spmm_ex -- es_spmm_norm with per-call launch options (`opts` may be NULL).
 * ES_ERR_INVALID_ARG for an option outside the ranges above.
 */
int es_spmm_ex(const int32_t* rowptr, const int32_t* colidx, const float* vals,
               const float* X, float* Y,
               int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy,
               int32_t W, int32_t mode, uint64_t seed, int32_t norm,
               const es_launch_opts_t* opts, void* stream);

/*
 * es_spmm_ws -- es_spmm_ex with a caller-owned workspace, which lets the library
 * run the column-partitioned form of the product.  Stage 2 of Algorithm 1
 * (Section 4.3) gathers one row of X per kept entry; on a graph with hundreds of
 * entries per row and an X several times larger than a 4 MB L2 nearly every
 * gather misses.  The partitioned form cuts the columns of A into 8 equal
 * ranges, lets each of the chip's 8 XCDs multiply only the entries of "its"
 * range -- so it only ever touches one eighth of X -- and builds every row of Y
 * in 8 stream-ordered launches (the first stores, the others add).  It is used
 * for ES_FULL and ES_FASTRAND when the library (or opts->column_partition)
 * decides so.  A row's share of a column range is found by binary search in its
 * column ids, so the locality is there for rows stored in increasing column
 * order (the usual CSR); for any other order the result is still the same
 * product -- the eight pieces always tile the row -- only the locality is lost.
 * Same sampled entries as es_spmm; Y differs only by fp32 summation order and
 * is bit-reproducible.
 *   workspace        device memory, 16-byte aligned, at least
 *                    es_spmm_workspace_bytes(N) bytes; contents on entry are
 *                    irrelevant, contents on return are unspecified.  NULL or
 *                    too small: the call runs exactly as es_spmm_ex.
 * Calls that share a workspace must be ordered (same stream).
 */
size_t es_spmm_workspace_bytes(int64_t N);

int es_spmm_ws(const int32_t* rowptr, const int32_t* colidx, const float* vals,
               const float* X, float* Y,
               int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy,
               int32_t W, int32_t mode, uint64_t seed, int32_t norm,
               const es_launch_opts_t* opts, void* workspace, size_t workspace_bytes, void* stream);

/*
 * es_spmm_static_ws -- es_spmm_ws for callers that cannot allocate device
 * memory for a workspace: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, rules and results
 * as es_spmm_ws, except that the workspace is a fixed array inside the library
 * (static device memory of ES_SPMM_STATIC_WS_MAX_ROWS * 32 bytes, held on every
 * GPU the library runs on until the process ends).  The call allocates and
 * frees nothing, on the host or on the device.
 *   N > ES_SPMM_STATIC_WS_MAX_ROWS  ->  ES_ERR_UNSUPPORTED, nothing is launched
 *                                       (use es_spmm_ws with a workspace of your own)
 * Every call on a GPU shares that GPU's array: calls that may overlap in time
 * on one GPU (different streams, different threads) race on it and must be
 * ordered by the caller; calls on one stream are ordered by the stream.  The
 * array keeps the previous call's contents; every call overwrites the part it
 * reads, so nothing needs clearing in between.
 */
#define ES_SPMM_STATIC_WS_MAX_ROWS 1048576

int es_spmm_static_ws(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                      const float* X, float* Y,
                      int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy,
                      int32_t W, int32_t mode, uint64_t seed, int32_t norm,
                      const es_launch_opts_t* opts, void* stream);

/* es_spmm_backward_ex -- es_spmm_backward with per-call launch options. */
int es_spmm_backward_ex(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                        const float* dY, float* dX,
                        int64_t N, int64_t nnz, int32_t F, int32_t ldy, int32_t ldx,
                        int32_t W, int32_t mode, uint64_t seed, int32_t norm,
                        const es_launch_opts_t* opts, void* stream);

/*
 * es_spmm_launch_info -- the launch shape es_spmm_ws (backward == 0; without a
 * workspace, es_spmm_ex runs the same shape with column_ranges = 1) or
 * es_spmm_backward_ex (backward != 0) would pick for these sizes and options
 * (`opts` may be NULL), without launching anything and without a GPU.
 * `aligned16`: both matrices are 16-byte aligned.  The shape is how Section
 * 4.5's "thread management" maps onto wave64: lanes_per_row x edge_slots lanes
 * form a row's thread group, rows_per_wave such groups share a wavefront.
 * N must be >= 1.
 */
typedef struct {
    int32_t vector_width;        /* floats per load: 4 (128-bit) or 1              */
    int32_t aligned;             /* 1: rows are 16-byte aligned                     */
    int32_t lanes_per_row;       /* G: lanes spanning the feature columns           */
    int32_t chunks_per_lane;     /* CH: column chunks each of those lanes owns      */
    int32_t rows_per_wave;       /* R                                               */
    int32_t edge_slots;          /* E = 64 / (R * G): entries of a row in flight    */
    int32_t loads_in_flight;     /* U: independent loads per lane before the FMAs   */
    int32_t tile_slots_per_row;  /* LDS (column, value) slots per row and refill    */
    int32_t long_row_threshold;  /* rows keeping more entries are split             */
    int64_t long_row_workgroups; /* leading workgroups that serve such rows (or 0)  */
    int64_t grid_x, grid_y;      /* launch grid, 256 threads per workgroup          */
    int32_t flattened;           /* 1: the flattened kernel would run (rows_per_wave then
                                    is the number of rows a wave lays end to end)     */
    int32_t column_ranges;       /* 8: es_spmm_ws with a sufficient workspace would run
                                    the column-partitioned product (grid_x then is the
                                    grid of each of its 8 launches); 1: it would not  */
} es_launch_info_t;

int es_spmm_launch_info(int64_t N, int64_t nnz, int32_t F, int32_t ldx, int32_t ldy, int32_t W,
                        int32_t mode, int32_t aligned16, int32_t backward,
                        const es_launch_opts_t* opts, es_launch_info_t* info);

/* Human-readable name of a status code (static storage, never NULL). */
const char* es_spmm_status_string(int status);

/* Largest W es_spmm accepts for feature width F (tiles are refilled, so this is
 * INT32_MAX for every valid F; 0 for F < 1). */
int32_t es_spmm_max_W(int32_t F);

/* Number of (colidx, vals) slots one row can hold in LDS at once when
 * `rows_per_wave` rows share a wavefront (Section 4.2's shared-memory width);
 * rows_per_wave = 0 reports the single-row tile.  0 for an invalid argument. */
int32_t es_spmm_tile_slots(int32_t rows_per_wave);

#ifdef __cplusplus
}
#endif
#endif /* ES_SPMM_H */
