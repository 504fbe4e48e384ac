/*
 * libstrassen_tc -- fp64 tensor contraction  C := alpha * A * B + beta * C  on one AMD MI355X (gfx950),
 * evaluated classically or through one- or two-level Strassen, with no explicit tensor transposition.
 *
 * The operation is the general tensor contraction of the paper (Sec. 2.3 "Tensor Contraction"):
 * every index label occurs in exactly two of the three tensors; labels shared by A and C form the free
 * bundle I, labels shared by B and C the free bundle J, labels shared by A and B the contracted bundle P,
 *
 *     C[I J] := alpha * sum_P A[I P] * B[P J] + beta * C[I J],
 *
 * with the labels of each tensor listed in any order and every dimension carrying its own stride
 * (Sec. 2.3 "General stride layouts").  The library views the contraction as a matrix product over the
 * bundles, addressed through scatter vectors and block scatter vectors (Sec. 2.3 "Block Scatter Matrix
 * View"), splits that matrix view 2x2 (4x4) for Strassen (Sec. 3, the display of the general
 * primitive; the seven products M_0..M_6 displayed in Sec. 2.2), forms the operand sums while staging tiles into LDS (Sec. 4.1) and adds each
 * product to several blocks of C from registers (Sec. 4.2).  Variants (Sec. 4.1): ABC keeps no temporary,
 * AB stores each product M densely and then accumulates it into C, Naive also stores the operand sums.
 *
 * Conventions
 *   - All tensors are fp64.  Lengths and strides are in elements.  Device pointers address the element
 *     whose multi-index is all zeros.
 *   - Every function returns TC_OK (0) or a negative tc_status_t; nothing throws or aborts across this
 *     boundary.  tc_strerror() names a status.
 *   - Descriptor arrays are read during tc_plan only; the caller may free them afterwards.
 *   - A plan owns small device-side tables (scatter vectors, block scatter vectors, product schedule) that
 *     tc_destroy() releases.  A plan is immutable after creation and may be used for any number of
 *     tc_contract() calls; calls that overlap in time on different streams must not share C or workspace.
 *   - tc_contract() only enqueues work on the given HIP stream and never synchronises with the host.
 */
#ifndef STRASSEN_TC_H
#define STRASSEN_TC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tc_plan tc_plan_t; /* opaque; created by tc_plan(), released by tc_destroy() */

typedef enum {
    TC_VARIANT_NAIVE = 0, /* operand sums and product stored in dense temporaries (Sec. 4.1) */
    TC_VARIANT_AB = 1,    /* operand sums fused into tile staging; product M stored densely, then accumulated into C */
    TC_VARIANT_ABC = 2,   /* fully fused: no temporaries, each product added to up to 2^L blocks of C from registers */
    TC_VARIANT_HYBRID = 3 /* the operand sums of the first level are stored in dense temporaries as in Naive (a single block
                           * is used in place), everything after that is fused as in ABC: at one level each product of
                           * two temporaries is added to its blocks of C; at two levels the second level runs inside
                           * the kernel and each of its products is added to up to four blocks of C.  Not one of the
                           * paper's variants: this GPU gathers dense temporaries and two-block sums at a higher rate
                           * than the two- and four-block sums of one- and two-level ABC. */
} tc_variant_t;

typedef enum {
    TC_OK = 0,
    TC_ERR_NULL = -1,      /* a required pointer argument is NULL */
    TC_ERR_NDIM = -2,      /* ndim < 0 or > TC_MAX_NDIM */
    TC_ERR_LABEL = -3,     /* label repeated inside a tensor, or not in exactly two tensors */
    TC_ERR_LENGTH = -4,    /* negative length, or one label with two different lengths */
    TC_ERR_STRIDE = -5,    /* negative stride, zero stride on a dimension longer than 1, or two elements of C share a
                            * location.  (Sec. 2.3 "General stride layouts" allows any strides in the naturals.  Layouts
                            * of C whose dimensions nest, with or without padding, are always accepted; layouts that
                            * interleave dimensions are checked exactly up to 2^22 elements and refused beyond that.) */
    TC_ERR_LEVEL = -6,     /* level not in {0, 1, 2} and not TC_LEVEL_AUTO */
    TC_ERR_VARIANT = -7,   /* unknown variant */
    TC_ERR_WORKSPACE = -8, /* workspace is NULL although tc_plan_workspace_bytes() > 0 */
    TC_ERR_HIP = -9,       /* a HIP runtime call failed (no device, out of memory, launch failure) */
    TC_ERR_STATE = -10,    /* plan was created host-only and cannot run, or option value out of range */
    TC_ERR_RANGE = -11,    /* output buffer too small / index out of range in an inspection call */
    TC_ERR_CAPACITY = -12  /* tc_contract_static: the plan's workspace exceeds TC_STATIC_WORKSPACE_BYTES */
} tc_status_t;

#define TC_MAX_NDIM 16

/* Sec. 5 ("Performance Model") lets the library choose: pass TC_LEVEL_AUTO and/or TC_VARIANT_AUTO to tc_plan() and
 * the plan takes the level in {0, 1, 2} and/or the variant with the smallest modelled time (tc_plan_predict). */
#define TC_LEVEL_AUTO (-1)
#define TC_VARIANT_AUTO (-1)

/* One tensor of the contraction (Sec. 2.3 "Tensor" and "General stride layouts").
 * idx holds ndim single-character labels, e.g. "aebf" (not necessarily NUL-terminated). */
typedef struct {
    int ndim;
    const int64_t *len;    /* host array, ndim entries */
    const int64_t *stride; /* host array, ndim entries, in elements */
    const char *idx;       /* host array, ndim labels */
} tc_tensor_desc_t;

/* Optional knobs for tc_plan_ex(); zero-initialise for defaults. */
typedef struct {
    int bs_block;   /* entries per block of the block scatter vectors (Sec. 2.3); 0 = default 16 */
    int host_only;  /* 1: analyse and schedule on the host only (no HIP call); the plan cannot run */
    int no_merge;   /* 1: one kernel launch per Strassen product even where destinations are disjoint */
    int split_k;    /* level 0 only: 0 or 1 = off; 2..4 = cut the contracted bundle into that many chunks whose products
                     * run side by side into dense temporaries and are summed into C by one element-wise pass (for
                     * shapes with too few 128 x 128 tiles to fill the device; needs workspace; not from the paper);
                     * -1 = as many chunks as the performance model likes best (1 when tail_split is automatic:
                     * the tail split then does this job inside the kernel) */
    int tail_split; /* 0 = automatic: where the tiles of a launch do not fill a whole number of rounds of the device's
                     * compute units, the left-over tiles are cut along the contracted bundle into chunks computed by
                     * one workgroup each, and a small second kernel adds the chunks (in a fixed order: results are
                     * reproducible) and updates the destinations; the chunk count is the one the performance model
                     * likes best, possibly none; needs workspace for the chunks (not from the paper);
                     * -1 = never; 2..16 = that many chunks (each a multiple of 64 entries long, so possibly fewer)
                     * in every launch that has a tail, whatever the model says (for tests and measurements) */
    int tile_n;     /* tile shape of the launches whose products have single-block operand sums (level 0, and the stored-sum
                     * variants): 0 = the performance model chooses; 128 = 128 x 128 tiles, one workgroup of 512 threads
                     * per compute unit; 64 = 128 x 64 tiles, two workgroups of 256 threads per compute unit (one
                     * workgroup's set-up and destination update overlap the other's matrix-core work: the faster shape
                     * where every tile is gathered by stride, the slower one through the scatter tables; a launch that
                     * mixes the two kinds of tile is kept in 128 x 128 tiles by the automatic choice).  Launches with
                     * multi-block sums always use 128. */
    int no_peel;    /* Sizes that 2^level does not divide (Sec. 3, last paragraph, names dynamic peeling and zero padding):
                     * 0 = the Strassen products cover a leading part of the row and of the column bundle and one
                     * classical product each does the rows / columns left over (dynamic peeling).  The leading part is
                     * a whole number of 128-wide tiles per block if that leaves at most a tenth of the bundle over;
                     * else, in the ABC and AB variants, if the bundle is no whole number of equal blocks and at least
                     * 2^level tiles long, the largest whole number of block units (2 or 16 entries); else nothing is
                     * peeled.  The contracted bundle and whatever is not peeled are completed with zeros.
                     * 1 = zero padding everywhere (the last block of a direction is then shorter than the others, and
                     * sums of blocks of different length run a slower, padding-checked loop in the tiles where they differ). */
    int no_repack;  /* An operand that the kernel could only gather element by element, with consecutive entries of the
                     * gather direction in different memory lines (both A and B have their unit-stride index in the
                     * contracted bundle, whose order can follow only one of them; or a tensor without a unit-stride
                     * index), is copied once into a dense temporary in the workspace by an element-wise pass and
                     * the products read that (the packing of Sec. 4.1 made explicit, once per contraction; classical,
                     * ABC and AB schedules).  1 = never: every product gathers from the caller's tensors. */
} tc_options_t;

/* Facts about a plan (tc_plan_info). */
typedef struct {
    int64_t m, n, k;      /* bundle lengths N_I, N_J, N_P of the matrix view */
    int level_requested;
    int level;            /* level actually executed: lowered while a bundle is shorter than 2^level */
    int variant;
    int n_products;       /* 1, 7 or 49 (fewer if blocks lie wholly in the zero padding); the chunks with split_k */
    int n_launches;       /* kernel launches per tc_contract() */
    int bs_block;
    int a_mode, b_mode;   /* 0: stride-1 direction of the operand is its free bundle, 1: the contracted bundle */
    int64_t mb, nb, kb;   /* extents of one Strassen block: ceil(length / 2^level) rounded up to an even number (to a multiple of
                           * 16 where an operand reads the bundle through its block scatter vector) */
    char I[TC_MAX_NDIM + 1], J[TC_MAX_NDIM + 1], P[TC_MAX_NDIM + 1]; /* labels of each bundle, fastest first, NUL-terminated */
    int64_t m_peel, n_peel; /* last rows / columns of the matrix view left to classical edge products (dynamic peeling); the
                             * 2^level x 2^level block grid of tc_plan_schedule covers the first m - m_peel rows and
                             * n - n_peel columns */
} tc_plan_info_t;

/* One term of a Strassen product as scheduled (tc_plan_schedule): block (row, col) of the 2^L x 2^L grid and its sign. */
typedef struct {
    int n_a, n_b, n_c;
    int a_row[4], a_col[4], a_sign[4];
    int b_row[4], b_col[4], b_sign[4];
    int c_row[4], c_col[4], c_sign[4];
    int c_first[4]; /* 1 where this product is the first to write that block of C (beta is applied there) */
    int launch;     /* index of the kernel launch that runs this product */
} tc_product_t;

/* Parameters of the performance model (Sec. 5, notation table): tau_a = 1 / (rho_a * peak_flops),
 * tau_b = 8 / (rho_b * bandwidth).  The arithmetic penalty rho_a depends on how many blocks the larger operand sum
 * of a product has (1, 2, 4: index 0, 1, 2), which is what makes this kernel slower; rho_a holds for the tiles gathered
 * by stride, rho_table for the tiles gathered through the scatter tables (general layouts: the fraction of each kind
 * in a launch is what tc_launch_info_t.tiles_table_free reports); in 128 x 64 tiles they are multiplied by rho_small
 * and rho_small_table respectively, and both by rho_gather for launches that gather an operand element by element (the
 * operand has no stride-one index on the side the gather runs along: the model's bandwidth penalty for such operands,
 * which here shows as matrix cores waiting for the gather).  t_launch is added per kernel launch; the arithmetic term
 * counts whole waves of tiles (one 128 x 128 tile or two 128 x 64 tiles per compute unit), each wave with a fixed cost
 * t_tile (gather tables, filling and draining a tile's pipeline).  lambda_ab is the fraction of the operand reads
 * T_m^{Ax} + T_m^{Bx} (every tile reads its panels of the summed blocks of A and B once) that is not hidden behind
 * the matrix cores, the counterpart of the model's prefetch efficiency lambda. */
typedef struct {
    double peak_flops;  /* flop/s of the device */
    double rho_a[3];
    double bandwidth;   /* bytes/s */
    double rho_b;
    double t_launch;    /* seconds */
    double t_tile;      /* seconds per wave of tiles */
    int units;          /* compute units: each runs one 128 x 128 tile, or two 128 x 64 tiles, at a time */
    int reserved[3];
    double rho_small;    /* 128 x 64 tiles: factor on rho_a (above 1 where two workgroups per compute unit hide each other's set-up) */
    double t_tile_small; /* 128 x 64 tiles: seconds per wave of tiles */
    double rho_gather;   /* element-by-element gathers: factor on rho_a */
    double lambda_ab;    /* weight of the operand reads */
    double rho_table[3]; /* as rho_a, for tiles gathered through the scatter tables */
    double rho_small_table; /* 128 x 64 tiles: factor on rho_table */
} tc_model_params_t;

/* One kernel launch of the plan's schedule, for inspection (tc_plan_launch). */
typedef struct {
    int kind;             /* 0: fused kernel (products), 1: element-wise kernel */
    int n_products;       /* fused: products sharing the launch */
    int max_terms;        /* fused: largest number of blocks in an operand sum of the launch */
    int tail_tiles;       /* fused: tiles cut into chunks (0: none); a split launch is followed by the kernel that adds the chunks */
    int tail_chunks;      /* chunks per tail tile */
    int terms_a, terms_b; /* fused: the kernel family of the launch = blocks in the operand sum of A and of B (1, 2 or 4 each;
                           * 0, 0: the family that counts up to four terms at run time) */
    int tile_n;           /* fused: tile columns, 128 or 64 (tiles always have 128 rows) */
    int64_t rows, cols;   /* extents of one product (fused) or of the pass (element-wise) */
    int64_t depth;        /* fused: contracted extent of one product */
    int64_t tiles;        /* fused: 128 x tile_n tiles of the launch */
    int64_t tail_kc;      /* contracted entries per chunk */
    int64_t tiles_table_free; /* fused: tiles gathered by stride, without scatter tables (Sec. 4.1 "Packing": every block
                               * scatter entry of the tile's rows and columns is non-zero in every summed block, the
                               * contracted bundle is one constant-stride run, no zero padding in the tile); the other
                               * tiles of the launch go through the scatter tables */
    double moved_elems;   /* what the model's memory terms count (Sec. 5, T_m^{Cx} and T_m^{+}): fused: destination elements
                           * read or written by the updates of all products; element-wise: elements read or written */
    int pairs_a, pairs_b; /* fused: 1 if the operand is gathered two contiguous elements at a time (it has a stride-one
                           * index on the side the gather runs along), 0 if element by element */
} tc_launch_info_t;

/* Modelled time of one tc_contract() with beta != 0, in seconds, split as in Sec. 5 eq. (2)-(4):
 * arith = W_a^x T_a^x (whole waves of tiles), c_update = W_m^{C x} T_m^{C x} (destination updates of the products),
 * temporaries = the T_m^{+} terms (element-wise passes of the AB and Naive variants), launch = launches * t_launch.
 * Reading A and B is taken as hidden behind the matrix cores.  A launch that splits its tail counts its whole tiles in
 * whole waves of full depth plus the chunks in whole waves of chunk depth (arith), the chunks written and read back
 * (temporaries) and one more launch. */
typedef struct {
    double total, arith, c_update, temporaries, launch;
    double operands; /* T_m^{Ax} + T_m^{Bx}, weighted by lambda_ab (part of total) */
} tc_model_time_t;

/* Build a plan: classify labels into bundles (Sec. 2.3), choose the order inside each bundle, compute the
 * scatter and block scatter vectors on the device (planner kernel, enqueued on `stream`, a hipStream_t or NULL),
 * and schedule the 1 / 7 / 49 products of level 0 / 1 / 2 (Sec. 2.2, the display of the seven products M_0..M_6; Sec. 3, the display of the general primitive).
 * On failure *plan_out is set to NULL.  Synchronises `stream` before returning. */
int tc_plan(tc_plan_t **plan_out, const tc_tensor_desc_t *A, const tc_tensor_desc_t *B, const tc_tensor_desc_t *C,
            int level, int variant, void *stream);
int tc_plan_ex(tc_plan_t **plan_out, const tc_tensor_desc_t *A, const tc_tensor_desc_t *B, const tc_tensor_desc_t *C,
               int level, int variant, const tc_options_t *opts, void *stream);

/* Bytes of device workspace tc_contract() needs.  Sec. 4.1 names the temporaries of each variant: ABC keeps none; AB
 * stores every product M as a dense matrix before it is accumulated into C (one block of C here: the products run one
 * after the other); Naive also stores the operand sums (plus one block of A and one of B); HYBRID: one first-level
 * block of A and of B.  Level 0 needs none unless split_k is used.  Where a launch splits its tail
 * (tc_options_t.tail_split) add one dense tile (128 x tile_n elements: 128 or 64 KiB) per chunk of a tail tile (at
 * most 1024 chunks). */
size_t tc_plan_workspace_bytes(const tc_plan_t *plan);

/* C := alpha * A * B + beta * C: the tensor contraction as defined in Sec. 2.3 ("Tensor Contraction": the sum over the
 * contracted bundle P for every multi-index of I and J, each element located by the general stride layout), evaluated
 * on the matrix view by the plan's schedule: per product the general primitive of Sec. 3 (operand sums formed while
 * tiles are staged, Sec. 4.1; the product added to each of its blocks of C, or stored as M, Sec. 4.2 and 4.1).
 * A_dev, B_dev, C_dev, workspace_dev are device pointers owned by the caller;
 * C must not overlap A, B or the workspace.  With beta == 0, C is written without being read.
 * A bundle of length zero: empty I or J makes the call a no-op; empty P gives C := beta * C.
 * Work is enqueued on `stream` in order; the call returns without waiting for it. */
int tc_contract(const tc_plan_t *plan, double alpha, const double *A_dev, const double *B_dev, double beta,
                double *C_dev, void *workspace_dev, void *stream);

/* tc_contract() for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The workspace is a buffer of TC_STATIC_WORKSPACE_BYTES that
 * the library holds in the memory of every GPU it runs on, from the time its code is loaded there until the process
 * ends; the call itself allocates and frees nothing.  Same kernels, same launch order and same results (bit for bit)
 * as tc_contract() with a workspace of tc_plan_workspace_bytes().  Returns TC_ERR_CAPACITY, and enqueues nothing, if
 * the plan needs more than TC_STATIC_WORKSPACE_BYTES (then use tc_contract()).  All calls on one GPU share that
 * GPU's buffer: two calls that overlap in time on one GPU (different streams or threads) race; calls in stream order
 * are safe.  The buffer keeps the previous call's contents, which is harmless: every kernel writes the part of the
 * workspace it later reads.  The plan must have been created with the same GPU current. */
#define TC_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
int tc_contract_static(const tc_plan_t *plan, double alpha, const double *A_dev, const double *B_dev, double beta,
                       double *C_dev, void *stream);

/* Release the plan and its device tables.  NULL is accepted. */
int tc_destroy(tc_plan_t *plan);

const char *tc_strerror(int status);

/* Performance model (Sec. 5).  tc_model_defaults() fills the parameters measured on MI355X; tc_plan_predict()
 * evaluates the model for the plan's schedule (params == NULL: the defaults).  Host-only, no HIP call. */
int tc_model_defaults(tc_model_params_t *out);
int tc_plan_predict(const tc_plan_t *plan, const tc_model_params_t *params, tc_model_time_t *out);

/* Inspection (tests, tools). */
int tc_plan_info(const tc_plan_t *plan, tc_plan_info_t *out);
/* Schedule entry `index` (0 <= index < n_products). */
int tc_plan_schedule(const tc_plan_t *plan, int index, tc_product_t *out);
/* Launch `index` (0 <= index < n_launches; a fused launch that splits its tail counts once). */
int tc_plan_launch(const tc_plan_t *plan, int index, tc_launch_info_t *out);
/* Copy one planner output to host memory: which = 0..5 scatter vectors rscat_A, cscat_A, rscat_B, cscat_B, rscat_C, cscat_C;
 * 6..11 the block scatter vectors rbs_A, cbs_A, rbs_B, cbs_B, rbs_C, cbs_C (Sec. 2.3).  Returns the number of entries
 * (also when host_out is NULL), or a negative status; copies at most `capacity` entries.  Synchronous. */
int64_t tc_plan_vector(const tc_plan_t *plan, int which, int64_t *host_out, int64_t capacity);

/* ------------------------------------------------------------------------------------------------------------------
 * Tools for benchmarks (not for production call paths: the call below creates and destroys HIP events and blocks the
 * host until the work is done).
 * ------------------------------------------------------------------------------------------------------------------ */

/* Time spent per kind of kernel in one tc_contract() (tc_contract_timed). */
typedef struct {
    double fused_ms;        /* the gather + multiply + update kernel (Sec. 4.1, 4.2) */
    double elementwise_ms;  /* temporaries of the AB / Naive / HYBRID variants, split_k sums, C := beta C */
    int fused_launches, elementwise_launches;
} tc_launch_times_t;

/* Same work as tc_contract(), with a HIP event recorded on `stream` after every launch; waits for the last one and
 * writes the duration of launch i (the index tc_plan_launch() uses; a fused launch that splits its tail includes the
 * kernel that adds the chunks) to ms_out[i], in milliseconds.  Returns the number of launches, or a negative status
 * (TC_ERR_RANGE if capacity is smaller than the plan's n_launches). */
int tc_contract_launch_times(const tc_plan_t *plan, double alpha, const double *A_dev, const double *B_dev, double beta,
                             double *C_dev, void *workspace_dev, void *stream, double *ms_out, int capacity);

/* The same, summed per kind of kernel. */
int tc_contract_timed(const tc_plan_t *plan, double alpha, const double *A_dev, const double *B_dev, double beta,
                      double *C_dev, void *workspace_dev, void *stream, tc_launch_times_t *out);

/* What the FP64 matrix cores of this GPU sustain when they do nothing else: a kernel of independent MFMA chains, no
 * memory traffic (instruction 0: v_mfma_f64_4x4x4_4b_f64; 1: v_mfma_f64_16x16x4_f64, the one the library's kernels use).
 * Writes the achieved TFLOP/s to *tflops_out.  Uses the static workspace of tc_contract_static for its (discarded)
 * results; blocks until the measurement is done (about 50 ms). */
int tc_bench_mfma_peak(int instruction, void *stream, double *tflops_out);

#ifdef __cplusplus
}
#endif
#endif /* STRASSEN_TC_H */
