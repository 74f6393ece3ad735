/*
 * sagnn -- one GPU's share of the sparsity-aware block-row SpMM of full-graph GCN
 * training, for AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * Paper: "Sparsity-Aware Communication for Distributed Graph Neural Network Training"
 * (ICPP'24).  A process P(i) that owns row block A_i of the (transposed) adjacency matrix
 *   1. finds NnzCols(i,q), the nonzero column indices of each block A_iq, i.e. the rows of
 *      H_q it needs                                   (Sec. 4.1, paragraph defining NnzCols)
 *   2. obtains exactly those rows, packed one block after the other
 *                                                     (Alg. 1, statement "T <- [H[NnzCols..]]")
 *   3. multiplies: Z_i = sum_q A_iq H_q               (Sec. 4.1 block-sum equation; Alg. 1/2
 *                                                      "Z <- Z + SpMM(A_iq, H^)")
 *   4. applies the dense layer: H' = sigma(Z W)       (Sec. 2.1 forward equations; Alg. 1
 *                                                      "GEMM(Z, W)")
 *   5. and in the backward pass computes G' = (A G W^T) .* sigma'(Z') and Y = H'^T (A G)
 *                                                     (Sec. 2.1 backward equations)
 * The exchange between steps 2 and 3 (all-to-allv / isend-recv) is not part of this
 * library: the remote H is any device-resident matrix that is read only through the
 * packed row set.
 *
 * Conventions for every entry point
 *   - d_* pointers are device memory owned by the caller, h_* pointers are host memory
 *     owned by the caller.  The library allocates no device memory and keeps no state
 *     besides the last HIP error code and one small host descriptor per prepared SpMM
 *     workspace, from spmm_csr_prepare() until spmm_csr_release().
 *   - Matrices are row-major; ld* are leading dimensions in elements.
 *   - CSR: rowptr has m+1 int32 entries with rowptr[0] = 0 and rowptr[m] = nnz; colidx and
 *     val have nnz entries.  Entries of a row may be unsorted and may repeat: the planner
 *     treats them as a set, the products sum them.
 *   - Dense float pointers must be 16-byte aligned and ld* / f multiples of 4, otherwise
 *     SAGNN_EINVAL.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously unless stated otherwise.
 *   - Return value: SAGNN_OK or a negative error code.  Arguments are validated on the host
 *     before anything is launched; no entry point throws or aborts.  Kernels bounds-check
 *     every index they read from device memory (an out-of-range column index is clamped
 *     or skipped), so malformed device data cannot fault the GPU.
 */
#ifndef SAGNN_H
#define SAGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SAGNN_OK = 0,
  SAGNN_EINVAL = -1,    /* null pointer, negative size, misaligned pointer, unsupported f */
  SAGNN_ECAPACITY = -2, /* an output buffer or the workspace is too small                 */
  SAGNN_EFORMAT = -3,   /* validation requested and the CSR / block offsets are malformed  */
  SAGNN_EHIP = -4       /* a HIP runtime call failed; see sagnn_last_hip_error()            */
};

#define SAGNN_PLAN_VALIDATE 1u  /* flags bit 0 of spmm_plan_needed_rows */
#define SAGNN_PLAN_OBLIVIOUS 2u /* flags bit 1: plan of the sparsity-oblivious algorithm   */
#define SAGNN_PLAN_MULTIPASS 4u /* flags bit 2: never take the one-launch path of small blocks */

#define SAGNN_ACT_IDENTITY 0
#define SAGNN_ACT_RELU 1

#define SAGNN_GEMM_FP32 0 /* fp32 operands, fp32 MFMA                          */
#define SAGNN_GEMM_BF16 1 /* operands rounded to bfloat16 (RNE), fp32 accumulate */
#define SAGNN_GEMM_FP32_BF16X3 2 /* fp32 operands (finite, below 2^127), each split exactly into three
                                   bfloat16 terms (round to nearest, remainder, remainder); the six
                                   products down to 2^-16 of the leading one run on the bfloat16
                                   matrix cores with fp32 accumulation.  The dropped products are below
                                   2^-23 |x||w|: the accuracy of SAGNN_GEMM_FP32, results not bit-equal
                                   to it.  dense_gemm_act, gcn_layer_fwd (with d_T given, or through a
                                   workspace whose sweep ends with the dense transform) and both
                                   gradients of gcn_layer_bwd run it; the row-range one-kernel layer
                                   (gcn_layer_fwd_fused, gcn_layer_fwd without d_T and without such a
                                   workspace) returns SAGNN_EINVAL */

/* Text for an error code (static string). */
const char* sagnn_strerror(int code);
/* hipError_t of the most recent failing HIP call made by this library (0 if none). */
int sagnn_last_hip_error(void);
/* Library version: major*10000 + minor*100 + patch. */
int sagnn_version(void);

/* ---------------------------------------------------------------------------------------
 * Step 1: needed rows (NnzCols; Sec. 4.1).
 *
 * For the row block given as CSR (m rows, n columns) and nb contiguous column blocks
 * [h_colblk[q], h_colblk[q+1]) with h_colblk[0] = 0 and h_colblk[nb] = n (ascending),
 * computes
 *   d_needed[0..N)        global column ids that hold at least one stored entry, ascending;
 *                         block q owns positions [h_blk_off[q], h_blk_off[q+1]); this is the
 *                         order in which Alg. 1 concatenates the packed rows
 *   h_blk_off[0..nb]      host output, h_blk_off[nb] = N
 *   d_colidx_compact[nnz] for every entry e the position p with d_needed[p] == d_colidx[e]
 *                         (column index into the packed buffer); may be NULL to skip.
 *                         An entry whose column is outside [0,n) gets -1.
 * All integer work; the result is unique, so it is bit-exact by construction.
 *
 * Synchronises the stream once (N has to reach the host).  If N > needed_cap returns
 * SAGNN_ECAPACITY with h_blk_off filled in (so the caller knows the size to allocate) and
 * d_needed / d_colidx_compact untouched.  With SAGNN_PLAN_VALIDATE the CSR is checked on
 * the device first (rowptr monotone from 0 to nnz, every column in [0,n)) and
 * SAGNN_EFORMAT is returned on failure.
 *
 * With SAGNN_PLAN_OBLIVIOUS the sparsity of the block is ignored, as in the
 * sparsity-oblivious algorithm the paper compares against (Sec. 4.1: every process transfers
 * its whole block row of H): every column of [0,n) is "needed", so d_needed = 0..n-1,
 * h_blk_off = h_colblk and d_colidx_compact = d_colidx.  Same kernels downstream; it exists so
 * that both algorithms can be measured on one harness.
 *
 * Small blocks (n <= 262,144 columns, m <= 262,144 rows, nnz <= 65,536, nb <= 16, not oblivious) are
 * planned by one workgroup in one launch with one copy back (the launch-latency regime: the general
 * path is ten launches and three copies); SAGNN_PLAN_MULTIPASS switches that off.  Results are the
 * same either way.
 *
 * Workspace: spmm_plan_workspace_bytes(); contents are scratch.  Its size is a few bytes per
 * column plus, for wide blocks with many entries (n above about 5 M columns and nnz >= 2^22),
 * 8*nnz bytes for the entries sorted into column ranges and the place every entry went to.
 */
int spmm_plan_workspace_bytes(int64_t m, int64_t n, int64_t nnz, int32_t nb, size_t* bytes);
int spmm_plan_needed_rows(const int32_t* d_rowptr, const int32_t* d_colidx, int64_t m,
                          int64_t n, int64_t nnz, const int64_t* h_colblk, int32_t nb,
                          int32_t* d_needed, int64_t needed_cap, int64_t* h_blk_off,
                          int32_t* d_colidx_compact, void* d_ws, size_t ws_bytes,
                          uint32_t flags, void* stream);

/* spmm_plan_needed_rows() for callers that cannot allocate device memory (tight serving loops,
 * harnesses that forbid hipMalloc, code that runs beside a graph capture): same arguments without
 * the workspace, same outputs bit for bit.  The scratch arrays live in a fixed 8 MiB array of
 * device memory that each GPU the library runs on holds until the process ends; the call
 * allocates nothing on the device or through any allocating library routine.
 * Limits: n <= SAGNN_PLAN_NOALLOC_MAX_COLS and nb <= SAGNN_PLAN_NOALLOC_MAX_BLOCKS, otherwise
 * SAGNN_ECAPACITY (nothing is launched).  All calls on one GPU share that GPU's array: the
 * call clears what it needs cleared itself, and two such calls that overlap in time on one
 * GPU (different streams or threads) race -- serialise them.  Like spmm_plan_needed_rows() it
 * synchronises the stream once to return N.
 */
#define SAGNN_PLAN_NOALLOC_MAX_COLS 5000000
#define SAGNN_PLAN_NOALLOC_MAX_BLOCKS 1024
int spmm_plan_needed_rows_noalloc(const int32_t* d_rowptr, const int32_t* d_colidx, int64_t m,
                                  int64_t n, int64_t nnz, const int64_t* h_colblk, int32_t nb,
                                  int32_t* d_needed, int64_t needed_cap, int64_t* h_blk_off,
                                  int32_t* d_colidx_compact, uint32_t flags, void* stream);

/* ---------------------------------------------------------------------------------------
 * Streams and graphs.  Every entry point enqueues its work on the stream it is given.  The
 * set-up calls (spmm_plan_needed_rows, spmm_csr_prepare, spmm_csr_prepare_tuned, spmm_split_colblocks,
 * spmm_csr_transpose) copy small results back and synchronise that stream, so they cannot be
 * recorded into a graph.  The per-step calls (spmm_pack_rows, spmm_csr_tallskinny,
 * dense_gemm_act, gcn_layer_fwd, gcn_layer_bwd, spmm_stage_loop) only launch kernels and, in the
 * stage loop, record and wait for events between its two streams (forked from and joined back
 * into the product stream): no host synchronisation, no memset, no allocation.  They may be
 * captured into a HIP graph and replayed; a replay gives the same bits as the eager calls.
 */

/* ---------------------------------------------------------------------------------------
 * Step 2: pack / gather (Alg. 1 first statement; Alg. 2 "H[srows,:]").
 *
 *   d_out[r, 0:f) = d_H[d_rows[r], 0:f)   for r in [0,N)
 *
 * d_H is n x f (leading dimension ldh), d_out is N x f (leading dimension ldo).  A row id
 * outside [0,n) produces a row of zeros.  Pure copy: bit-exact.  Element offsets are 64-bit
 * (n*ldh may exceed 2^32).
 */
int spmm_pack_rows(const float* d_H, int64_t n, int64_t ldh, int32_t f, const int32_t* d_rows,
                   int64_t N, float* d_out, int64_t ldo, void* stream);

/* ---------------------------------------------------------------------------------------
 * Step 3: local SpMM (Alg. 1/2 "Z <- Z + SpMM(A_iq, H^)").
 *
 *   C[r, 0:f) (+)= sum_e val[e] * B[colidx[e], 0:f)   over the stored entries of row r
 *
 * A is m x k CSR, B is k x f (ldb), C is m x f (ldc); accumulate = 0 overwrites C,
 * accumulate = 1 adds to it (the per-block accumulation of the algorithms).  fp32 FMA.
 * The summation order is a fixed function of (rowptr, colidx, m, k, nnz, f), so results are
 * reproducible run to run and across preparations (no floating-point atomics); it differs
 * from the stored order, so they agree with a sequential sum up to rounding.  No serial run of
 * additions is longer than 256 terms (partial sums are folded in a second level), which keeps
 * |err| <= 1e-5 * sum |val||B| even for rows whose products are all equal; ~1e-7 is typical.
 * A column index outside [0,k) is clamped into range (never read out of bounds).
 *
 * Scheduling: the pattern (and here also the values) of A is fixed during training, so a
 * one-time spmm_csr_prepare() builds a schedule in the workspace:
 *   - always: the entries are cut into equal chunks (nonzero splitting) and the row in which
 *     each chunk starts is recorded, so hub rows and runs of short rows are balanced;
 *   - for large power-law matrices with f a multiple of 64 (or exactly 32 or 16): the entries
 *     of long rows are copied
 *     into the workspace re-ordered by column slab ("slab sweep"), so that all wavefronts of an
 *     XCD touch the same small part of B at the same time (L2 reuse).  Requires ascending
 *     column indices inside long rows and k < 2^27; otherwise the first schedule is used.
 *     At f = 128 and f = 64 the re-ordered copy is laid out for kernels that fetch two / four
 *     rows of B per load instruction, which a later call must match: a workspace prepared for
 *     f = 128 serves calls with f = 128 or 64, one prepared for f = 64 only f = 64.
 *     The short rows are swept as well, as whole rows in wavefronts of their own, where the
 *     matrix allows it (short_rows of sagnn_spmm_options); otherwise they go through the first
 *     schedule on a compacted copy.
 * The workspace then holds a private copy of colidx/val: call spmm_csr_prepare() again if
 * they change.  d_ws must be passed unchanged to every spmm_csr_tallskinny() call with the
 * same (rowptr, colidx, val, m, k, nnz) and f <= the prepared f (a multiple of 64 if the
 * slab-sweep schedule was chosen, see spmm_csr_schedule_info; exactly the prepared f if that
 * was 32 or 16); part of it is scratch for
 * partial row sums, so two calls that share a workspace must not overlap in time.
 * spmm_csr_prepare() plans on the device (row classification, cutting of long rows, dealing of
 * the pieces to wavefronts, layout of the re-ordered copy); the host reads a few totals and
 * flags back, which synchronises the stream three or four times.  The library remembers a small host descriptor per prepared workspace address; passing a
 * workspace that was not prepared in this process returns SAGNN_EINVAL.  If the workspace
 * memory was overwritten after preparation, C is unspecified (the kernels check a generation
 * tag and exit), but nothing faults.
 * With d_ws == NULL a simple one-wavefront-per-row kernel is used (no preparation).
 * The planner's choices can be overridden through spmm_csr_prepare_opt() (the library reads no
 * environment variables); every setting gives the same product up to rounding.
 * B and C must not overlap.
 */
/* Planner options of the slab-sweep schedule.  A zeroed struct (or NULL) means "let the library
 * decide"; the fields exist for experiments and for tests that force a particular code path on
 * small inputs.  Every combination gives the same product up to rounding order. */
typedef struct sagnn_spmm_options {
  int32_t schedule;        /* 0 heuristic, 1 nonzero splitting only, 2 slab sweep whenever possible */
  int32_t min_long;        /* rows with at least this many entries are swept (0 = decide; >= 16;
                              negative: -min_long replaces 64 where the rule would pick 64)         */
  int32_t piece;           /* longest piece a swept row is cut into (0 = 4096; 1024..32768)         */
  int32_t slab_kb;         /* KiB of B per slab (0 = 4096); -1 = as many slabs as the format allows  */
  int32_t min_waves;       /* fewer than 16 pieces per wavefront below this many wavefronts (0 = 8192) */
  int32_t window_pct;      /* dealing window in % of the resident pieces (0 = 400); -1 = one window  */
  int32_t snake;           /* 1: deal pieces in snake order instead of longest-first (one stream per wavefront) */
  int32_t groups;          /* lane groups: 0 decide, 1 never, 2 whenever the width has them         */
  int32_t sync_slabs;      /* slabs per interval of the sweep (0 = decide, -1 = one interval).  At
                              interval boundaries the wavefronts are kept in step, by pacing or
                              by barriers (next two fields); without either the layout is inert  */
  int32_t pace_ps_per_step;/* pacing: a wavefront does not start interval i before its own start
                              time + this many picoseconds x the average number of stream steps
                              up to i, so that all wavefronts pass the slabs at one pace and an
                              XCD's L2 has to hold one part of B at a time.  0 or -1 = none;
                              -2 = spmm_csr_prepare_tuned searches the pace after choosing the plan
                              variant (about seventy more products) and keeps it only if it is
                              more than 1.5 % faster                                               */
  int32_t barriers;        /* 1: instead of pacing, the workgroups of an XCD that run together
                              wait for each other at every interval boundary (bounded wait).
                              Kept for experiments: it moves less data than pacing and is slower */
  int32_t sync_timeout_us; /* longest wait at such a barrier before all barriers of the launch are
                              given up (0 = 200)                                                    */
  int32_t sync_test_extra; /* test hook: added to the number of arrivals a barrier waits for, so
                              that every wait runs into the time limit and the give-up path runs   */
  int32_t narrow_slots;    /* 1: at width 128 a wavefront owns 14 (15 without lane groups) pieces
                              instead of 16, which lets a CU hold five workgroups instead of four
                              (16 rows need 32768 bytes of LDS per workgroup and 5 x 32768 do not
                              fit).  Measured slower on the free-running sweep (more wavefronts
                              thrash the L2 more) and equal under pacing; off unless asked for     */
  int32_t slab_width;      /* widest column slab of B one launch covers: 0 = 256; 128 = operands wider
                              than 128 are processed as 128-wide slabs by the kernels that fetch two
                              rows of B per load (faster on the 2.45 M-vertex power-law graph at
                              f = 256, slower on the community-ordered one; the measured choice of
                              spmm_csr_prepare_tuned tries it)                                       */
  int32_t short_rows;      /* the rows below the long-row threshold are swept too -- as whole rows, 16
                              per wavefront in order of their length, behind the wavefronts of the long
                              rows, every row one segment of its wavefront's stream -- instead of going
                              through the nonzero-splitting kernel on a compacted CSR.  Every row then
                              ends in a wavefront of the sweep, so gcn_layer_fwd with d_T = NULL can
                              take its sweep-epilogue form on graphs with many short rows.  Possible
                              with widths of 64 and up, 16 accumulator rows, no slab intervals and
                              short rows of at most 255 entries.
                              0 or 1 = where possible, -1 = never                                     */
  int32_t dense_tiles;     /* 1: the tiles of A that are dense enough to re-use staged rows of the dense
                              operand are taken out of the matrix and multiplied by a kernel that keeps
                              those rows in LDS (see "dense tiles" below); needs a workspace sized by
                              spmm_csr_workspace_bytes_opt with the same setting and f = 64, 128 or 256
                              (other widths: ignored).  0 or -1 = no.  Measured slower than the slab
                              sweep on the power-law graphs it was built for (see below); kept as an
                              option                                                                  */
  int32_t tile_reuse_x10;  /* a tile is kept when it holds at least this many entries per column, in
                              tenths (0 = 25, i.e. every staged row is used 2.5 times on average)     */
} sagnn_spmm_options;
int spmm_csr_workspace_bytes(int64_t m, int64_t nnz, int32_t f, size_t* bytes);
/* Workspace size for a preparation with the given options: spmm_csr_workspace_bytes() plus, with
 * dense_tiles = 1, the tile region.  h_opt may be NULL.
 *
 * Dense tiles (high-degree graphs such as the 233 k-vertex one with ~490 entries per row): rows of A
 * are ranked by their number of entries, columns by the number of entries that reference them; the
 * first 131,072 rows and 65,536 columns form tiles of 512 rows x (16384 / f) columns (256 rows at
 * f = 256).  A tile with at least tile_reuse_x10 / 10 entries per column is multiplied by a kernel
 * that stages the tile's rows of the dense operand (64 KB) in LDS, double-buffered, while the 16
 * wavefronts of a workgroup keep the sums of the tile's rows in registers; the sums of a row group's
 * work items are added to C in a fixed order by a second kernel (reproducible, no floating-point
 * atomics).  All other entries stay in a rest CSR (stored in the tile region, rows still ascending)
 * that is prepared and multiplied like any other matrix.  If no tile qualifies the preparation is
 * the plain one.  The tile region holds the rest CSR, the tile entry streams and the partial sums:
 * about 28 bytes per entry of A.  gcn_layer_fwd with d_T = NULL uses its row-range form on such a
 * workspace (rows with entries in tiles are not finished by one wavefront). */
int spmm_csr_workspace_bytes_opt(int64_t m, int64_t k, int64_t nnz, int32_t f,
                                 const sagnn_spmm_options* h_opt, size_t* bytes);
/* What a preparation with dense_tiles = 1 decided (host query).  h_info[6]: [0] 1 if tiles are in
 * use, [1] entries in kept tiles, [2] kept tiles, [3] work items, [4] ranked rows, [5] entries of
 * the rest CSR.  SAGNN_EINVAL if the workspace is unknown. */
int spmm_csr_tile_info(const void* d_ws, int64_t* h_info);
int spmm_csr_prepare(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                     int64_t m, int64_t k, int64_t nnz, int32_t f, void* d_ws, size_t ws_bytes,
                     void* stream);
int spmm_csr_prepare_opt(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                         int64_t m, int64_t k, int64_t nnz, int32_t f, void* d_ws, size_t ws_bytes,
                         const sagnn_spmm_options* h_opt, void* stream);
/* spmm_csr_prepare() with a measured choice between a few variants of the slab-sweep plan (how
 * long rows are cut into pieces, from which length a row counts as long): each variant is
 * prepared into d_ws and the product is run six times on the caller's operand d_B (k x f,
 * ldb), writing d_C (m x f, ldc; overwritten, holds a valid product afterwards); the fastest
 * variant is left in d_ws.  Which wavefronts share a part of B in cache at a time depends on
 * such details and moves the time of the product by a few per cent either way, differently for
 * every matrix and width; the pattern is fixed for a training run, so measuring once pays.
 * A variant replaces the default plan only if it is more than 1.5 % faster.  Costs about five
 * preparations and thirty products; synchronises the stream.  When the plain
 * schedule is chosen there is nothing to vary and the call equals spmm_csr_prepare().  Every
 * variant computes the same product up to rounding order.
 * For operands wider than 128 two more variants take B as 128-wide column slabs (indices 5 and 6;
 * slab_width of sagnn_spmm_options).
 * h_choice (host, 4 values, may be NULL): piece length and long-row threshold of the variant
 * kept (0 = default), its best time in microseconds, its index.  h_opt (may be NULL): options
 * every variant starts from (see sagnn_spmm_options below).
 */
int spmm_csr_prepare_tuned(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                           int64_t m, int64_t k, int64_t nnz, int32_t f, void* d_ws,
                           size_t ws_bytes, const float* d_B, int64_t ldb, float* d_C,
                           int64_t ldc, int32_t* h_choice, const sagnn_spmm_options* h_opt,
                           void* stream);
/* What spmm_csr_prepare() decided for a workspace (host query, no GPU work).  h_info[16]:
 * [0] schedule (0 nonzero splitting, 1 slab sweep, with nonzero splitting for the short rows
 *     unless they are swept too: then [3] = [4] = [5] = 0),
 * [1] wavefront streams of the sweep, [2] entries in them, [3] rows, [4] entries and
 * [5] chunks of the nonzero-splitting part, [6] rows cut into several pieces,
 * [7] 1 if the matrix has empty rows, [8] barrier intervals of the sweep, [9] slabs per
 * interval (0 = one interval), [10] byte offset inside the workspace of a 32-bit flag that the
 * most recent product left at 1 if a barrier wait ran into its time limit (the product is
 * correct either way), [11] lane groups per wavefront, [12] pacing in picoseconds per stream
 * step (0 = none), [13] 1 if barriers are used, [14] accumulator rows per wavefront,
 * [15] steps (entries per lane group, padding included) of the longest wavefront stream; the
 * average is [2] / ([1] * [11]).
 * SAGNN_EINVAL if the workspace is unknown. */
int spmm_csr_schedule_info(const void* d_ws, int64_t* h_info);
/* Forget the host descriptor of a prepared workspace.  Call it before the workspace memory is
 * freed or reused for something else: afterwards the address is unknown to the library again
 * (spmm_csr_tallskinny with it returns SAGNN_EINVAL until it is prepared anew), and nothing of
 * the preparation stays behind in the process.  Unknown addresses are accepted (no-op). */
int spmm_csr_release(const void* d_ws);
int spmm_csr_tallskinny(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                        int64_t m, int64_t k, int64_t nnz, const float* d_B, int64_t ldb,
                        int32_t f, float* d_C, int64_t ldc, int32_t accumulate, void* d_ws,
                        size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Dense transform on the matrix cores:  Z = op(X) * op(W), optional epilogue.
 *
 *   transW = 0: W is kdim x nout (ldw);  transW = 1: W is nout x kdim (ldw), used as W^T
 *   X is m x kdim (ldx), Z is m x nout (ldz)
 *   prec: SAGNN_GEMM_FP32, SAGNN_GEMM_BF16 or SAGNN_GEMM_FP32_BF16X3
 *   d_Z   (may be NULL) receives the product
 *   d_act (may be NULL) receives ReLU(product) when act = SAGNN_ACT_RELU, else the product
 *   d_mask (may be NULL, m x nout, ldmask): the product is zeroed where d_mask <= 0
 *         (the ".* sigma'(Z)" factor of the backward equation) before it is stored
 * kdim and nout: multiples of 4, at most 256 (W stays resident in LDS; the matrix-core tiles
 * are zero-padded to multiples of 32).
 */
int dense_gemm_act(const float* d_X, int64_t ldx, const float* d_W, int64_t ldw, int32_t transW,
                   int64_t m, int32_t kdim, int32_t nout, int32_t prec, int32_t act,
                   const float* d_mask, int64_t ldmask, float* d_Z, int64_t ldz, float* d_act,
                   int64_t ldact, void* stream);

/* ---------------------------------------------------------------------------------------
 * Step 4: one GCN layer forward (Sec. 2.1 forward equations in the order of Alg. 1):
 *
 *   T = A * H            (m x f_in; kept because the backward pass needs it)
 *   Z = T * W            (m x f_out, W is f_in x f_out row-major, ld = f_out)
 *   Hout = sigma(Z)      sigma = ReLU or identity
 *
 * A, H as in spmm_csr_tallskinny (H is k x f_in, ldh).  d_Z or d_Hout may be NULL (not
 * stored).  d_T, d_Z, d_Hout are dense with ld = f_in / f_out / f_out.
 * d_ws: SpMM workspace prepared for (rowptr, m, nnz, f_in), or NULL.
 *
 * Two forms.  With d_T != NULL the layer is the sparse product (spmm_csr_tallskinny with its
 * prepared schedule) followed by the dense transform, two kernels with T in HBM between them.
 * With d_T == NULL (inference, or a backward pass that recomputes T) the layer runs as ONE
 * kernel, gcn_layer_fwd_fused below: a workgroup computes whole rows of T for a tile of rows,
 * keeps the tile in LDS beside W and multiplies it on the matrix cores, so T never reaches
 * HBM (2 m f_in 4 bytes less traffic) and d_ws is not used.  The fused form exists for
 * f_in in {64, 128, 256}, f_out <= 256 with W and one tile fitting the LDS (fp32: f_in * f_out
 * <= 128 * 256; bfloat16: up to 256 x 256); other shapes return SAGNN_EINVAL when d_T is NULL.
 * It balances work per tile of rows, not per entry: on matrices with rows of similar length it
 * is the cheaper form, on power-law matrices the two-kernel form with the slab-sweep schedule
 * is faster (rows longer than 512 entries are shared by a workgroup's wavefronts, so they
 * are correct but slow).  Same rounding bound as the two-kernel form.
 * With d_T == NULL and a workspace that was prepared for the slab sweep (spmm_csr_schedule_info:
 * schedule 1; f_in 64, 128 or 256 covered by one launch of the prepared kernels: 256 needs lane
 * groups 1, 128 lane groups 1 or 2, 64 any) whose wavefronts finish all but at most 65536 rows
 * (rows outside the sweep and rows cut into several pieces are the exceptions; a partitioned
 * graph's blocks have none, a power-law graph whose short rows are swept as whole rows --
 * short_rows of sagnn_spmm_options, the default where possible -- a few thousand), the sweep kernel
 * itself ends with the dense transform: a workgroup's 64 finished rows of A H are multiplied by
 * W on the matrix cores straight out of LDS, the few other rows go through a small kernel.
 * gcn_layer_fwd_form() tells which form a call would take.
 * gcn_layer_fwd_fused may also be called directly, with d_T non-NULL to get T as a by-product.
 */
int gcn_layer_fwd(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                  int64_t m, int64_t k, int64_t nnz, const float* d_H, int64_t ldh,
                  int32_t f_in, const float* d_W, int32_t f_out, int32_t act,
                  int32_t gemm_prec, float* d_T, float* d_Z, float* d_Hout, void* d_ws,
                  size_t ws_bytes, void* stream);
/* Host query: *h_form = 2 if gcn_layer_fwd(d_T = NULL) with this prepared workspace (may be NULL)
 * and these widths runs as the slab sweep with the dense transform as its epilogue, 1 if it
 * runs as the row-range kernel, 0 if neither supports the shape or the operand mode. */
int gcn_layer_fwd_form(const void* d_ws, int32_t f_in, int32_t f_out, int32_t gemm_prec, int32_t* h_form);
int gcn_layer_fwd_fused(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                        int64_t m, int64_t k, int64_t nnz, const float* d_H, int64_t ldh,
                        int32_t f_in, const float* d_W, int32_t f_out, int32_t act,
                        int32_t gemm_prec, float* d_T, float* d_Z, float* d_Hout, void* stream);

/* ---------------------------------------------------------------------------------------
 * Step 5: one GCN layer backward (Sec. 2.1 backward equations; Sec. 4.1 paragraphs on the
 * two gradient equations).  For the layer whose forward was Z = (A Hprev) W and incoming
 * gradient G = dLoss/dZ (m x f_out):
 *
 *   S     = A_bwd * G                        (m x f_out)  the CSR passed here is the
 *                                             orientation the backward equation multiplies
 *                                             by; for a symmetric graph it is the same CSR
 *   Gprev = (S * W^T) .* [Zprev > 0]          (m x f_in)   skipped if d_Gprev == NULL;
 *                                             mask skipped if d_Zprev == NULL.  Any array
 *                                             that is positive exactly where Z^{l-1} is
 *                                             (e.g. ReLU(Z^{l-1})) serves as d_Zprev
 *   Y     = Hprev^T * S                       (f_in x f_out, fp32) skipped if d_Y == NULL
 *
 * The cross-process sum of Y is not part of this library.  d_ws: SpMM workspace prepared for
 * (rowptr, m, nnz, f_out) or NULL.  d_yws: scratch of gcn_bwd_workspace_bytes() bytes for
 * the partial sums of Y (required if d_Y != NULL).
 */
int gcn_bwd_workspace_bytes(int64_t m, int32_t f_in, int32_t f_out, size_t* bytes);
int gcn_layer_bwd(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                  int64_t m, int64_t nnz, const float* d_G, int32_t f_out, const float* d_W,
                  int32_t f_in, const float* d_Zprev, const float* d_Hprev, int32_t gemm_prec,
                  float* d_S, float* d_Gprev, float* d_Y, void* d_ws, size_t ws_bytes,
                  void* d_yws, size_t yws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Column-block split (Sec. 4.2 column-block partition of a row block; Alg. 2 multiplies one
 * block A_iq per stage).
 *
 * Splits the CSR row block (m rows) into nb CSR matrices, one per contiguous range
 * [h_bounds[q], h_bounds[q+1]) of the index space d_colidx lives in: global column ids with
 * the h_colblk of the plan, or packed positions with its h_blk_off (then block q's column ids
 * index that block's part of the packed buffer).  h_bounds is ascending, nb <= 256.
 *   d_rowptr_blk  nb*(m+1) int32: block q's row pointer is d_rowptr_blk + q*(m+1), starts at 0
 *   d_colidx_blk, d_val_blk   nnz entries each: block q's entries are
 *                 [h_nnz_off[q], h_nnz_off[q+1]), column ids relative to h_bounds[q]; inside a
 *                 row the stored order is kept (stable), so a block product sums in the same
 *                 order as the unsplit product restricted to that block
 *   h_nnz_off     nb+1 int64, host output
 * Entries whose column is outside [h_bounds[0], h_bounds[nb]) are dropped.  Integer work with
 * a unique result: bit-exact.  Synchronises the stream once.  d_ws: scratch of
 * spmm_split_workspace_bytes() bytes.
 */
int spmm_split_workspace_bytes(int64_t m, int32_t nb, size_t* bytes);
int spmm_split_colblocks(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                         int64_t m, int64_t nnz, const int64_t* h_bounds, int32_t nb,
                         int32_t* d_rowptr_blk, int32_t* d_colidx_blk, float* d_val_blk,
                         int64_t* h_nnz_off, void* d_ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * CSR transpose (Sec. 2.1 / Sec. 4.1: the forward pass multiplies by A^T, the backward pass by
 * A; for a directed graph the two differ, and a process needs both orientations of its block).
 *
 * Writes A^T (n rows, m columns, nnz entries) as CSR: d_rowptr_t[n+1], d_colidx_t[nnz] (row
 * ids of A), d_val_t[nnz].  The entries of a transposed row are in ascending order of the
 * row of A they came from, entries of one row of A that repeat a column keep their stored
 * order (stable), so the result is unique: bit-exact.  Returns SAGNN_EFORMAT if a column index
 * is outside [0,n) (outputs are then unspecified, nothing faults).  One-time set-up step;
 * synchronises the stream once.  d_ws: scratch of spmm_transpose_workspace_bytes() bytes
 * (about 16 bytes per stored entry).
 */
int spmm_transpose_workspace_bytes(int64_t nnz, size_t* bytes);
int spmm_csr_transpose(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                       int64_t m, int64_t n, int64_t nnz, int32_t* d_rowptr_t,
                       int32_t* d_colidx_t, float* d_val_t, void* d_ws, size_t ws_bytes,
                       void* stream);

/* ---------------------------------------------------------------------------------------
 * Locality reordering (Sec. 5 and Sec. 6.1: the graph is partitioned, the vertices are renumbered
 * so that every part owns a contiguous range, A is permuted symmetrically and the rows of the
 * dense matrices follow; Sec. 5 argues that this is what makes NnzCols small).
 *
 * spmm_perm_from_labels: d_labels[v] in [0, n_parts) is the part of vertex v.  Writes
 *   d_perm[i] = old id of the vertex that gets new id i (vertices ordered by label, inside a
 *               part by old id: a stable sort, so the result is unique)
 *   d_inv[v]  = new id of old vertex v
 *   h_part_off[0..n_parts] (host): part q owns new ids [h_part_off[q], h_part_off[q+1])
 * n_parts <= 1024.  SAGNN_EFORMAT if a label is out of range.
 *
 * spmm_csr_permute_symmetric: B = P A P^T for the square CSR matrix A (n x n):
 *   B[d_inv[r], d_inv[c]] = A[r, c].  Rows of B come out with ascending column ids (entries
 *   that repeat a position keep their stored order), so B is unique: bit-exact.
 *   SAGNN_EFORMAT if d_inv is not a permutation of [0, n) or a column index is out of range.
 *
 * The dense side needs no call of its own: H_new = H[d_perm, :] is spmm_pack_rows(H, d_perm)
 * and Z_old = Z_new[d_inv, :] is spmm_pack_rows(Z_new, d_inv).
 * One-time set-up steps; both synchronise the stream.  d_ws: scratch of
 * spmm_permute_workspace_bytes(n, nnz) bytes (serves both calls).
 */
int spmm_permute_workspace_bytes(int64_t n, int64_t nnz, size_t* bytes);
int spmm_perm_from_labels(const int32_t* d_labels, int64_t n, int32_t n_parts, int32_t* d_perm,
                          int32_t* d_inv, int64_t* h_part_off, void* d_ws, size_t ws_bytes,
                          void* stream);
int spmm_csr_permute_symmetric(const int32_t* d_rowptr, const int32_t* d_colidx, const float* d_val,
                               int64_t n, int64_t nnz, const int32_t* d_inv, int32_t* d_rowptr_p,
                               int32_t* d_colidx_p, float* d_val_p, void* d_ws, size_t ws_bytes,
                               void* stream);

/* ---------------------------------------------------------------------------------------
 * Stage loop of one rank of the 1.5D algorithm (Alg. 2, the loop over k = 0..s-1 with
 * q = j*s + k: obtain the rows NnzCols(i,q) of H, then Z^ <- Z^ + SpMM(A_iq, H^)).
 *
 * The receive of Alg. 2 is replaced by a pack out of the device-resident d_H (n x f, ldh):
 * the exchange itself is not part of this library.  For stage k
 *   T_k = d_H[stage.d_rows[0..N), :]                    on stream_pack
 *   d_Z (+)= A_k * T_k                                  on stream_spmm
 * with two packed buffers d_T0 / d_T1 (each t_cap_rows x f, ld = f) used alternately, so the
 * pack of stage k+1 overlaps the product of stage k when the two streams differ (they may be
 * the same stream: then the stages run back to back).  accumulate_first = 0 makes the first
 * stage overwrite d_Z (m x f, ldz), 1 adds to its current contents; later stages always add.
 * The all-reduce over the replicas that follows in Alg. 2 is outside this library.
 * Ordering: work already queued on stream_spmm is waited for by stream_pack; on return all
 * of the loop's work is ordered before later work on stream_spmm.  Returns SAGNN_ECAPACITY if
 * some stage has N > t_cap_rows.
 */
typedef struct sagnn_stage {
  const int32_t* d_rowptr; /* A_iq as CSR, m+1 entries                                      */
  const int32_t* d_colidx; /* column ids = positions in this stage's packed buffer, [0,N)   */
  const float* d_val;
  int64_t nnz;
  const int32_t* d_rows;   /* NnzCols(i,q): N global row ids of d_H, in packed order        */
  int64_t N;
  void* d_ws;              /* SpMM workspace prepared for this block, or NULL               */
  size_t ws_bytes;
} sagnn_stage;
int spmm_stage_loop(const sagnn_stage* h_stages, int32_t n_stages, int64_t m, const float* d_H,
                    int64_t n, int64_t ldh, int32_t f, float* d_T0, float* d_T1,
                    int64_t t_cap_rows, float* d_Z, int64_t ldz, int32_t accumulate_first,
                    void* stream_spmm, void* stream_pack);

/* ---------------------------------------------------------------------------------------
 * Communication-volume statistics of one SpMM (Sec. 4.1 cost paragraph: cut_P(G), the largest
 * |NnzCols(i,j)| over i != j; Sec. 5, Table 2: average and maximum data per process and the
 * load imbalance, which for every row of that table equals (max / average - 1) * 100).
 *
 * h_counts is P x P row-major, h_counts[i*P + q] = |NnzCols(i,q)| = rows of H_q that P(i)
 * needs (diff of the plan's h_blk_off for row block i); the diagonal is ignored (local rows).
 * Host arithmetic only.  h_out[8]:
 *   0 total bytes moved        = sum_{i != q} counts * f * elem_bytes
 *   1 average bytes per process (total / P)
 *   2 maximum bytes received by one process   3 its imbalance % = (max / avg - 1) * 100
 *   4 maximum bytes sent by one process       5 its imbalance %
 *   6 cut_P (rows)                            7 cut_P * f * elem_bytes
 * Imbalances are 0 when nothing is moved.
 */
int spmm_volume_stats(const int64_t* h_counts, int32_t P, int32_t f, int32_t elem_bytes,
                      double* h_out);

#ifdef __cplusplus
}
#endif
#endif /* SAGNN_H */
