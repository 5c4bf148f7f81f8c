/*
 * pivot_fc.h - C ABI of the pruned fully-connected inference library for
 * AMD MI355X (gfx950).
 *
 * A pruned FC layer is kept in permutation-block-permutation (PBP) form,
 *     M_sparse = P_row * M_block * P_col                       (paper Eq. 1)
 * and applied as
 *     a_out = P_row (M_block (P_col a_in))                     (paper Eq. 2)
 * plus a bias and a point-wise activation:
 *     y = act(P_r^T * BSR(W') * (P_c x) + b).
 *
 * Conventions used by every entry point
 * -------------------------------------
 *  - A permutation is an index array that acts as a gather,
 *    out[i] = in[idx[i]] (Section 4.1.4: the index array of "cab" relative to
 *    "abc" is [2,0,1]).  With W' the pivoted (block-space) matrix:
 *        W'[r][c] = W[prow[r]][pcol[c]],   xg[c] = x[pcol[c]],   y[prow[r]] = v[r]
 *    (Listing 1 gathers the input through P_col and scatters the output
 *    through P_row).
 *  - The tile mask lives in block space: tile (i,j) covers block-space rows
 *    [i*bh,(i+1)*bh) and columns [j*bw,(j+1)*bw).  nbr = ceil(M/bh),
 *    nbc = ceil(K/bw); rows >= M and columns >= K of the last tiles are zero
 *    padding and are never gathered or scattered (Section 4.1.5 allows
 *    irregular shapes; padding is the form used here).
 *  - Several kept tiles may share a block row; their partial results are
 *    summed in a fixed order (Section 4.1.5), so repeated runs give identical
 *    bits.
 *  - "host" pointers are ordinary CPU memory, borrowed for the duration of the
 *    call.  "device" pointers are HIP device memory on the plan's device,
 *    borrowed until the work enqueued on `stream` has finished.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Run calls are asynchronous: they enqueue kernels, never allocate, never
 *    synchronise.
 *  - Every function returns PIVOT_OK (0) or a negative PIVOT_E_* code and
 *    never throws or aborts; pivot_last_error() gives a thread-local text.
 */
#ifndef PIVOT_FC_H
#define PIVOT_FC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIVOT_VERSION 100

#define PIVOT_OK                  0
#define PIVOT_E_NULL             -1   /* a required pointer is NULL */
#define PIVOT_E_SHAPE            -2   /* sizes are not positive / do not match */
#define PIVOT_E_NOT_PERMUTATION  -3   /* prow or pcol is not a bijection of its range */
#define PIVOT_E_UNSUPPORTED      -4   /* tile shape / dtype / layout / batch not supported on the device path */
#define PIVOT_E_ALLOC            -5   /* host or device allocation failed */
#define PIVOT_E_HIP              -6   /* a HIP call failed */
#define PIVOT_E_WORKSPACE        -7   /* workspace missing or too small */
#define PIVOT_E_NO_DEVICE        -8   /* a host-only plan was given to a run call */

/* weight storage type; x has the same type, accumulation is fp32 */
#define PIVOT_F32 0
#define PIVOT_F16 1

/* physical layout of the kept tiles (Section 4.1.1), rightmost axis fastest */
#define PIVOT_BRC 0   /* block, row, column : row-major inside a tile    */
#define PIVOT_BCR 1   /* block, column, row : column-major inside a tile */
#define PIVOT_CBR 2   /* column, block, row : one column position of all tiles together */

#define PIVOT_ACT_NONE 0
#define PIVOT_ACT_RELU 1

/* coordinate space of the weight matrix handed to pivot_fc_plan */
#define PIVOT_W_NATURAL 0   /* W[M][K] as trained; entries outside kept tiles are ignored */
#define PIVOT_W_PIVOTED 1   /* W'[M][K] already in block space */

typedef struct pivot_fc_desc {
    int32_t M;            /* outputs (rows of the weight matrix)                         */
    int32_t K;            /* inputs  (columns)                                           */
    int32_t bh;           /* tile rows                                                   */
    int32_t bw;           /* tile columns                                                */
    int32_t wdtype;       /* PIVOT_F32 or PIVOT_F16                                      */
    int32_t layout;       /* PIVOT_BRC / BCR / CBR                                       */
    int32_t act;          /* PIVOT_ACT_*                                                 */
    int32_t chunk_tiles;  /* max tiles per work item; 0 = the library chooses: whole block rows
                           * unless LDS forces a cut, a work item would stream 256 KB or more while
                           * compute units idle, or the longest block row has at least four times
                           * the average number of tiles (then pieces of twice the average row,
                           * 32..96 KB per work item)                                     */
    int32_t device;       /* HIP device ordinal, or -1 for a host-only plan (no GPU use) */
    int32_t wg_waves;     /* wavefronts per work item: 1 (batch 1 only; 4 at other batches), 4, 8 or 16; 0 = the library chooses */
    int32_t row_slices;   /* independent work items per tile height: 1, 2, 4 or 8; 0 = the library chooses */
    int32_t flags;        /* PIVOT_PLAN_* bits, 0 = defaults                             */
} pivot_fc_desc;

/* The layer kernels have two forms of the column gather: each gathered
 * element a dependent load x[index] from global memory, or the whole of x
 * first copied into LDS with loads that depend on nothing and the gather run
 * from there (possible when x is small enough: rows of 16-byte vectors, at
 * most 8 vectors per thread and 64 KB of LDS; at batch 1 up to 16 vectors per
 * thread and 150 KB when every work item has a compute unit of its own).  By
 * default the library takes the second form when it is possible and a work
 * item streams 32 KB of weights or more.  These bits force the first form, or
 * the second whenever possible.                                               */
#define PIVOT_PLAN_GATHER_FROM_GLOBAL 1
#define PIVOT_PLAN_GATHER_FROM_LDS_COPY 4
/* pivot_lstm_run normally runs the whole sequence in one launch when the plan
 * allows it (see there); this bit forces one layer launch and one cell launch
 * per step instead (for measurements and as the reference of the parity test). */
#define PIVOT_PLAN_LSTM_LAUNCH_PER_STEP 2
/* ... and this one keeps the one-launch form (where the plan allows it) also for sequences of fewer than
 * 4 steps, which pivot_lstm_run otherwise runs with a launch per step (for measurements and tests). */
#define PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS 8

typedef struct pivot_fc_plan pivot_fc_plan_t;
typedef struct pivot_mlp_plan pivot_mlp_plan_t;

/* Read-only view of a plan's canonical host arrays (valid until the plan is
 * destroyed).  Tiles are numbered by (block row, block column) ascending.
 * Offsets of element (r,c) of tile t in `vals`:
 *   BRC ((t*bh)+r)*bw+c     BCR ((t*bw)+c)*bh+r     CBR ((c*T)+t)*bh+r
 * `chunks` holds nchunks rows of (block_row, tile_begin, tile_end, slot):
 * every block row's tile list cut into consecutive pieces of at most
 * chunk_tiles tiles (an empty block row gives one empty piece), `slot` =
 * ordinal in (block_row, tile_begin) order, rows then stably sorted by
 * descending length (launch order).  part_base[i] = first slot of block row i.
 * Partials of a split block row are added in ascending slot order. */
typedef struct pivot_plan_view {
    int32_t M, K, bh, bw, wdtype, layout, act;
    int32_t nbr, nbc, M_pad, K_pad;
    int32_t T;                 /* kept tiles */
    int32_t chunk_tiles;       /* resolved value */
    int32_t wg_waves;          /* resolved value */
    int32_t row_slices;        /* resolved value */
    int32_t nchunks;
    const int32_t* row_ptr;    /* [nbr+1] */
    const int32_t* col_idx;    /* [T]     */
    const void*    vals;       /* [T*bh*bw] of wdtype */
    const float*   bias_p;     /* [M_pad]  bias_p[r] = bias[prow[r]], 0 in padding */
    const int32_t* invprow;    /* [M]      invprow[prow[r]] = r */
    const int32_t* invpcol;    /* [K]      invpcol[pcol[c]] = c */
    const int32_t* prow_pad;   /* [M_pad]  prow, -1 in padding */
    const int32_t* pcol_pad;   /* [K_pad]  pcol, -1 in padding */
    const int32_t* chunks;     /* [nchunks][4] */
    const int32_t* part_base;  /* [nbr+1] */
    const int32_t* xidx;       /* [T*bw]   xidx[t*bw+c] = pcol_pad[col_idx[t]*bw+c]: the column gather
                                  composed with the tile list, what the device reads */
    const int32_t* xsort;      /* [T*bw] or NULL: the same gather as one list per piece (positions
                                  [tile_begin*bw, tile_end*bw)), ordered by ascending source index, padding
                                  columns last; entry = source | position-in-piece << 19, source field all
                                  ones for a padding column.  Built for fp16 BRC plans whose tiles fit an
                                  MFMA shape, K_pad < 2^19 - 1 and at most 8192 columns per piece: what the
                                  batch 3..16 kernel reads, so that neighbouring lanes gather neighbouring
                                  addresses */
    const int32_t* xsort_blk;  /* same for an input already in block order (source = col_idx[t]*bw+c, all
                                  ones for a padding column, i.e. one at or past K) */
} pivot_plan_view;

int         pivot_version(void);
const char* pivot_last_error(void);

/*
 * pivot_fc_plan - the static, data-independent "compile" step (Eq. 1: the
 * permutations depend on the sparsity pattern only; Section 4.2.1: done at
 * network implementation time).  Validates the permutations, builds the
 * block-sparse index, packs the kept tiles of W' in the requested layout,
 * permutes the bias, cuts the load-balance schedule and (device >= 0) uploads
 * everything in one device allocation owned by the plan.
 *
 *   W         host, M*K elements of wdtype, row-major, in the space `w_space`
 *   tile_mask host, nbr*nbc bytes, row-major, non-zero = tile kept
 *   prow      host, M int32;  pcol host, K int32
 *   bias      host, M floats in natural output coordinates, or NULL (= 0)
 *   out       receives the plan; NULL on error (nothing is leaked)
 *
 * The device path supports BRC plans with power-of-two tiles,
 * 8 <= bh <= 64 and 8 <= bw <= 64 (wdtype F16: bw >= 8; F32: bw >= 4 also
 * holds).  Other shapes/layouts still build host-only plans (device = -1).
 */
int  pivot_fc_plan(const pivot_fc_desc* desc, const void* W, int w_space,
                   const uint8_t* tile_mask, const int32_t* prow, const int32_t* pcol,
                   const float* bias, pivot_fc_plan_t** out);
int  pivot_fc_plan_host_view(const pivot_fc_plan_t* plan, pivot_plan_view* view);
/* A second plan with its own copy of all device arrays (used to rotate
 * through cache-cold copies when measuring). */
int  pivot_fc_plan_clone(const pivot_fc_plan_t* plan, pivot_fc_plan_t** out);
void pivot_fc_plan_destroy(pivot_fc_plan_t* plan);   /* NULL-safe */

/* Scratch a run needs for `batch` rows: arrival counters of split block rows
 * (first; their size does not depend on the batch), their partial sums, and
 * for the matrix-core form that wants it a copy of x in block order.
 * Reuse rule: clear the buffer once with pivot_workspace_init before its first
 * use with a plan; after that any number of runs of THAT plan may share it, in
 * any order of batch sizes (every run leaves the counters at zero, nothing
 * else is read before it is written), as long as it holds
 * pivot_fc_workspace_bytes(plan, batch) for each of them.  Clear it again
 * before using it with another plan (or chain): the counters of one plan lie
 * where another plan keeps partial sums.  Two runs that overlap in time must
 * not share a workspace.  The same rule holds for the chain and recurrent
 * workspaces below. */
size_t pivot_fc_workspace_bytes(const pivot_fc_plan_t* plan, int batch);
int    pivot_workspace_init(void* ws_dev, size_t ws_bytes, void* stream);

/*
 * pivot_fc_run - one application of the layer (Listing 1, generalised to
 * tiles that share rows): gather x through pcol into LDS, stream the kept
 * tiles, reduce, add bias, activate, scatter through prow.
 *
 *   x_dev  device, [batch][K] of wdtype, row stride ldx elements, natural coordinates
 *   y_dev  device, [batch][M] fp32, row stride ldy elements, natural coordinates
 *   batch  1..64.  F16 plans whose tiles fit an MFMA shape use the matrix
 *          cores from batch 3 on: fed from x-segments staged
 *          in LDS (4 or 8 batch rows per workgroup, gathered through the
 *          plan's source-ordered lists) while the staged rows of a work item
 *          fit in 48 KB (beyond batch 16: and the launch rows together
 *          stage at most 5120 columns per work item), else (batch >= 8)
 *          from a copy of x in block order made by one small extra kernel.
 *          Batch 5..16 with at most 4096 input columns, from a quarter of
 *          them staged per work item on: the rows of x are copied into
 *          LDS and the fragments gathered from there (fastest when x is
 *          16-byte aligned, K a multiple of 8 and ldx == K; anything else
 *          gives the same results through an element-wise copy).
 */
int  pivot_fc_run(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx,
                  void* y_dev, int64_t ldy, int batch,
                  void* ws_dev, size_t ws_bytes, void* stream);

/* Which kernel instantiation pivot_fc_run launches for this plan at this
 * batch ("pivot::fc_gemv_kernel<float, 16, 32, 1, 8, 1>": the name a profiler
 * shows), for an x that is 16-byte aligned with densely packed rows (other
 * inputs take the form that gathers from global memory).  buf receives at
 * most buf_len bytes including the terminating 0.  Needs no device. */
int  pivot_fc_kernel_name(const pivot_fc_plan_t* plan, int batch, char* buf, size_t buf_len);

/*
 * pivot_fc_run_static - pivot_fc_run for callers that cannot allocate device
 * memory and have no workspace to hand over: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels, same result bits as pivot_fc_run without the workspace: the scratch
 * of the run (arrival counters and partial sums of split block rows, the
 * block-order copy of x of the matrix-core form that wants one) is a fixed
 * array in device memory that belongs to the library, PIVOT_STATIC_COUNTER_BYTES
 * + PIVOT_STATIC_DATA_BYTES = 16 MiB on every GPU the library runs on, held
 * until the process ends.  The call allocates and frees nothing and never
 * synchronises; its first call on a device looks the array up and enqueues
 * one small kernel on `stream` that clears the counters.
 * A plan whose counters need more than PIVOT_STATIC_COUNTER_BYTES, or whose
 * partial sums and staged input at this batch need more than
 * PIVOT_STATIC_DATA_BYTES, is refused with PIVOT_E_WORKSPACE (use pivot_fc_run).
 * All calls on one GPU share the one array: calls that overlap in time on one
 * GPU (two streams, two threads) race and give undefined results; calls
 * ordered on one stream, or by events, are fine, also with different plans
 * and batch sizes in any order.
 */
#define PIVOT_STATIC_COUNTER_BYTES ((size_t)4 << 20)
#define PIVOT_STATIC_DATA_BYTES    ((size_t)12 << 20)
int  pivot_fc_run_static(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx,
                         void* y_dev, int64_t ldy, int batch, void* stream);

/*
 * Chains of layers (Section 4.2).  Between layer l and l+1 the producer's row
 * scatter and the consumer's column gather are composed at plan time into one
 * index array q_l[c] = invprow_l[pcol_{l+1}[c]] (Section 4.2.1); the device
 * applies it on the producer's store, so intermediates live in the consumer's
 * block order and no separate gather or scatter pass runs.  If
 * pcol_{l+1} == prow_l the composed array is the identity and nothing
 * irregular remains at that boundary (Section 4.2.3).  With
 * PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER the last layer's scatter is dropped and
 * the host relabels outputs with prow of the last layer (Section 4.2.2):
 * y_dev then holds M_pad_last values per batch row in block order (padding
 * entries are not written).
 * Intermediates have the plans' wdtype (F16 chains round once per boundary).
 * All layers must share wdtype and device.  Layer plans are borrowed and must
 * outlive the chain plan.
 *
 * Two forms.  A chain of BRC plans of one tile width whose work items
 * are whole block rows, at most 1024 per layer and all resident on the device
 * at once, runs at batch 1 in ONE launch (view.one_launch = 1): workgroup g
 * takes work item g of every layer in turn, an intermediate activation is
 * stored as a (value, launch tag) pair, and the next layer's gather re-reads
 * the pairs it needs until they carry this launch's tag.  The pairs and the
 * launch counters live in device memory owned by the chain plan, so launches
 * of one chain plan must not overlap (one stream, or ordered by events), and
 * nothing else should occupy the device while it runs: its workgroups wait
 * for each other.  A wait that does not end within 2^18 polls gives up, the
 * status word reads 1 and y_dev is undefined; pivot_mlp_status synchronises
 * the stream, returns the status of the launches since its last call and
 * clears it.  Every other chain and batch (or PIVOT_MLP_LAUNCH_PER_LAYER)
 * runs one launch per layer.
 */
#define PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER 1
#define PIVOT_MLP_LAUNCH_PER_LAYER       2

typedef struct pivot_mlp_view {
    int32_t L;
    int32_t flags;
    const int32_t* const* q;     /* [L-1] arrays, q[l] has K_{l+1} entries                    */
    const int32_t* const* dst;   /* [L-1] arrays, dst[l] has M_pad_l entries:
                                    dst[l][r] = invpcol_{l+1}[prow_l[r]], -1 in padding        */
    const int32_t* identity;     /* [L-1] flags: 1 if q[l] is the identity                    */
    int32_t one_launch;          /* 1 if batch-1 runs of this chain take the one-launch form  */
} pivot_mlp_view;

int    pivot_mlp_plan(pivot_fc_plan_t* const* layers, int L, int flags, pivot_mlp_plan_t** out);
int    pivot_mlp_plan_host_view(const pivot_mlp_plan_t* plan, pivot_mlp_view* view);
void   pivot_mlp_plan_destroy(pivot_mlp_plan_t* plan);
size_t pivot_mlp_workspace_bytes(const pivot_mlp_plan_t* plan, int batch);
/* x_dev [batch][K_1] (stride ldx), y_dev [batch][M_L] fp32 (stride ldy), or
 * [batch][M_pad_L] in block order with PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER. */
int    pivot_mlp_run(const pivot_mlp_plan_t* plan, const void* x_dev, int64_t ldx,
                     void* y_dev, int64_t ldy, int batch,
                     void* ws_dev, size_t ws_bytes, void* stream);
/* *status = 0 if every one-launch run of this chain since the last call completed, 1 if a wait gave up. */
int    pivot_mlp_status(const pivot_mlp_plan_t* plan, void* stream, int* status);
/* The same information without a synchronising call: *word_dev receives the device address of the chain's
 * status word (a uint32 owned by the chain plan; NULL if the chain has no one-launch form).  It reads 0 while
 * every one-launch run since the last pivot_mlp_status completed and 1 once a wait has given up; the caller
 * may read it on its own schedule, e.g. with an asynchronous copy to pinned host memory enqueued behind the
 * run, or from a kernel of its own.  When it reads 1 the outputs of that run are undefined and the caller
 * has to run the chain again through a chain plan made with PIVOT_MLP_LAUNCH_PER_LAYER (whose kernels wait
 * for nothing).  When to choose which form: the one-launch form needs the device to itself for the few
 * microseconds it runs (its workgroups wait for each other and must all be resident); a process that shares
 * the GPU with other streams or processes that can occupy compute units for long should make its chain
 * plans with PIVOT_MLP_LAUNCH_PER_LAYER, and its recurrent plans with PIVOT_PLAN_LSTM_LAUNCH_PER_STEP. */
int    pivot_mlp_status_word(const pivot_mlp_plan_t* plan, const uint32_t** word_dev);

/*
 * Recurrent use: an LSTM whose gate matrix (4H x (H+I), gate order i,f,g,o,
 * input [h_{t-1}; x_t]) is a pruned layer.  The recurrence is a PBP layer
 * back-to-back with itself through a point-wise cell, so the boundary fusion
 * of Section 4.2.1 applies: the cell writes h_t straight into the block-order
 * input of the next step through invpcol, so no step gathers its input; all
 * x_t are placed once up front.
 *
 *   xs_dev   device, [steps][batch][I] of wdtype
 *   h_dev    device, [batch][H] fp32: h_0 on entry, h_steps on return
 *   c_dev    device, [batch][H] fp32: c_0 on entry, c_steps on return
 *   z_dbg    device, optional [batch][4H] fp32: gate pre-activations of the
 *            last step in natural order (NULL to skip)
 *
 * Two forms.  Plans with fp16 16x32 BRC tiles, batch <= 8, at most 15 kept
 * tiles per wavefront of a full-device grid (one workgroup per compute unit,
 * all co-resident) and K_pad/32 <= that grid run the whole sequence in ONE
 * launch: the kept tiles stay in registers for all steps and per step only h,
 * x_t and the gate sums move.  There are no grid barriers: the exchanged data
 * carries the step it belongs to and a consumer re-reads until it sees its
 * step.  Its workgroups wait for each other, so nothing else should occupy
 * the device while it runs; a wait that does not end within 2^18 polls gives
 * up, every workgroup leaves, h/c are left unwritten and the status word
 * reads 1.  Every other plan (or
 * PIVOT_PLAN_LSTM_LAUNCH_PER_STEP), and every sequence of fewer than 4 steps,
 * runs one layer launch and one cell launch per step (the one-launch form
 * loads every kept tile into registers first: a first step from weights that
 * are not in cache costs it 23 us on the 8192x3072 workload against 18 us with
 * launches per step, every further step 6.8 against 9.1 us: it is ahead from
 * the fourth step on).  pivot_lstm_status synchronises the stream and returns the status
 * word of the last pivot_lstm_run on this workspace (0 = completed).
 */
size_t pivot_lstm_workspace_bytes(const pivot_fc_plan_t* plan, int H, int I, int steps, int batch);
int    pivot_lstm_status(const pivot_fc_plan_t* plan, int steps, int batch, const void* ws_dev, void* stream, int* status);
/* Device address of that status word inside the workspace (for the same steps and batch), for callers that
 * read it on their own schedule instead of synchronising; see pivot_mlp_status_word.  The launch-per-step
 * form leaves it at 0. */
int    pivot_lstm_status_word(const pivot_fc_plan_t* plan, int steps, int batch, const void* ws_dev, const uint32_t** word_dev);
int    pivot_lstm_run(const pivot_fc_plan_t* plan, int H, int I, const void* xs_dev,
                      float* h_dev, float* c_dev, float* z_dbg, int steps, int batch,
                      void* ws_dev, size_t ws_bytes, void* stream);

/*
 * The dense comparator: y = act(W x + b) with the full M x K matrix streamed
 * by this library's own dense kernel (the denominator of "speedup vs dense",
 * Section 5.1).  W_dev [M][K] of wdtype row-major, x_dev [batch][K] of
 * wdtype, bias_dev [M] fp32 or NULL, y_dev [batch][M] fp32.  batch 1..16.
 */
int  pivot_dense_run(const void* W_dev, int wdtype, int M, int K,
                     const void* x_dev, int64_t ldx, const float* bias_dev,
                     void* y_dev, int64_t ldy, int batch, int act, void* stream);

/*
 * pivot_feedback_search - the producer of pivot_fc_plan's inputs: feed-back
 * PBP pruning (Section 3.2).  From the magnitudes |W| of a trained dense layer
 * it picks prow and pcol by `levels` rounds of bisection: every block's rows
 * and columns are split in halves so that the upper-left and lower-right
 * sub-blocks hold as much magnitude as a greedy alternating search finds (the
 * off-diagonal sub-blocks are what pruning then deletes, so every level halves
 * the fill-in).  The search starts from prow0 / pcol0 (the paper starts from
 * random permutations; the caller draws them) and is deterministic.  All
 * pointers are host memory.  absW is M*K row-major, non-negative.  On return
 * W'[r][c] = W[prow_out[r]][pcol_out[c]] has its kept mass in 2^levels diagonal
 * blocks whose row ranges follow from halving [0,M) `levels` times (floor
 * first), columns likewise; *captured_mass (optional) is the sum of absW there.
 */
int  pivot_feedback_search(const float* absW, int M, int K, int levels, int max_iter,
                           const int32_t* prow0, const int32_t* pcol0,
                           int32_t* prow_out, int32_t* pcol_out, double* captured_mass);

/*
 * The generic sparse comparator: y = act(A x + b), A given in plain CSR
 * (natural coordinates, all on the device: row_ptr [M+1], col [nnz],
 * val [nnz] of wdtype), x [K] of wdtype, bias [M] fp32 or NULL, y [M] fp32,
 * batch 1.  This is the kind of routine a pruned layer is usually handed to;
 * the paper's second speedup column (Table 1a) is measured against one.
 */
int  pivot_csr_run(const int32_t* row_ptr_dev, const int32_t* col_dev, const void* val_dev, int wdtype,
                   int M, int64_t nnz, const void* x_dev, const float* bias_dev, float* y_dev,
                   int act, void* stream);

/* Measurement aid: enqueues one empty kernel (a single wavefront that does
 * nothing), so that a harness can report the launch floor of the device next
 * to the layer times (the paper averages whole calls, Section 5.1). */
int  pivot_null_run(void* stream);

/* Measurement aid: one launch (256 workgroups of 8 wavefronts, 16 bytes per
 * lane, eight loads in flight per wavefront) that does nothing but read the
 * first bytes/1024 KB of buf_dev once and store one float per wavefront to
 * out_dev (2048 floats).  Its time, cache-cold, is what a single launch of the
 * layer kernel cannot beat for the same number of bytes on this device: the
 * measured counterpart of the bandwidth roofline for layers of a few MB. */
int  pivot_stream_read_run(const void* buf_dev, size_t bytes, float* out_dev, void* stream);

/* Measurement aid for the one-launch forms, whose workgroups hand data to each
 * other inside a launch (chains: Section 4.2; the recurrent loop): what ONE
 * trip between two workgroups costs.  One launch of one workgroup per compute
 * unit (at most 256); every workgroup publishes the number of the XCD it runs
 * on, then workgroup 0 bounces a 4-byte word `rounds` times with a partner on
 * its own XCD and with one on another XCD, timing each series with the
 * device's 100 MHz clock:
 *   out[1] same XCD, device-coherent store / load (what the kernels use)
 *   out[2] same XCD, workgroup-scope atomics
 *   out[3] other XCD, device-coherent store / load
 *   out[6] same XCD, plain store, L1 invalidate + plain load (through the XCD's L2)
 * each in clock ticks for the whole series (2 * rounds trips), or -1 if a wait
 * gave up (every wait is bounded); out[0] = 1 when the probe ran, -1 if the
 * workgroups were not all resident or no partner was found; out[4], out[5] =
 * the partners.  scratch_dev: PIVOT_PROBE_SCRATCH_BYTES of device memory,
 * 256-byte aligned; the call clears it (on `stream`) and leaves the results,
 * eight int64, at its start.  rounds: 1..100000.  Asynchronous like the other
 * run calls; PIVOT_E_* on bad arguments. */
#define PIVOT_PROBE_SCRATCH_BYTES ((size_t)32768)
int  pivot_exchange_probe_run(void* scratch_dev, size_t scratch_bytes, int rounds, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PIVOT_FC_H */
