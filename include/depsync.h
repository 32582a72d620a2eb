/*
 * depsync -- fine-grained synchronisation of dependent tiled kernels on one MI355X (gfx950).
 *
 * C ABI of the library.  A "chain" is a producer kernel followed by a consumer kernel whose
 * one input is the producer's output (Section III of the paper, Fig. 4a: the host function
 * MLP(BS, H, X, W1, XW1, W2, XW12)).  Instead of letting the whole producer finish before
 * the consumer starts, both are launched on two streams of the same GPU and every consumer
 * tile waits, through semaphores in device memory, only for the producer tiles it reads
 * (Sections III-A to III-D).  A synchronisation policy maps producer tiles to semaphores
 * (Section III-E).
 *
 * Conventions
 *  - Every function returns an int status: DEPSYNC_OK (0) or a negative DEPSYNC_E* code.
 *    Nothing throws or aborts across this boundary.
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library never frees
 *    or reallocates them and keeps no reference after the call returns.
 *  - Calls that enqueue work are asynchronous.  On return, work enqueued later on
 *    stream_producer is ordered after the whole chain (the library forks the consumer
 *    stream off the producer stream with an event and joins it back).  One exception: a chain
 *    whose stages are split along K keeps fp32 partial tiles in a scratch buffer the policy
 *    owns, and the first chain that needs a larger one than any before it on that policy
 *    synchronises the device and reallocates it (hipFree + hipMalloc) before it enqueues.
 *    All chains that use one policy must be enqueued on the same stream_producer (the implicit
 *    re-zeroing of the workspace is ordered on it).
 *  - Streams are hipStream_t handles passed as void*; NULL means the default stream for
 *    stream_producer and "use the policy's own internal stream" for stream_consumer.
 *  - Semaphores, the tile-dispatch counter and the status block live in a small workspace
 *    owned by the sync_policy_t object.  One policy object must not be used by two chains
 *    that can run concurrently; calls using one policy must be enqueued in host-call order.
 *  - Element type is 16-bit (bf16 or fp16) with fp32 accumulation; the intermediate and the
 *    output are rounded to the 16-bit type with round-to-nearest-even.
 *  - Every row must start on a 16-byte boundary: base pointers 16-byte aligned and leading
 *    dimensions multiples of 8 elements; inner (K) dimensions multiples of 64.  The
 *    intermediate (H, mid) must additionally be 128-byte aligned with a leading dimension
 *    that is a multiple of 64 elements, so that no cache line holds the output of two producer
 *    tiles.  Violations return DEPSYNC_EINVAL.
 */
#ifndef DEPSYNC_H
#define DEPSYNC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------------------ */
#define DEPSYNC_OK 0
#define DEPSYNC_EINVAL (-1)   /* null pointer, bad shape, bad alignment, bad enum          */
#define DEPSYNC_ENOMEM (-2)   /* workspace allocation failed                               */
#define DEPSYNC_EHIP (-3)     /* a HIP call failed; see depsync_last_hip_error()           */
#define DEPSYNC_ETIMEOUT (-4) /* a bounded wait (spin_limit) expired; see depsync_last_status */
#define DEPSYNC_ENOTIMPL (-5) /* valid request this build does not implement               */
#define DEPSYNC_ELIMIT (-6)   /* dep_gemm_chain_static: the chain needs more semaphores, arrival
                                 counters or split-K scratch than the fixed workspace holds   */

/* Synchronisation policies (Section III-E and Section IV-B). */
typedef enum {
    DEPSYNC_ROWSYNC = 0,    /* all column tiles of a producer row share a semaphore       */
    DEPSYNC_TILESYNC = 1,   /* one semaphore per producer tile                            */
    DEPSYNC_STRIDEDSYNC = 2,/* producer tiles at a fixed stride share a semaphore         */
    DEPSYNC_AUTOSYNC = 3    /* whichever of the three depsync_*_chain_autotune_policy measured
                               fastest for the chain's shape (Section IV-A: the policy is part
                               of what the paper's generator searches); where nothing was
                               measured, the rule of thumb of Section V-C: TILESYNC up to 256
                               rows, ROWSYNC beyond, STRIDEDSYNC for attention and convolutions;
                               copy chains: TILESYNC                                           */
} depsync_policy_kind;

/* How the two kernels of a chain are ordered. */
typedef enum {
    DEPSYNC_MODE_FINE = 0,       /* two streams, per-tile semaphores (the paper's method)  */
    DEPSYNC_MODE_STREAMSYNC = 1, /* the same kernels on one stream (the paper's baseline)  */
    DEPSYNC_MODE_PLAIN = 2,      /* the same tile code with the sync hooks compiled out,
                                    one stream, hardware block order                        */
    DEPSYNC_MODE_FUSED = 3       /* per-tile semaphores as in FINE, but ONE dispatch holding the
                                    workgroups of all stages on stream_producer: no second
                                    stream, no event fork/join (a few microseconds each on
                                    this GPU).  Possible because every workgroup draws its
                                    tile from the shared queues whichever launch it is from  */
} depsync_mode;

/* What sits between the two GeMMs. */
typedef enum {
    DEPSYNC_MID_NONE = 0,
    DEPSYNC_MID_GELU = 1,        /* Fig. 2a; exact erf form                                 */
    DEPSYNC_MID_RELU = 2,
    DEPSYNC_MID_SWIGLU = 3,      /* Fig. 3: silu(gate) * up, fused into the producer tile   */
    DEPSYNC_MID_CAUSAL_ATTN = 4  /* Fig. 2b, prompt phase: a third, middle kernel           */
} depsync_mid;

typedef enum { DEPSYNC_BF16 = 0, DEPSYNC_FP16 = 1 } depsync_dtype;

/* Layout of the weight operands of a GeMM chain (both are K-contiguous per output column n):
 *   ROWS     [N x K] row-major with a leading dimension (the nn.Linear layout);
 *   KBLOCKED [K/64][N][64]: blocks of 64 K-elements, all N rows of a block adjacent, so that
 *            the slice one tile reads per pipeline step is one contiguous run of memory
 *            (weights are static: packed once; ldw1 / ldw2 are ignored).                     */
typedef enum { DEPSYNC_W_ROWS = 0, DEPSYNC_W_KBLOCKED = 1 } depsync_w_layout;

/* Macro-tile shapes (rows x columns of the output computed by one workgroup). */
typedef enum {
    DEPSYNC_TILE_AUTO = 0,
    DEPSYNC_TILE_256x256 = 1,
    DEPSYNC_TILE_256x128 = 2,
    DEPSYNC_TILE_128x256 = 3,
    DEPSYNC_TILE_128x128 = 4,
    DEPSYNC_TILE_64x128 = 5,
    DEPSYNC_TILE_64x64 = 6,
    DEPSYNC_TILE_256x192 = 7,  /* 192-wide tiles divide widths of the form 3 * 2^k evenly */
    DEPSYNC_TILE_128x192 = 8,
    DEPSYNC_TILE_256x64 = 9,   /* narrow outputs (64 channels)                           */
    DEPSYNC_TILE_64x64_DEEP = 10, /* 64x64 with an 8-stage operand pipeline, one workgroup per
                                  CU: for chains of few tiles that stream weights from HBM */
    DEPSYNC_TILE_64x192 = 11,  /* 64 rows, 192 columns, 4-stage pipeline, one workgroup per CU: skinny M on
                                  widths of the form 3 * 2^k, where it splits into 256 equal parts     */
    DEPSYNC_TILE_128x192_DEEP = 12, /* 128x192 and 128x128 with a 4-stage operand pipeline, one workgroup */
    DEPSYNC_TILE_128x128_DEEP = 13, /* per CU: mid-size M, where a tile's weights come from HBM, not L2  */
    DEPSYNC_TILE__COUNT = 14
} depsync_tile;

/* Policy flags. */
#define DEPSYNC_FLAG_NO_REORDER 1u    /* do NOT load the independent operand before the wait
                                         (switches off the reordering of Section IV-C)       */
#define DEPSYNC_FLAG_COUNT 2u         /* count posts / waits / polling waits in the status   */
#define DEPSYNC_FLAG_REVERSE_ORDER 4u /* debug: hand producer tiles out in reverse order     */
#define DEPSYNC_FLAG_HW_ORDER 8u      /* take the tile from the hardware block index, no dispatch
                                         counter ("avoid custom tile order", Section IV-C).  In FINE
                                         mode only legal when the tiles of all stages fit on the GPU
                                         at once (otherwise DEPSYNC_EINVAL).  In FUSED mode legal for
                                         any chain, but for a chain of more tiles than resident
                                         workgroups it rests on each XCD starting the workgroups of
                                         one dispatch in index order, producers first, which HIP
                                         does not promise (observed on MI355X; the bounded wait turns
                                         a violation into DEPSYNC_ETIMEOUT).  Without this flag the
                                         library names tiles by the block index only when every tile
                                         has a resident workgroup of its own, where any start order
                                         is safe, and draws them from the dispatch queues otherwise. */

typedef struct {
    uint32_t stride;      /* STRIDEDSYNC on a GeMM chain: distance, in producer column tiles,
                             between tiles that share a semaphore; 0 = derive from the chain  */
    uint32_t count;       /* STRIDEDSYNC: tiles per semaphore; 0 = derive                     */
    uint32_t flags;       /* DEPSYNC_FLAG_*                                                   */
    uint32_t spin_limit;  /* give up a wait after this many polls, record DEPSYNC_ETIMEOUT in the
                             status and skip the tile's stores; 0 = the default bound (2^22 polls,
                             a few seconds), 0xffffffff = wait without bound                    */
    uint32_t delay_tile;  /* debug: producer tile (row-major index) + 1 to delay; 0 = none    */
    uint32_t delay_iters; /* debug: s_sleep iterations the delayed tile spends before its post */
    uint32_t ksplit;      /* workgroups per output tile, each over an equal part of K (the grid's z
                             of Tables I and IV).  0 = the library splits stages that would leave
                             most of the chip idle; 1 = never; n = n parts wherever K divides so
                             that parts start on dependency boundaries.  The parts leave fp32
                             partial tiles in a scratch buffer the policy owns; the last to arrive
                             adds them in K order, so results do not depend on timing.           */
} depsync_policy_params;

#define DEPSYNC_FLAG_TRACE 16u        /* record per-tile start / ready / end times (FINE and
                                         STREAMSYNC); read them with depsync_read_trace        */
#define DEPSYNC_FLAG_QUEUE_ORDER 32u  /* FUSED: draw tiles from the dispatch queues (persistent
                                         workgroups) even where the library would name them by the
                                         block index (chains whose tiles are all resident at once) */

typedef struct sync_policy sync_policy_t;

/* Per-tile timing record; times are ticks of the GPU's constant 100 MHz counter. */
typedef struct {
    uint32_t rel;       /* producer tiles: row-major index; later stages: offset by the tiles
                           of the stages before                                               */
    uint32_t where;     /* bits 0-7: 1 if the tile had a dependency, else 0; 8-15: XCD;
                           16-23: CU within its shader array; 24-31: shader engine            */
    uint32_t tx, ty;    /* column tile, row tile                                              */
    uint64_t t_enter;   /* workgroup started (before it drew its tile)                        */
    uint64_t t_start;   /* tile handed out                                                    */
    uint64_t t_ready;   /* first dependency satisfied (t_start's neighbour if none)           */
    uint64_t t_end;     /* stores and post done                                               */
} depsync_trace_rec;

typedef struct {
    int32_t timed_out;       /* number of waves (four per tile) whose bounded wait expired    */
    int32_t first_timeout;   /* dispatch ticket of the first such tile, -1 if none            */
    uint32_t posts;          /* with DEPSYNC_FLAG_COUNT: semaphore increments                 */
    uint32_t waits;          /* with DEPSYNC_FLAG_COUNT: semaphore waits executed             */
    uint32_t polling_waits;  /* ... of which the first read did not already satisfy the wait  */
    uint32_t launches;       /* chains enqueued with this policy since create/reset           */
} depsync_status;

/* What the library decided for a chain (for reports; filled by depsync_*_chain_plan). */
typedef struct {
    int32_t tile_prod, tile_mid, tile_cons;   /* depsync_tile ids (tile_mid: attention only)  */
    int32_t prod_grid_x, prod_grid_y;         /* column tiles, row tiles of the producer      */
    int32_t mid_grid_x, mid_grid_y;
    int32_t cons_grid_x, cons_grid_y;
    int32_t n_prod, n_mid, n_cons;            /* tiles per stage                              */
    int32_t n_sems;                           /* semaphores used                              */
    int32_t slots;                            /* workgroups resident at once (CUs x occupancy) */
    int32_t waves_streamsync, waves_fine;     /* ceil(P/slots)+ceil(C/slots), ceil((P+C)/slots) */
    double flops;                             /* algorithmic flops of the chain               */
    double bytes;                             /* algorithmic bytes: every operand once        */
} depsync_plan_info;

/*
 * GeMM -> (pointwise | attention) -> GeMM (Fig. 2a, Fig. 2b, Fig. 3).
 *   H = mid(X W1)        X[M x K1], W1 mathematically [K1 x N1w]
 *   Y = H' W2            W2 mathematically [K2 x N2]
 * Weights are passed TRANSPOSED, i.e. as row-major [N x K] arrays (the layout in which
 * torch.nn.Linear stores its weight), so that both MFMA operands are contiguous along K.
 *   mid = NONE/GELU/RELU : N1w = N1, H[M x N1] is the intermediate, K2 = N1.
 *   mid = SWIGLU         : W1t has 2*N1 rows: gate rows [0,N1), up rows [N1,2*N1);
 *                          H[M x N1] = silu(gate) * up, K2 = N1.
 *   mid = CAUSAL_ATTN    : N1 = 3*heads*head_dim, H = QKV[M x N1] with column blocks
 *                          Q | K | V, head h at columns h*head_dim inside each block;
 *                          T[M x heads*head_dim] = per-head causal softmax(QK^T/sqrt(d)) V
 *                          over each of `batch` sequences of `seq` rows (M = batch*seq);
 *                          K2 = heads*head_dim, Y = T W2.  Built for head_dim = 128 (other
 *                          values: DEPSYNC_ENOTIMPL); with batch > 1, seq must be a multiple
 *                          of 128 (else DEPSYNC_ENOTIMPL).  T, like H, must be 128-byte
 *                          aligned with ldt a multiple of 64.  The chain then has three
 *                          stages; with DEPSYNC_STRIDEDSYNC the attention stage waits on one
 *                          semaphore per producer row tile shared by the Q, K and V column
 *                          tiles of its head and the last GeMM waits per attention tile
 *                          (Section V-C, "Strided + TileSync").
 */
typedef struct {
    int32_t M, K1, N1, N2;
    int32_t dtype;               /* depsync_dtype                                            */
    int32_t mid;                 /* depsync_mid                                              */
    const void* X;   int64_t ldx;   /* [M x K1]                                              */
    const void* W1t; int64_t ldw1;  /* [N1 (2*N1 for SWIGLU) x K1]                           */
    void* H;         int64_t ldh;   /* [M x N1]   intermediate, written then read            */
    const void* W2t; int64_t ldw2;  /* [N2 x K2]                                             */
    void* Y;         int64_t ldy;   /* [M x N2]                                              */
    void* T;         int64_t ldt;   /* CAUSAL_ATTN only: [M x heads*head_dim]                */
    int32_t batch, seq, heads, head_dim; /* CAUSAL_ATTN only; batch > 1 needs seq % 128 == 0 or seq < 128 */
    int32_t tile_prod, tile_cons;   /* depsync_tile of the first and of the last GeMM; 0 = chosen by
                                     * the library.  They may differ (the consumer waits by the rows
                                     * and columns of the producer's tiles, Section III-C): each stage
                                     * is then a launch of its own kernel, so MODE_FUSED returns
                                     * DEPSYNC_ENOTIMPL, and MODE_FINE holds the consumer's launch
                                     * back with the wait kernel of Section III-B until the
                                     * producer's workgroups are resident.  CAUSAL_ATTN chains take
                                     * one shape for all three stages (else DEPSYNC_ENOTIMPL).     */
    int32_t w_layout;               /* depsync_w_layout of W1t and W2t                       */
    /* CAUSAL_ATTN, token generation (Fig. 2b, cached keys and values): `cached` earlier tokens
     * per sequence whose keys and values are read from k_cache / v_cache, [batch][cached] rows of
     * ld_cache elements (>= heads*head_dim, multiple of 8), head h in columns h*head_dim..;
     * device, 16-byte aligned, read only.  New token i of a sequence attends to all cached
     * tokens and to new tokens 0..i.  cached = 0: prompt phase, the pointers are ignored.      */
    const void* k_cache;
    const void* v_cache;
    int64_t ld_cache;
    int32_t cached;
} depsync_gemm_chain_desc;

/*
 * Conv2D -> ReLU -> Conv2D by implicit GeMM (Section IV-B "Conv2D"): 3x3, stride 1, zero
 * padding 1, cross-correlation, NHWC activations, weights [K][3][3][C] (C contiguous):
 *   mid[b,y,x,k] = relu(sum_{r,s,c} in[b,y+r-1,x+s-1,c] w1[k,r,s,c]);  out = conv(mid, w2).
 * C and K1 must be multiples of 64.
 */
typedef struct {
    int32_t B, H, W, C, K1, K2;
    int32_t dtype;
    const void* in;   /* [B,H,W,C]   */
    const void* w1;   /* [K1,3,3,C]  */
    void* mid;        /* [B,H,W,K1]  */
    const void* w2;   /* [K2,3,3,K1] */
    void* out;        /* [B,H,W,K2]  */
    int32_t tile_prod, tile_cons;   /* as in depsync_gemm_chain_desc: may differ (not in MODE_FUSED) */
} depsync_conv_chain_desc;

/*
 * Chain of n = 2..4 such convolutions with ReLU between them and none after the last, as in the
 * layers of VGG (Section V, the chains of more than two convolutions): conv i reads the output
 * of conv i-1 (conv 0 reads `in`) and each later stage waits on the one before it as the
 * policy says.  K[i] = output channels of conv i; C and K[i] for i < n-1 multiples of 64, K[n-1]
 * a multiple of 8.  w[i]: [K[i],3,3,Cin_i]; out[i]: [B,H,W,K[i]], out[n-1] the result, the
 * others intermediates (caller's buffers, 128-byte aligned, written then read).  Entries of K, w
 * and out beyond n are ignored.  n = 2 is the same computation as depsync_conv_chain_desc.
 */
typedef struct {
    int32_t B, H, W, C;
    int32_t n;
    int32_t K[4];
    int32_t dtype;
    const void* in;
    const void* w[4];
    void* out[4];
    int32_t tile_prod, tile_cons;   /* 0 = library's choice; for n = 2 they may differ as in
                                     * depsync_conv_chain_desc, for n > 2 one shape serves every
                                     * stage (else DEPSYNC_ENOTIMPL)                              */
} depsync_conv_chain_n_desc;

/* ---- policy objects (CuStage + policy of Fig. 4; init of Section III-D) ------------- */

/* Create a policy and its workspace on the current device.  params may be NULL.          */
int sync_policy_create(depsync_policy_kind kind, const depsync_policy_params* params,
                       sync_policy_t** out);
/* Synchronises the device, then frees the workspace.                                      */
int sync_policy_destroy(sync_policy_t* pol);
/* Bytes of device memory sync_policy_create allocates for a policy's workspace (dispatch
 * counters, status block, zero page, semaphores, trace records, arrival counters); the same
 * for every policy.  The split-K partial tiles are extra and grow with the chains run.   */
size_t depsync_workspace_bytes(void);
/* Re-zero semaphores, dispatch counter and status on `stream` (a fill kernel, safe under
 * graph capture) and restart the launch epoch.  Needed only after DEPSYNC_ETIMEOUT.       */
int dep_chain_reset(sync_policy_t* pol, void* stream);
/* Synchronises the policy's streams, then copies the status block to the host.  Returns
 * DEPSYNC_ETIMEOUT if a bounded wait expired since the last reset.                        */
int depsync_last_status(sync_policy_t* pol, depsync_status* out);

/* Synchronises the device and copies up to max_records trace records (index = rel) of the
 * last chain run with DEPSYNC_FLAG_TRACE; returns the number copied or a negative status.
 * At most 8192 tiles are traced.                                                          */
int depsync_read_trace(sync_policy_t* pol, depsync_trace_rec* out, int max_records);

/* ---- chains -------------------------------------------------------------------------- */

/* Enqueue the GeMM chain.  Section III, Fig. 4a.                                          */
int dep_gemm_chain(const depsync_gemm_chain_desc* d, sync_policy_t* pol, depsync_mode mode,
                   void* stream_producer, void* stream_consumer);
/* Enqueue the Conv2D chain.  Section IV-B.                                                */
int dep_conv_chain(const depsync_conv_chain_desc* d, sync_policy_t* pol, depsync_mode mode,
                   void* stream_producer, void* stream_consumer);
/* Enqueue a chain of 2..4 convolutions (same conventions; two-stream mode uses one stream per
 * stage, the library's own for the third and fourth).  DEPSYNC_EINVAL for n outside 2..4.    */
int dep_conv_chain_n(const depsync_conv_chain_n_desc* d, sync_policy_t* pol, depsync_mode mode,
                     void* stream_producer, void* stream_consumer);
/* Dry run: validate the descriptor and report tiles, grids, wave counts, flops and bytes
 * without touching the device workspace.  n_cu <= 0 reads the CU count from the current
 * device (which then must exist).                                                          */
int depsync_gemm_chain_plan(const depsync_gemm_chain_desc* d, const sync_policy_t* pol,
                            int n_cu, depsync_plan_info* out);
int depsync_conv_chain_plan(const depsync_conv_chain_desc* d, const sync_policy_t* pol,
                            int n_cu, depsync_plan_info* out);
/* For chains of more than three stages n_mid counts the tiles of all middle stages and the
 * middle grid is that of the second stage.                                                  */
int depsync_conv_chain_n_plan(const depsync_conv_chain_n_desc* d, const sync_policy_t* pol,
                              int n_cu, depsync_plan_info* out);

/* Tile selection by measurement (the role of the paper's policy/order search of Section IV-A,
 * narrowed to the macro-tile shape and the split along K): runs the chain in one-dispatch mode
 * on `stream` with every macro-tile shape it supports, with and without the library's own
 * split along K, with tiles drawn from the dispatch queues or named by the block index (two passes; a warm-up launch, then at least `reps` timed launches each, more
 * for chains too short to time; reps <= 0 means 3), synchronises, and remembers the fastest
 * combination for this chain shape, element type and policy kind for the rest of the process:
 * later calls that leave the tile to the library (DEPSYNC_TILE_AUTO) use it, in every launch
 * mode.  The intermediate and output buffers are
 * overwritten.  The tile ids in `d` are ignored; *tile_out (nullable) receives the choice.     */
int depsync_gemm_chain_autotune(const depsync_gemm_chain_desc* d, sync_policy_t* pol, void* stream,
                                int reps, int* tile_out);
int depsync_conv_chain_autotune(const depsync_conv_chain_desc* d, sync_policy_t* pol, void* stream,
                                int reps, int* tile_out);
int depsync_conv_chain_n_autotune(const depsync_conv_chain_n_desc* d, sync_policy_t* pol, void* stream,
                                  int reps, int* tile_out);

/* The policy part of that search: runs the autotuner above under each of ROWSYNC, TILESYNC and
 * STRIDEDSYNC (kinds the chain cannot run under are skipped), remembers the fastest kind for this
 * chain shape and element type for the rest of the process, and with it the tile choice of every
 * kind tried.  Policies created as DEPSYNC_AUTOSYNC resolve to the remembered kind at every
 * launch.  `pol` lends its workspace and parameters (any kind; unchanged on return).  *kind_out,
 * *tile_out (nullable) receive the choice; us_out (nullable) points to three floats that receive
 * the best one-dispatch latency under each kind in microseconds, -1 where the kind was skipped.    */
int depsync_gemm_chain_autotune_policy(const depsync_gemm_chain_desc* d, sync_policy_t* pol, void* stream,
                                       int reps, int* kind_out, int* tile_out, float* us_out);
int depsync_conv_chain_n_autotune_policy(const depsync_conv_chain_n_desc* d, sync_policy_t* pol, void* stream,
                                         int reps, int* kind_out, int* tile_out, float* us_out);
/* The kind a chain of this shape runs under with `pol`: pol's own, or what DEPSYNC_AUTOSYNC
 * resolves to (no device access).                                                              */
int depsync_gemm_chain_policy(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int* kind);
int depsync_conv_chain_n_policy(const depsync_conv_chain_n_desc* d, const sync_policy_t* pol, int* kind);

/* The remembered choice for this chain shape, element type and policy kind, read or set without
 * measuring (to carry a tuning result from one process to the next).  `tile` is a DEPSYNC_TILE_*
 * id, 0 when nothing is remembered (setting 0 forgets the entry); `flags`: DEPSYNC_TUNED_*.
 * Only the shape fields of `d` are read (no pointer in it is dereferenced).  Setting a tile the
 * chain cannot run with makes later launches that leave the tile to the library fail with
 * DEPSYNC_EINVAL; a wrong flag can only cost time.  DEPSYNC_EINVAL for null arguments, an
 * unknown tile id or unknown flag bits.                                                       */
enum {
    DEPSYNC_TUNED_NO_SPLIT = 1,   /* do not split stages along K (Section V-C's partial waves are
                                   * left to the overlap of the stages alone)                   */
    DEPSYNC_TUNED_HW_ORDER = 2    /* one-dispatch mode names tiles by the block index instead of
                                   * drawing them from the dispatch queues (Section IV-C, the
                                   * optimisation that avoids a custom tile order); honoured only
                                   * for chains whose tiles are all resident at once, and measured
                                   * by the autotuner only for those (or under DEPSYNC_FLAG_HW_ORDER) */
};
int depsync_gemm_chain_tuned(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int* tile, int* flags);
int depsync_conv_chain_tuned(const depsync_conv_chain_desc* d, const sync_policy_t* pol, int* tile, int* flags);
int depsync_gemm_chain_set_tuned(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int tile, int flags);
int depsync_conv_chain_set_tuned(const depsync_conv_chain_desc* d, const sync_policy_t* pol, int tile, int flags);


/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The same chain as dep_gemm_chain in DEPSYNC_MODE_FUSED (one
 * dispatch on `stream`, per-tile semaphores, bit-identical results for the same policy kind and
 * parameters), but it needs no sync_policy_t object and calls no hipMalloc / hipFree or any other
 * allocating routine: dispatch counters, semaphores, arrival counters and the split-K partial tiles
 * live in one fixed array in device memory that is part of the library's code object (129.5 MiB:
 * 1.5 MiB for counters and up to 8192 semaphores and 4096 arrival counters, 128 MiB for partial
 * tiles; every GPU the library runs on holds its own copy until the process ends).  A chain that
 * needs more than that returns DEPSYNC_ELIMIT and enqueues nothing; params->ksplit = 1 (no split
 * along K) makes any chain need no partial tiles.  DEPSYNC_FLAG_TRACE is not available here
 * (DEPSYNC_EINVAL).  `kind` and `params` (nullable) are what sync_policy_create would be given.
 * The first call on a device looks up the array's device address and enqueues one small fill
 * kernel before the chain.  All calls on one GPU share that GPU's array, which keeps what the last
 * call left in it (the library re-zeroes by fill kernels on `stream` whatever must start at zero
 * when the chain's geometry changes): calls must be enqueued on one stream, or otherwise be ordered
 * one after the other; chains of this entry point that overlap on one GPU race.  The status of
 * bounded waits is not readable through this entry point.                                         */
int dep_gemm_chain_static(const depsync_gemm_chain_desc* d, depsync_policy_kind kind,
                          const depsync_policy_params* params, void* stream);

/* Host-side check of the wait placement (no device needed; n_cu as for the planners; pointers in
 * `d` are validated but not dereferenced): plans the chain for the given policy kind and
 * parameters, walks every consumer tile's K loop the way the kernel does, and counts in
 * *uncovered the (row tile, K part) pairs for which some K step loads a slice of the previous
 * stage's output that no wait issued at or before that step covers (Section III-C: a tile may
 * only read what the tiles it depends on have posted).  0 for every chain the library accepts. */
int depsync_gemm_chain_check_waits(const depsync_gemm_chain_desc* d, depsync_policy_kind kind,
                                   const depsync_policy_params* params, int n_cu, int64_t* uncovered);
int depsync_conv_chain_n_check_waits(const depsync_conv_chain_n_desc* d, depsync_policy_kind kind,
                                     const depsync_policy_params* params, int n_cu, int64_t* uncovered);

/* ---- copy -> copy chain: what the synchronisation itself costs (Section V, overhead of
 * synchronisation: tile i of the consumer depends on tile i of the producer and the kernels
 * only move bytes) ------------------------------------------------------------------------ */
typedef struct depsync_copy_chain_desc {
    const void* src;      /* device, 16-byte aligned, `bytes` long; read only                 */
    void* mid;            /* device, 128-byte aligned, `bytes` long; written by stage 0        */
    void* dst;            /* device, 16-byte aligned, `bytes` long; written by stage 1         */
    uint64_t bytes;       /* > 0, multiple of 16                                               */
    uint32_t tile_bytes;  /* bytes one workgroup copies per tile: multiple of 4096; 0 = 65536  */
} depsync_copy_chain_desc;

/* dst = mid = src, as two dependent stages of ceil(bytes / tile_bytes) tiles each, with the
 * same dispatch, post and wait as the GeMM and conv chains and the same launch modes.
 * TILESYNC: consumer tile i waits for producer tile i (one semaphore per tile, at most 65536
 * tiles, else DEPSYNC_ENOMEM); ROWSYNC: one semaphore that every producer tile posts to, so
 * the consumer tiles start when the whole producer stage is done; STRIDEDSYNC:
 * DEPSYNC_ENOTIMPL.  Buffers are the caller's and must not overlap; asynchronous like the
 * other chains.  DEPSYNC_EINVAL for null or misaligned pointers and bad sizes.              */
int dep_copy_chain(const depsync_copy_chain_desc* d, sync_policy_t* pol, depsync_mode mode,
                   void* stream_producer, void* stream_consumer);
/* Tiles per stage, workgroup slots (CUs x 8) and algorithmic bytes (4 x bytes: each stage
 * reads and writes the buffer once) of the chain; n_cu 0 = the current device.              */
int depsync_copy_chain_plan(const depsync_copy_chain_desc* d, const sync_policy_t* pol, int n_cu,
                            depsync_plan_info* out);

/* ---- host mirrors of the device index arithmetic (Fig. 4b; Section II-A) -------------- */

/* Linear position of tile (x,y) in row-major order: y*grid_x + x.                         */
int depsync_row_major(int tile_x, int tile_y, int grid_x, int grid_y);
/* Semaphore index of producer tile (x,y); stride is used by STRIDEDSYNC only.             */
int depsync_policy_sem(depsync_policy_kind kind, int tile_x, int tile_y, int grid_x,
                       int grid_y, int stride);
/* Value the semaphore holds when everything mapped to it has posted once.                 */
int depsync_policy_value(depsync_policy_kind kind, int grid_x, int grid_y, int stride);
/* waves = ceil(tiles / (occupancy * n_cu)); *utilization = tiles / (waves * occupancy * n_cu). */
int depsync_wave_model(int n_tiles, int occupancy, int n_cu, int* waves, double* utilization);
/* Number of semaphore waits a GeMM chain performs under a policy when every consumer tile
 * reads full producer rows (Section III-E).                                                */
int depsync_sync_count(depsync_policy_kind kind, int prod_grid_x, int prod_grid_y,
                       int cons_grid_x, int cons_grid_y, int prod_rows_per_cons_row);

/* The planner's schedule model: makespan of gx1*gy1 producer tiles of duration d1 followed by
 * gx2*gy2 consumer tiles of duration d2 on `slots` workgroup slots, row-major issue order;
 * consumer row y reads producer rows [y*r - halo, (y+1)*r - 1 + halo] with r = ceil(gy1/gy2).
 * stream_sync != 0 models the kernel-boundary barrier (Fig. 1b), 0 the per-tile waits (Fig. 1c). */
double depsync_simulate_chain(int slots, int gx1, int gy1, double d1, int gx2, int gy2, double d2,
                              int halo, int stream_sync);

/* ---- misc ------------------------------------------------------------------------------ */
const char* depsync_strerror(int status);
/* Last HIP error code seen by this thread's failing call (0 if none).                      */
int depsync_last_hip_error(void);
/* Rows and columns of a depsync_tile id; DEPSYNC_EINVAL for AUTO or unknown ids.           */
int depsync_tile_shape(int tile, int* rows, int* cols);
/* Measurement aid, not part of the method: runs a loop of nothing but bf16 MFMAs
 * (v_mfma_f32_32x32x16_bf16 on register operands, two workgroups of four waves per CU) on the
 * current device's null stream for about `milliseconds` (1..2000) and reports what the last
 * launch sustained, in TFLOP/s.  zero_operands != 0: all operand bits zero; else random bf16
 * values with |x| in [1/8, 4).  The difference between the two is the chip's power cap at
 * work: it is the practical ceiling of an MFMA-bound kernel on such data.  Allocates and frees
 * 1 MiB + 4 bytes per thread of device memory; synchronises.  DEPSYNC_EINVAL / DEPSYNC_EHIP.     */
int depsync_mfma_calibration(int zero_operands, int milliseconds, double* tflops);
/* CU count and shader clock (kHz) of the current device.                                   */
int depsync_device_info(int* n_cu, int* clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* DEPSYNC_H */
