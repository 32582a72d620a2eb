// Plain-data kernel arguments shared by the host launcher and the device code of the chain
// kernels.  A chain has up to four stages (producer, optional middle stages, consumer); each
// stage after the first has one dependency on the stage before it (Section III-A).
#pragma once
#include <stdint.h>

namespace depsync {

// How a stage addresses its A operand (rows of the implicit GeMM).
enum AMode : uint32_t { A_DENSE = 0, A_CONV3X3 = 1, A_COPY = 2 };   // A_COPY: the stage moves bytes (copy chain)
// How a stage maps rows of its B-operand tile to rows of the weight array.
enum BMode : uint32_t { B_DENSE = 0, B_GATE_UP = 1 };
// Epilogue applied to the fp32 accumulators before rounding to 16 bits.
enum Act : uint32_t { ACT_NONE = 0, ACT_GELU = 1, ACT_RELU = 2, ACT_SWIGLU = 3 };
// What a stage computes.
enum StageOp : uint32_t { OP_GEMM = 0, OP_ATTN = 1 };

// Dependency of a stage on the previous stage's output (its A operand).
enum DepKind : uint32_t {
    DEP_NONE = 0,
    DEP_ROW = 1,          // RowSync: wait once for every producer row tile this tile reads
    DEP_TILE = 2,         // TileSync: wait per producer column tile as the K loop reaches it
    DEP_STRIDED = 3,      // StridedSync on a GeMM: like TILE, semaphore shared at a stride
    DEP_CONV_ROW = 4,     // conv, RowSync: all halo row tiles up front
    DEP_CONV_TAPROW = 5,  // conv, StridedSync: per filter row r, the row tiles shifted by (r-1)*W
    DEP_CONV_TILE = 6,    // conv, TileSync: per (filter row, producer channel tile)
    DEP_ATTN_QKV = 7,     // attention stage on the QKV GeMM
    DEP_ATTN_OUT = 8      // output GeMM on the attention stage
};

struct StageDesc {
    const void* A;      // [M x K] rows of lda elements (conv: NHWC input)
    const void* B;      // [N x K] rows of ldb elements (K contiguous)
    void* C;            // [M x N] rows of ldc elements
    uint32_t M, N, K;   // N = output columns (B_GATE_UP: B has 2N rows)
    uint32_t lda, ldb, ldc;
    // B addressing in bytes: row n, K step kt (64 elements) at n * b_row_bytes + kt * b_kstep_bytes.
    // Row-major [N x K]: (2 * ldb, 128).  K-blocked [K/64][N][64]: (128, 128 * rows of B).
    uint32_t b_row_bytes, b_kstep_bytes;
    uint32_t grid_x, grid_y;   // column tiles, row tiles
    uint32_t queue_by_col;     // dispatch queue of tile (x,y): x mod 8 if set, else (y*grid_x + x) mod 8
    // split-K: each output tile is computed by `ksplit` workgroups over equal K ranges; they leave
    // fp32 partial tiles in `partials` and count in `arrive`, and the last one to arrive adds the
    // partials in K order, applies the epilogue and posts.  The dispatch sees grid_y * ksplit rows.
    uint32_t ksplit;
    float* partials;           // [tile][ksplit][TM*TN] fp32, fragment order
    uint32_t* arrive;          // one counter per tile (SYNC_WORD_STRIDE words apart), zero between chains
    uint32_t op, amode, bmode, act;
    // conv geometry (A_CONV3X3): image height, width, input channels
    uint32_t H, W, Cin;
    const void* zero_page;     // >= 256 zero bytes, source for padded taps
    // attention (OP_ATTN): A = QKV, C = T
    uint32_t batch, seq, heads, head_dim;
    // keys and values of earlier tokens (token generation, Fig. 2b): [batch][cached] rows of ld_cache
    // elements, head h in columns h*head_dim..; attended to before the new tokens' own keys
    const void* kcache;
    const void* vcache;
    uint32_t cached, ld_cache;
    // dependency on the previous stage
    uint32_t dep_kind;
    uint32_t* sems;            // semaphores this stage WAITS on (posted by the previous stage)
    uint32_t sem_target_base;  // semaphore value before this launch's posts
    uint32_t sem_value;        // posts per semaphore per launch
    uint32_t prod_tm;          // producer tile rows
    uint32_t prod_tn;          // producer tile columns of ITS OUTPUT (= K range per tile here)
    uint32_t prod_grid_x, prod_grid_y;
    uint32_t stride;           // DEP_STRIDED: semaphores per producer row
    // posting (this stage as a producer)
    uint32_t post_kind;        // DEP_NONE if nobody waits on this stage, else the consumer's kind
    uint32_t* post_sems;
    uint32_t post_stride;
};

struct StatusBlock {
    int32_t timed_out;
    int32_t first_timeout;
    uint32_t posts;
    uint32_t waits;
    uint32_t polling_waits;
    uint32_t pad[3];
};

// One record per tile, written when DEPSYNC_FLAG_TRACE is set (times in 10 ns ticks of the
// constant 100 MHz counter).
struct TraceRec {
    uint32_t rel;        // first_ticket[stage] + row-major tile index
    uint32_t where;      // stage | xcc << 8 | cu << 16 | se << 24
    uint32_t tx, ty;
    uint64_t t_enter;    // workgroup started
    uint64_t t_start;    // tile drawn
    uint64_t t_ready;    // first dependency satisfied (== t_start for tiles without one)
    uint64_t t_end;      // stores and post done
};

// Every dispatch counter and every semaphore has a 128-byte line of the workspace to itself:
// hundreds of waves poll semaphores while others draw tiles, and words that share a line (or
// a memory channel) make those requests queue up behind each other.
constexpr uint32_t SYNC_WORD_STRIDE = 32;   // in 32-bit words

struct ChainArgs {
    StageDesc st[4];
    uint32_t n_stages;
    uint32_t first_ticket[5];   // stage s owns tickets [first_ticket[s], first_ticket[s+1])
    uint32_t* ticket;           // dispatch counters: [stage][XCD queue], 4 x 8
    uint32_t epoch;             // chains run on this workspace since its last reset
    uint32_t queue_epoch;       // those of them that drew their tiles from the dispatch queues
    uint32_t block_offset;      // HW order / PLAIN: ticket of this launch's block 0
    uint32_t stage_lo, stage_hi; // stages the workgroups of this launch may draw tiles of
    uint32_t draw_cas;          // this launch may run late, into a later chain: it draws with compare-and-swap
    uint32_t flags;             // DEPSYNC_FLAG_*
    uint32_t spin_limit;
    uint32_t delay_tile, delay_iters;
    StatusBlock* status;
    TraceRec* trace;            // trace_cap records, or nullptr
    uint32_t trace_cap;
};

}  // namespace depsync
