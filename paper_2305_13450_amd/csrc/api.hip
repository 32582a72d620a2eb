// C-ABI layer: policy objects, chain planning, workspace/epoch management and the two-stream
// launch (Sections III-A and III-D of the paper; declarations in include/depsync.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <cstdint>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/depsync.h"
#include "chain_args.h"
#include "dep_map.hpp"
#include "host_model.h"
#include "launch.h"

using namespace depsync;

namespace {

thread_local int g_last_hip_error = 0;

// Workspace layout in 32-bit words.
constexpr uint32_t WS_TICKET = 0;        // 4 stages x 8 dispatch counters, one per 128-byte line
constexpr uint32_t WS_TICKET_WORDS = 32 * SYNC_WORD_STRIDE;
constexpr uint32_t WS_STATUS = WS_TICKET_WORDS;          // StatusBlock, 8 words
constexpr uint32_t WS_ZERO_PAGE = WS_STATUS + 64;        // 64 words = 256 zero bytes (never written after init)
constexpr uint32_t WS_SEMS = 2048;                       // one semaphore per 128-byte line
static_assert(WS_ZERO_PAGE + 64 <= WS_SEMS && WS_SEMS % SYNC_WORD_STRIDE == 0, "counters, status and zero page end before the semaphores");

// What follows the fixed part differs between a policy's own workspace (hipMalloc'ed by
// sync_policy_create) and the smaller one inside the library's static device array.
struct WsLayout {
    uint32_t max_sems;      // semaphores, from word WS_SEMS on
    uint32_t trace;         // word offset of the trace records
    uint32_t trace_cap;     // records (0: tracing unavailable)
    uint32_t arrive;        // word offset of the split-K arrival counters, one 128-byte line each
    uint32_t max_arrive;
    uint32_t words;         // total size in 32-bit words
};
constexpr WsLayout make_layout(uint32_t max_sems, uint32_t trace_cap, uint32_t max_arrive) {
    WsLayout l{};
    l.max_sems = max_sems;
    l.trace = WS_SEMS + max_sems * SYNC_WORD_STRIDE;
    l.trace_cap = trace_cap;
    l.arrive = l.trace + trace_cap * (uint32_t)(sizeof(TraceRec) / 4);
    l.max_arrive = max_arrive;
    l.words = l.arrive + max_arrive * SYNC_WORD_STRIDE;
    return l;
}
constexpr WsLayout HEAP_LAYOUT = make_layout(1u << 16, 8192, 1u << 15);

// The allocation-free entry point's workspace: a fixed array in device memory (one copy per GPU
// that loads the library, held until the process ends).  1.5 MiB of counters, semaphores and
// arrival counters, then 128 MiB for split-K partial tiles.
constexpr WsLayout STATIC_LAYOUT = make_layout(8192, 0, 4096);
constexpr size_t STATIC_PARTIAL_FLOATS = 32u << 20;
static_assert(STATIC_LAYOUT.words % 64 == 0, "the partial tiles start on a 256-byte boundary");
constexpr size_t STATIC_WORDS = (size_t)STATIC_LAYOUT.words + STATIC_PARTIAL_FLOATS;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return DEPSYNC_EHIP;
}
#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) return hip_fail(e__);   \
    } while (0)

}  // namespace

struct sync_policy {
    int kind;
    depsync_policy_params params;
    int device;
    uint32_t* ws;
    hipStream_t own_stream;    // second stream when the caller gives none
    hipStream_t third_stream;  // third stage of a chain in FINE mode
    hipStream_t fourth_stream; // fourth stage
    hipStream_t last_side;     // the caller's second stream of the last two-stream chain, if it gave one
    hipEvent_t ev_fork;
    hipEvent_t ev_side;        // used to order the side streams before a reset of the workspace
    bool side_used;            // a two-stream chain has been launched since the last reset
    // epoch state: semaphores and the dispatch counters only ever grow between resets
    uint64_t geom_sig;
    uint32_t epoch;
    uint32_t queue_epoch;      // chains that drew their tiles from the dispatch queues since the last reset
    int force_order;       // autotuner only: -1 none, 0 dispatch queues, 1 hardware order
    uint32_t launches;
    float* scratch;        // split-K partial tiles, grown on demand
    size_t scratch_floats;
    uint32_t sems_dirty;   // semaphores that may be non-zero (largest count used since they were last cleared)
    bool need_reset;
    WsLayout lay;          // where things are in ws
    bool fixed_scratch;    // ws and scratch are parts of the static device array: never (re)allocated
};

namespace {

struct Plan {
    int tile[4];
    int n_stages;
    uint32_t grid_x[4], grid_y[4], n_tiles[4];
    uint32_t dep_kind[4];      // dependency of stage s on stage s-1
    uint32_t sem_off[4];       // offset of that dependency's semaphores inside the sem area
    uint32_t sem_count[4];
    uint32_t sem_value[4];
    uint32_t stride[4];
    uint32_t out_tm[4], out_tn[4];   // rows / columns of its own output one tile of stage s covers
    uint32_t ksplit[4];              // workgroups per output tile (split along K)
    uint32_t arrive_off[4];          // first arrival counter of the stage
    size_t partial_off[4];           // first float of the stage's partial tiles
    size_t partial_floats;           // scratch the chain needs
    uint32_t n_arrive;               // arrival counters the chain needs
    uint32_t part_floats[4];         // floats one part of a split tile of the stage leaves in the scratch buffer (0: rows x columns of its tile)
    uint32_t n_sems;
    int slots;                       // workgroups of the first stage's tile shape that fit on the chip
    int stage_slots[4];              // ... of each stage's own shape (they differ when producer and consumer tiles do)
    double flops, bytes;
    uint32_t amode;
    int dtype;
    int order_pref;                  // tile order the autotuner found faster for one dispatch: -1 none, 0 queues, 1 block index
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
uint32_t cdiv(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

int device_cus(int n_cu) {
    if (n_cu > 0) return n_cu;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    return cus;
}

// Relative time per flop of the macro-tile shapes on a fully occupied CU, from measurements of
// the GPT-3 and LLaMA MLP chains at M = 1 .. 2048 on MI355X (128x192 = 1): smaller tiles read more
// LDS and L2 bytes per flop.  With these factors the model picks the tile measured fastest on all
// ten of those chains.
double tile_cost_factor(int tile, bool conv) {
    if (conv) {
        // the implicit-GeMM gather of A (a row of pixels per DMA row, taps that re-read their
        // neighbours' rows) moves the order: measured on the VGG pairs at batch 16
        switch (tile) {
            case DEPSYNC_TILE_256x128: return 1.25;
            case DEPSYNC_TILE_128x256: return 1.12;
            case DEPSYNC_TILE_128x128: return 1.08;
            case DEPSYNC_TILE_64x128: return 1.3;
            case DEPSYNC_TILE_128x192_DEEP: return 1.3;
            case DEPSYNC_TILE_64x64_DEEP: return 5.0;
            case DEPSYNC_TILE_256x192: return 1.18;
            default: break;
        }
    }
    switch (tile) {
        case DEPSYNC_TILE_256x256: return 1.30;   // its synchronised variant spills registers around the tile loop
        case DEPSYNC_TILE_256x128: return 1.04;
        case DEPSYNC_TILE_128x256: return 1.10;
        case DEPSYNC_TILE_128x128: return 1.20;
        case DEPSYNC_TILE_64x128: return 1.6;
        case DEPSYNC_TILE_64x64: return 2.3;
        case DEPSYNC_TILE_256x192: return 0.93;   // one workgroup per CU, three stages of A: ahead once its tiles fill the chip
        case DEPSYNC_TILE_128x192: return 1.00;
        case DEPSYNC_TILE_256x64: return 1.3;
        case DEPSYNC_TILE_64x64_DEEP: return 4.0;   // one workgroup per CU: only ever worth it when tiles are few
        case DEPSYNC_TILE_64x192: return 2.0;       // likewise
        case DEPSYNC_TILE_128x192_DEEP: return 1.10;   // one workgroup per CU, 4 stages: ahead of 128x192 only
        case DEPSYNC_TILE_128x128_DEEP: return 1.45;   // where that tile would have to split along K
        default: return 2.4;
    }
}

// Tiles found fastest by depsync_*_chain_autotune, per chain shape (and policy kind, which
// changes what overlaps).  Looked up before the model below when the caller leaves the tile
// to the library.
struct TuneKey {
    int64_t v[12];
    bool operator<(const TuneKey& o) const { return std::lexicographical_compare(v, v + 12, o.v, o.v + 12); }
};
std::map<TuneKey, int> g_tuned;
std::mutex g_tuned_mutex;

// `kind`: the policy kind the entry is for; -2 for the entry that remembers the best kind of a shape.
TuneKey tune_key(const depsync_gemm_chain_desc* d, int kind) {
    return TuneKey{{d->w_layout ? 2 : 0, d->M, d->K1, d->N1, d->N2, d->dtype, d->mid, kind, d->heads, d->seq, d->cached, 0}};
}
TuneKey tune_key(const depsync_conv_chain_n_desc* d, int kind) {
    if (d->n == 2) return TuneKey{{1, d->B, d->H, d->W, d->C, d->K[0], d->K[1], d->dtype, kind, 0, 0, 0}};
    return TuneKey{{3, d->B, d->H, d->W, d->C, d->K[0], d->K[1], d->dtype, kind, d->n, d->K[2], d->n > 3 ? d->K[3] : 0}};
}
depsync_conv_chain_n_desc as_chain_n(const depsync_conv_chain_desc& d);
TuneKey tune_key(const depsync_conv_chain_desc* d, int kind) {
    const depsync_conv_chain_n_desc c = as_chain_n(*d);
    return tune_key(&c, kind);
}
// The policy kind a chain runs under: the policy's own, or for DEPSYNC_AUTOSYNC the one
// depsync_*_chain_autotune_policy measured fastest for the chain's shape, else `fallback`.
int tuned_tile(const TuneKey& k);
template <class Desc>
int effective_kind(const Desc* d, const sync_policy* pol, int fallback) {
    if (!pol) return fallback;
    if (pol->kind != DEPSYNC_AUTOSYNC) return pol->kind;
    const int v = tuned_tile(tune_key(d, -2));
    return v ? v - 1 : fallback;
}
// Rule of thumb where nothing was measured (Section V-C): per-tile waits up to 256 rows, per-row
// waits beyond; the attention chain waits on strided groups of tiles.
int default_kind(const depsync_gemm_chain_desc* d) {
    if (d->mid == DEPSYNC_MID_CAUSAL_ATTN) return DEPSYNC_STRIDEDSYNC;
    return d->M <= 256 ? DEPSYNC_TILESYNC : DEPSYNC_ROWSYNC;
}
int tuned_tile(const TuneKey& k) {
    std::lock_guard<std::mutex> g(g_tuned_mutex);
    auto it = g_tuned.find(k);
    return it == g_tuned.end() ? 0 : it->second;
}

uint32_t choose_split(const sync_policy* pol, bool tuned_off, uint32_t tiles, uint32_t slots, uint32_t kt, uint32_t seg);

// Pick one macro-tile for both stages by simulating the fine-grained schedule of the chain
// on `slots` workgroup slots for every candidate shape (host_model.h).  A stage that would leave
// slots idle is modelled as the planner will run it: split along K into S parts, each costing
// 1/S of the tile plus 15 % per further part for the partial tiles and the workgroup that sums them.
int choose_tile(uint32_t M, uint32_t n_out1, uint32_t K1, uint32_t N2, uint32_t K2, bool gate_up,
                int n_cu, int rows_halo_tiles) {
    // The simulation walks every tile of every candidate shape (a millisecond of host time for
    // the largest conv pairs, which every launch with TILE_AUTO would pay): remember the answer.
    using Key = std::array<uint64_t, 4>;
    static std::map<Key, int> memo;
    static std::mutex memo_mutex;
    const Key key = {((uint64_t)M << 32) | n_out1, ((uint64_t)K1 << 32) | N2,
                     ((uint64_t)K2 << 32) | (uint32_t)n_cu, ((uint64_t)(uint32_t)rows_halo_tiles << 1) | (uint64_t)gate_up};
    {
        std::lock_guard<std::mutex> lock(memo_mutex);
        const auto it = memo.find(key);
        if (it != memo.end()) return it->second;
    }
    int best = 0;
    double best_t = 0;
    for (int t = 1; t < DEPSYNC_TILE__COUNT; ++t) {
        const TileShape* ts = tile_shape(t);
        if (gate_up && (ts->wave_cols % 64 || (ts->cols / 2) % 64)) continue;
        const uint32_t tn1 = gate_up ? ts->cols / 2 : ts->cols;
        const uint32_t gy = cdiv(M, ts->rows);
        const uint32_t gx1 = cdiv(n_out1, tn1), gx2 = cdiv(N2, ts->cols);
        const double f = tile_cost_factor(t, rows_halo_tiles > 0);
        // `occupancy` workgroups share a CU's matrix units, so each runs at 1/occupancy of its rate
        const uint32_t slots = (uint32_t)(n_cu * ts->occupancy);
        const uint32_t s1 = choose_split(nullptr, false, gx1 * gy, slots, K1 / 64, 1);
        const uint32_t s2 = choose_split(nullptr, false, gx2 * gy, slots, K2 / 64, 1);
        const double d1 = f * (double)ts->rows * ts->cols * K1 * ts->occupancy / s1 * (1.0 + 0.15 * (s1 - 1));
        const double d2 = f * (double)ts->rows * ts->cols * K2 * ts->occupancy / s2 * (1.0 + 0.15 * (s2 - 1));
        const double tm = simulate_chain((int)slots, gx1 * s1, gy, d1, gx2 * s2, gy, d2, rows_halo_tiles,
                                         /*stream_sync=*/false);
        if (best == 0 || tm < best_t) { best = t; best_t = tm; }
    }
    std::lock_guard<std::mutex> lock(memo_mutex);
    memo[key] = best;
    return best;
}

int policy_dep_kind_gemm(int kind) {
    switch (kind) {
        case DEPSYNC_ROWSYNC: return DEP_ROW;
        case DEPSYNC_TILESYNC: return DEP_TILE;
        default: return DEP_STRIDED;
    }
}
int policy_dep_kind_conv(int kind) {
    switch (kind) {
        case DEPSYNC_ROWSYNC: return DEP_CONV_ROW;
        case DEPSYNC_TILESYNC: return DEP_CONV_TILE;
        default: return DEP_CONV_TAPROW;
    }
}

// Workgroups per output tile for a stage with `tiles` output tiles and `kt` K steps whose
// dependency segments start every `seg` steps: split when the stage would leave at least half
// of the slots idle, as far as one wave of slots allows, keeping every part at least 16 steps
// long (the partial tiles and the arrival count cost about 10 us per stage) and starting on a
// segment boundary.  `tuned_off`: the autotuner found this chain faster without.
// (Splitting a stage of more tiles than slots so that it ends in a fuller last round was measured
// and is not done: LLaMA MLP at 2048 tokens, 344 producer tiles on 256 slots as 688 halves, three
// rounds of 64 steps instead of two of 128: 275 -> 283 us; the 88 MB of partial tiles and the
// finishing workgroups cost more than the shorter last round gains.)
uint32_t choose_split(const sync_policy* pol, bool tuned_off, uint32_t tiles, uint32_t slots, uint32_t kt, uint32_t seg) {
    const uint32_t want = pol ? pol->params.ksplit : 0;
    if (want == 1 || seg == 0 || (want == 0 && tuned_off)) return 1;
    static const uint32_t cand[] = {8, 6, 4, 3, 2};
    for (uint32_t S : cand) {
        if (kt % S || (kt / S) % seg) continue;
        if (want > 1) { if (S <= want) return S; continue; }
        if (tiles * S <= slots && kt / S >= 16) return S;
    }
    return 1;
}

// Fill in tile counts, arrival counters and partial-tile offsets once grids and splits are known.
int finish_split(Plan& p) {
    uint32_t arr = 0;
    size_t fl = 0;
    for (int s = 0; s < p.n_stages; ++s) {
        const uint32_t real = p.grid_x[s] * p.grid_y[s];
        p.n_tiles[s] = real * p.ksplit[s];
        p.arrive_off[s] = arr;
        p.partial_off[s] = fl;
        if (p.ksplit[s] > 1) {
            const TileShape* ts = tile_shape(p.tile[s]);
            arr += real;
            fl += (size_t)real * p.ksplit[s] * (p.part_floats[s] ? p.part_floats[s] : (uint32_t)(ts->rows * ts->cols));
        }
    }
    p.partial_floats = fl;
    p.n_arrive = arr;
    return DEPSYNC_OK;
}

int plan_gemm(const depsync_gemm_chain_desc* d, const sync_policy* pol, int n_cu, Plan& p) {
    if (!d) return DEPSYNC_EINVAL;
    if (d->M <= 0 || d->K1 <= 0 || d->N1 <= 0 || d->N2 <= 0) return DEPSYNC_EINVAL;
    if (d->dtype != DEPSYNC_BF16 && d->dtype != DEPSYNC_FP16) return DEPSYNC_EINVAL;
    if (d->mid < DEPSYNC_MID_NONE || d->mid > DEPSYNC_MID_CAUSAL_ATTN) return DEPSYNC_EINVAL;
    if (!d->X || !d->W1t || !d->H || !d->W2t || !d->Y) return DEPSYNC_EINVAL;
    if (!aligned16(d->X) || !aligned16(d->W1t) || !aligned16(d->H) || !aligned16(d->W2t) || !aligned16(d->Y))
        return DEPSYNC_EINVAL;
    const bool gate_up = d->mid == DEPSYNC_MID_SWIGLU;
    const bool attn = d->mid == DEPSYNC_MID_CAUSAL_ATTN;
    const uint32_t E = attn ? (uint32_t)d->heads * 128u : 0u;
    if (attn) {
        if (d->head_dim != 128) return d->head_dim > 0 ? DEPSYNC_ENOTIMPL : DEPSYNC_EINVAL;
        if (d->batch <= 0 || d->seq <= 0 || d->heads <= 0) return DEPSYNC_EINVAL;
        if ((int64_t)d->batch * d->seq != d->M || (int64_t)d->N1 != 3ll * E) return DEPSYNC_EINVAL;
        if (!d->T || (reinterpret_cast<uintptr_t>(d->T) & 127u) || d->ldt < (int64_t)E || d->ldt % 64) return DEPSYNC_EINVAL;
        // query blocks must not straddle sequences: whole blocks of 128, or one short block each
        if (d->batch > 1 && d->seq % 128 && d->seq > 128) return DEPSYNC_ENOTIMPL;
        if (d->cached < 0) return DEPSYNC_EINVAL;
        if (d->cached > 0) {
            if (!d->k_cache || !d->v_cache || !aligned16(d->k_cache) || !aligned16(d->v_cache)) return DEPSYNC_EINVAL;
            if (d->ld_cache < (int64_t)E || d->ld_cache % 8) return DEPSYNC_EINVAL;
            if ((uint64_t)d->batch * (uint64_t)d->cached * (uint64_t)d->ld_cache * 2 >= (1ull << 32)) return DEPSYNC_EINVAL;
        }
    }
    const uint32_t K2 = attn ? E : (uint32_t)d->N1;
    if (d->K1 % 64 || K2 % 64) return DEPSYNC_EINVAL;
    if (d->w_layout != DEPSYNC_W_ROWS && d->w_layout != DEPSYNC_W_KBLOCKED) return DEPSYNC_EINVAL;
    const bool wrows = d->w_layout == DEPSYNC_W_ROWS;
    if (d->ldx < d->K1 || (wrows && d->ldw1 < d->K1) || d->ldh < d->N1 || (wrows && d->ldw2 < (int64_t)K2) || d->ldy < d->N2)
        return DEPSYNC_EINVAL;
    if (d->ldx % 8 || (wrows && (d->ldw1 % 8 || d->ldw2 % 8)) || d->ldh % 8 || d->ldy % 8) return DEPSYNC_EINVAL;
    // rows of the intermediate must be whole 128-byte cache lines (see dep_wait in gemm_tile.hpp)
    if (d->ldh % 64 || (reinterpret_cast<uintptr_t>(d->H) & 127u)) return DEPSYNC_EINVAL;
    const uint64_t lim = 1ull << 32;
    const uint64_t w1_rows = gate_up ? 2ull * d->N1 : (uint64_t)d->N1;
    const uint64_t ldw1 = wrows ? (uint64_t)d->ldw1 : (uint64_t)d->K1, ldw2 = wrows ? (uint64_t)d->ldw2 : (uint64_t)K2;
    if ((uint64_t)d->M * d->ldx * 2 >= lim || w1_rows * ldw1 * 2 >= lim || (uint64_t)d->M * d->ldh * 2 >= lim ||
        (uint64_t)d->N2 * ldw2 * 2 >= lim || (uint64_t)d->M * d->ldy * 2 >= lim)
        return DEPSYNC_EINVAL;
    if (d->tile_prod < 0 || d->tile_prod >= DEPSYNC_TILE__COUNT || d->tile_cons < 0 ||
        d->tile_cons >= DEPSYNC_TILE__COUNT)
        return DEPSYNC_EINVAL;
    // Producer and consumer may use different macro-tile shapes (each stage is then a launch of its
    // own kernel: not in one dispatch); the attention chain's three stages share one.
    const bool mixed = d->tile_prod && d->tile_cons && d->tile_prod != d->tile_cons;
    if (mixed && attn) return DEPSYNC_ENOTIMPL;

    const int cus = device_cus(n_cu);
    if (cus <= 0) return DEPSYNC_EHIP;
    int tile = d->tile_prod ? d->tile_prod : d->tile_cons;
    bool tuned_off = false;
    int order_pref = -1;
    if (!tile) {
        const int v = tuned_tile(tune_key(d, pol ? effective_kind(d, pol, default_kind(d)) : -1));
        tile = v & 0xff;
        if (v) { tuned_off = (v & 0x100) != 0; order_pref = (v & 0x200) ? 1 : 0; }
    }
    if (!tile) tile = choose_tile(d->M, d->N1, d->K1, d->N2, K2, gate_up, cus, 0);
    const TileShape* ts = tile_shape(tile);                               // the producer's shape
    const TileShape* tsc = mixed ? tile_shape(d->tile_cons) : ts;         // the consumer's
    if (!ts || !tsc) return DEPSYNC_EINVAL;
    if (gate_up && ts->wave_cols % 64) return DEPSYNC_EINVAL;   // a wave needs whole gate/up pairs of 32-column blocks
    // a K step of the next stage (64 columns of the intermediate) must not straddle two producer
    // tiles: the per-tile waits are issued per producer column tile as the K loop reaches it
    if (gate_up && (ts->cols / 2) % 64) return DEPSYNC_EINVAL;

    std::memset(&p, 0, sizeof(p));
    const int last = attn ? 2 : 1;
    p.n_stages = last + 1;
    p.amode = A_DENSE;
    p.dtype = d->dtype;
    p.order_pref = order_pref;
    for (int s = 0; s < p.n_stages; ++s) { p.tile[s] = tile; p.stage_slots[s] = cus * ts->occupancy; }
    if (mixed) { p.tile[last] = d->tile_cons; p.stage_slots[last] = cus * tsc->occupancy; }
    const uint32_t tn1 = gate_up ? ts->cols / 2 : ts->cols;
    p.grid_y[0] = cdiv(d->M, ts->rows);
    p.grid_y[last] = cdiv(d->M, tsc->rows);
    p.grid_x[0] = cdiv(d->N1, tn1);
    p.grid_x[last] = cdiv(d->N2, tsc->cols);
    p.out_tm[0] = ts->rows; p.out_tn[0] = tn1;
    p.out_tm[last] = tsc->rows; p.out_tn[last] = tsc->cols;
    if (attn) {   // middle stage: one tile per (head, block of 128 query rows)
        p.grid_x[1] = d->heads;
        p.grid_y[1] = (uint32_t)d->batch * cdiv(d->seq, 128);
        p.out_tm[1] = (d->batch > 1 && d->seq < 128) ? (uint32_t)d->seq : 128u;   // rows one attention tile covers
        p.out_tn[1] = 128;
    }
    for (int s = 0; s < p.n_stages; ++s) { p.n_tiles[s] = p.grid_x[s] * p.grid_y[s]; p.ksplit[s] = 1; }

    // dependency of stage s on stage s-1, per policy
    const int kind = effective_kind(d, pol, pol ? default_kind(d) : DEPSYNC_ROWSYNC);
    uint32_t off = 0;
    for (int s = 1; s < p.n_stages; ++s) {
        uint32_t dk = policy_dep_kind_gemm(kind);
        const uint32_t pgx = p.grid_x[s - 1], pgy = p.grid_y[s - 1];
        if (attn && s == 2 && dk == DEP_STRIDED) dk = DEP_TILE;   // "Strided + TileSync" (Section V-C)
        if (attn && s == 1 && dk == DEP_STRIDED && E % p.out_tn[0]) dk = DEP_TILE;
        p.dep_kind[s] = dk;
        p.sem_off[s] = off;
        if (dk == DEP_ROW) {
            p.sem_count[s] = pgy;
            p.sem_value[s] = pgx;
        } else if (dk == DEP_TILE) {
            p.sem_count[s] = pgx * pgy;
            p.sem_value[s] = 1;
        } else {
            uint32_t stride;
            if (attn) {
                stride = E / p.out_tn[0];               // Q, K and V column tiles of a head share a semaphore
            } else {
                stride = pol ? pol->params.stride : 0;
                if (stride == 0) {
                    const uint32_t count = (pol && pol->params.count) ? pol->params.count : 3;
                    if (pgx % count) return DEPSYNC_EINVAL;
                    stride = pgx / count;
                }
            }
            if (stride == 0 || pgx % stride) return DEPSYNC_EINVAL;
            p.stride[s] = stride;
            p.sem_count[s] = pgy * stride;
            p.sem_value[s] = pgx / stride;
        }
        off += p.sem_count[s];
    }
    p.n_sems = off;
    p.slots = cus * ts->occupancy;
    // split along K where a stage is much smaller than the chip (not the prompt-phase attention stage)
    p.ksplit[0] = choose_split(pol, tuned_off, p.n_tiles[0], p.slots, d->K1 / 64, 1);
    if (attn && d->seq == 1) {
        // token generation: the keys of a (head, sequence) pair over up to 8 workgroups, at least 256
        // keys each, as far as one wave of slots allows
        uint32_t ks = std::min<uint32_t>(8u, ((uint32_t)d->cached + 1u) / 256u);
        while (ks > 1 && p.n_tiles[1] * ks > (uint32_t)p.slots) --ks;
        p.ksplit[1] = std::max<uint32_t>(ks, 1u);
        p.part_floats[1] = 130;
    } else if (attn) {
        // prompt phase: a causal tile walks its key blocks one after the other, the last query block
        // of a sequence the most.  Where the stage leaves most of the chip idle its keys are split
        // over up to 8 workgroups of at least 4 key blocks (256 keys) each.  A stage of many tiles is
        // left alone: measured on the GPT-3 shard at 2048 tokens, the parts (which re-read the
        // queries and exchange 65 KB of partial results each) shorten the stage but crowd out the
        // output GeMM's tiles that otherwise run next to the long attention tiles (404 -> 450 us).
        const uint32_t max_blocks = ((uint32_t)d->cached + (uint32_t)d->seq - 1u) / 64u + 1u;
        const uint32_t want = pol ? pol->params.ksplit : 0;
        const bool sparse = 2u * p.n_tiles[1] < (uint32_t)p.slots;
        uint32_t ks = want ? want : ((tuned_off || !sparse) ? 1u : (max_blocks + 3u) / 4u);
        p.ksplit[1] = std::min<uint32_t>(8u, std::max<uint32_t>(ks, 1u));
        p.part_floats[1] = 256 * 64 + 2 * 256;
    }
    {
        const uint32_t dk = p.dep_kind[last];
        const uint32_t seg = (dk == DEP_ROW) ? 1u : p.out_tn[last - 1] / 64;
        p.ksplit[last] = choose_split(pol, tuned_off, p.n_tiles[last], p.stage_slots[last], K2 / 64, seg);
    }
    if (int rc = finish_split(p); rc != DEPSYNC_OK) return rc;
    const double M = d->M, w1c = gate_up ? 2.0 * d->N1 : d->N1;
    p.flops = 2.0 * M * w1c * d->K1 + 2.0 * M * d->N2 * K2;
    p.bytes = 2.0 * (M * d->K1 + w1c * d->K1 + 2.0 * M * d->N1 + (double)d->N2 * K2 + M * d->N2);
    if (attn) {   // causal: each of Q K^T and P V does seq*(seq+1)/2 * d multiply-adds per head and sequence
        p.flops += 2.0 * 2.0 * d->batch * d->heads * 128.0 *
                   (0.5 * (double)d->seq * ((double)d->seq + 1.0) + (double)d->seq * (double)d->cached);
        p.bytes += 2.0 * 2.0 * M * E;   // T written and read once
        p.bytes += 2.0 * 2.0 * (double)d->batch * (double)d->cached * E;   // cached keys and values read once
    }
    return DEPSYNC_OK;
}

// The two-convolution descriptor as a chain of n = 2.
depsync_conv_chain_n_desc as_chain_n(const depsync_conv_chain_desc& d) {
    depsync_conv_chain_n_desc c;
    std::memset(&c, 0, sizeof(c));
    c.B = d.B; c.H = d.H; c.W = d.W; c.C = d.C; c.n = 2;
    c.K[0] = d.K1; c.K[1] = d.K2;
    c.dtype = d.dtype;
    c.in = d.in; c.w[0] = d.w1; c.w[1] = d.w2; c.out[0] = d.mid; c.out[1] = d.out;
    c.tile_prod = d.tile_prod; c.tile_cons = d.tile_cons;
    return c;
}

// Chain of n = 2..4 3x3 convolutions: stage i is conv i, each later stage depends on the one
// before it in the way the policy says (per halo row tile, per filter row, or per filter row
// and channel tile).
int plan_conv_n(const depsync_conv_chain_n_desc* d, const sync_policy* pol, int n_cu, Plan& p) {
    if (!d) return DEPSYNC_EINVAL;
    if (d->n < 2 || d->n > 4) return DEPSYNC_EINVAL;
    if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0) return DEPSYNC_EINVAL;
    if (d->dtype != DEPSYNC_BF16 && d->dtype != DEPSYNC_FP16) return DEPSYNC_EINVAL;
    if (!d->in || !aligned16(d->in) || d->C % 64) return DEPSYNC_EINVAL;
    if (d->H >= 32768 || d->W >= 32768) return DEPSYNC_EINVAL;
    const uint64_t Mpix = (uint64_t)d->B * d->H * d->W;
    const uint64_t lim = 1ull << 32;
    const int n = d->n;
    int cin[4];                                            // input channels of conv i
    for (int i = 0; i < n; ++i) {
        cin[i] = i == 0 ? d->C : d->K[i - 1];
        if (d->K[i] <= 0 || !d->w[i] || !d->out[i] || !aligned16(d->w[i]) || !aligned16(d->out[i])) return DEPSYNC_EINVAL;
        const bool last = i == n - 1;
        if (last ? d->K[i] % 8 : d->K[i] % 64) return DEPSYNC_EINVAL;
        if (!last && (reinterpret_cast<uintptr_t>(d->out[i]) & 127u)) return DEPSYNC_EINVAL;   // whole cache lines per pixel
        if (Mpix * (uint64_t)std::max(cin[i], d->K[i]) * 2 >= lim || 9ull * cin[i] * d->K[i] * 2 >= lim) return DEPSYNC_EINVAL;
    }
    if (d->tile_prod < 0 || d->tile_prod >= DEPSYNC_TILE__COUNT || d->tile_cons < 0 ||
        d->tile_cons >= DEPSYNC_TILE__COUNT)
        return DEPSYNC_EINVAL;
    // differing producer and consumer shapes: chains of two convolutions only (each stage then is a
    // launch of its own kernel)
    const bool mixed = d->tile_prod && d->tile_cons && d->tile_prod != d->tile_cons;
    if (mixed && n != 2) return DEPSYNC_ENOTIMPL;
    const int cus = device_cus(n_cu);
    if (cus <= 0) return DEPSYNC_EHIP;
    const uint32_t M = (uint32_t)Mpix;
    int tile = d->tile_prod ? d->tile_prod : d->tile_cons;
    bool tuned_off = false;
    int order_pref = -1;
    if (!tile) {
        const int v = tuned_tile(tune_key(d, pol ? effective_kind(d, pol, DEPSYNC_STRIDEDSYNC) : -1));
        tile = v & 0xff;
        if (v) { tuned_off = (v & 0x100) != 0; order_pref = (v & 0x200) ? 1 : 0; }
    }
    if (!tile) {
        // halo: a consumer row tile reads W+1 rows beyond each end (modelled on the first two stages)
        tile = choose_tile(M, d->K[0], 9 * d->C, d->K[1], 9 * d->K[0], false, cus, 1);
    }
    if (!tile_shape(tile) || (mixed && !tile_shape(d->tile_cons))) return DEPSYNC_EINVAL;

    std::memset(&p, 0, sizeof(p));
    p.n_stages = n;
    p.amode = A_CONV3X3;
    p.dtype = d->dtype;
    p.order_pref = order_pref;
    const int kind = effective_kind(d, pol, DEPSYNC_STRIDEDSYNC);
    for (int s = 0; s < n; ++s) {
        p.tile[s] = (mixed && s == n - 1) ? d->tile_cons : tile;
        const TileShape* ts = tile_shape(p.tile[s]);
        p.stage_slots[s] = cus * ts->occupancy;
        p.grid_y[s] = cdiv(M, ts->rows);
        p.grid_x[s] = cdiv(d->K[s], ts->cols);
        p.out_tm[s] = ts->rows; p.out_tn[s] = ts->cols;
        p.n_tiles[s] = p.grid_x[s] * p.grid_y[s];
        p.ksplit[s] = 1;
    }
    p.slots = p.stage_slots[0];
    for (int s = 1; s < n; ++s) {
        p.dep_kind[s] = policy_dep_kind_conv(kind);
        p.sem_off[s] = p.n_sems;
        if (p.dep_kind[s] == DEP_CONV_TILE) {
            if (p.out_tn[s - 1] % 64) return DEPSYNC_EINVAL;
            p.sem_count[s] = p.n_tiles[s - 1];
            p.sem_value[s] = 1;
        } else {
            p.sem_count[s] = p.grid_y[s - 1];
            p.sem_value[s] = p.grid_x[s - 1];
        }
        p.n_sems += p.sem_count[s];
    }
    p.ksplit[0] = choose_split(pol, tuned_off, p.n_tiles[0], p.stage_slots[0], 9u * d->C / 64, 1);
    for (int s = 1; s < n; ++s) {
        uint32_t seg = 1;                                   // CONV_ROW: the whole halo is waited for by every part
        // per filter row or per (filter row, channel tile): the wait at a filter row's first tap
        // also covers its other two taps, so parts must be whole filter rows
        if (p.dep_kind[s] != DEP_CONV_ROW) seg = 3u * cin[s] / 64;
        p.ksplit[s] = choose_split(pol, tuned_off, p.n_tiles[s], p.stage_slots[s], 9u * cin[s] / 64, seg);
    }
    if (int rc = finish_split(p); rc != DEPSYNC_OK) return rc;
    const double Md = (double)M;
    p.flops = 0.0;
    p.bytes = 2.0 * Md * d->C;                              // the input once
    for (int i = 0; i < n; ++i) {
        p.flops += 2.0 * Md * d->K[i] * 9.0 * cin[i];
        p.bytes += 2.0 * (9.0 * cin[i] * d->K[i] + (i == n - 1 ? 1.0 : 2.0) * Md * d->K[i]);   // weights; output written (and read)
    }
    return DEPSYNC_OK;
}

int plan_conv(const depsync_conv_chain_desc* d, const sync_policy* pol, int n_cu, Plan& p) {
    if (!d) return DEPSYNC_EINVAL;
    const depsync_conv_chain_n_desc c = as_chain_n(*d);
    return plan_conv_n(&c, pol, n_cu, p);
}

// Copy chain: two stages of ceil(bytes / tile_bytes) tiles, one row of tiles each.
int plan_copy(const depsync_copy_chain_desc* d, const sync_policy* pol, int n_cu, Plan& p) {
    if (!d || !pol) return DEPSYNC_EINVAL;
    if (!d->src || !d->mid || !d->dst || d->bytes == 0 || (d->bytes & 15u)) return DEPSYNC_EINVAL;
    if (!aligned16(d->src) || !aligned16(d->dst) || (reinterpret_cast<uintptr_t>(d->mid) & 127u)) return DEPSYNC_EINVAL;
    const uint32_t tb = d->tile_bytes ? d->tile_bytes : 65536u;
    if (tb % 4096u) return DEPSYNC_EINVAL;
    if (pol->kind == DEPSYNC_STRIDEDSYNC) return DEPSYNC_ENOTIMPL;   // (DEPSYNC_AUTOSYNC: per-tile waits)
    const uint64_t tiles64 = (d->bytes + tb - 1) / tb;
    if (tiles64 > (1u << 20) || (d->bytes >> 4) > 0xffffffffull) return DEPSYNC_EINVAL;
    const uint32_t tiles = (uint32_t)tiles64;
    const int cus = device_cus(n_cu);
    if (cus <= 0) return DEPSYNC_EHIP;
    std::memset(&p, 0, sizeof(p));
    p.n_stages = 2;
    for (int s = 0; s < 2; ++s) {
        p.tile[s] = 0;
        p.grid_x[s] = tiles; p.grid_y[s] = 1; p.n_tiles[s] = tiles;
        p.out_tm[s] = 1; p.out_tn[s] = 1; p.ksplit[s] = 1;
    }
    const bool row = pol->kind == DEPSYNC_ROWSYNC;
    p.dep_kind[1] = row ? DEP_ROW : DEP_TILE;
    p.sem_off[1] = 0;
    p.sem_count[1] = row ? 1u : tiles;
    p.sem_value[1] = row ? tiles : 1u;
    p.n_sems = p.sem_count[1];
    p.slots = cus * 8;                     // 256 threads, no LDS to speak of: eight workgroups per CU
    p.stage_slots[0] = p.stage_slots[1] = p.slots;
    p.flops = 0.0;
    p.bytes = 4.0 * (double)d->bytes;      // each stage reads the buffer once and writes it once
    p.amode = A_COPY;
    p.dtype = 0;
    p.order_pref = 0;
    return DEPSYNC_OK;
}

void fill_plan_info(const Plan& p, depsync_plan_info* o) {
    std::memset(o, 0, sizeof(*o));
    o->tile_prod = p.tile[0];
    o->tile_cons = p.tile[p.n_stages - 1];
    o->tile_mid = p.n_stages >= 3 ? p.tile[1] : 0;
    o->prod_grid_x = p.grid_x[0]; o->prod_grid_y = p.grid_y[0];
    o->cons_grid_x = p.grid_x[p.n_stages - 1]; o->cons_grid_y = p.grid_y[p.n_stages - 1];
    o->n_prod = p.n_tiles[0];
    o->n_cons = p.n_tiles[p.n_stages - 1];
    if (p.n_stages >= 3) {   // four stages: the grid of the second, the tiles of both middle stages
        o->mid_grid_x = p.grid_x[1]; o->mid_grid_y = p.grid_y[1];
        for (int s = 1; s + 1 < p.n_stages; ++s) o->n_mid += p.n_tiles[s];
    }
    o->n_sems = p.n_sems;
    o->slots = p.slots;
    uint32_t total = 0;
    int ws = 0;
    for (int s = 0; s < p.n_stages; ++s) { ws += cdiv(p.n_tiles[s], p.stage_slots[s]); total += p.n_tiles[s]; }
    o->waves_streamsync = ws;
    o->waves_fine = cdiv(total, p.slots);
    o->flops = p.flops;
    o->bytes = p.bytes;
}

uint64_t geom_signature(const Plan& p) {
    uint64_t h = 1469598103934665603ull;
    auto mix = [&](uint64_t v) { h = (h ^ v) * 1099511628211ull; };
    mix(p.n_stages);
    // everything the dispatch queues' lengths and the semaphore targets depend on
    for (int s = 0; s < p.n_stages; ++s) { mix(p.grid_x[s]); mix(p.grid_y[s]); mix(p.ksplit[s]); mix(p.sem_count[s]); mix(p.sem_value[s]); mix(p.dep_kind[s]); }
    return h;
}

// Two-stream launches are not joined back (see launch_chain), so a side stream's launch may still
// be winding down when a later chain starts.  That is harmless while the workspace keeps its
// meaning (such a launch draws with compare-and-swap and finds its epoch's queues handed out), but
// before the workspace is re-zeroed every side launch must have ended: order the side streams'
// work enqueued so far before whatever `stream` runs next.
int settle_side_launches(sync_policy* pol, hipStream_t stream) {
    if (!pol->side_used || !pol->ev_side) return DEPSYNC_OK;
    hipStream_t side[4] = {pol->own_stream, pol->third_stream, pol->fourth_stream, pol->last_side};
    for (int i = 0; i < 4; ++i) {
        hipStream_t st = side[i];
        if (!st) continue;
        const hipError_t e = hipEventRecord(pol->ev_side, st);
        if (e != hipSuccess) {
            // a caller's stream that no longer exists has nothing left to order
            if (i == 3) { (void)hipGetLastError(); continue; }
            return hip_fail(e);
        }
        HIP_TRY(hipStreamWaitEvent(stream, pol->ev_side, 0));
    }
    pol->last_side = nullptr;
    pol->side_used = false;
    return DEPSYNC_OK;
}

// Make semaphores/counter consistent for a launch with geometry `p`; returns the epoch.
int prepare_epoch(sync_policy* pol, const Plan& p, hipStream_t stream, uint32_t* epoch_out) {
    uint32_t total = 0, vmax = 1;
    for (int s = 0; s < p.n_stages; ++s) { total += p.n_tiles[s]; vmax = std::max(vmax, p.sem_value[s]); }
    const uint64_t sig = geom_signature(p);
    const uint64_t next = (uint64_t)(pol->epoch + 2) * std::max(total, vmax);
    if (pol->need_reset || sig != pol->geom_sig || next >= (1ull << 31)) {
        // zero the dispatch counters and every semaphore the previous geometry may have touched,
        // once no launch of an earlier chain can still be drawing from them
        if (int rc = settle_side_launches(pol, stream); rc != DEPSYNC_OK) return rc;
        hipError_t e = launch_fill_u32(pol->ws + WS_TICKET, 0u, WS_TICKET_WORDS, stream);
        if (e == hipSuccess) e = launch_fill_u32(pol->ws + WS_SEMS, 0u, pol->sems_dirty * SYNC_WORD_STRIDE, stream);
        if (e == hipSuccess && pol->need_reset) {
            // a chain gave up a wait: tiles it skipped may have left arrival counts behind, and
            // the status block still shows its time-out
            e = launch_fill_u32(pol->ws + pol->lay.arrive, 0u, pol->lay.max_arrive * SYNC_WORD_STRIDE, stream);
            if (e == hipSuccess) e = launch_fill_u32(pol->ws + WS_STATUS, 0u, 8, stream);
            if (e == hipSuccess) e = launch_fill_u32(pol->ws + WS_STATUS + 1, 0xffffffffu, 1, stream);   // first_timeout = -1
        }
        if (e != hipSuccess) return hip_fail(e);
        pol->epoch = 0;
        pol->queue_epoch = 0;
        pol->geom_sig = sig;
        pol->need_reset = false;
        pol->sems_dirty = 0;
    }
    pol->sems_dirty = std::max(pol->sems_dirty, p.n_sems);
    *epoch_out = pol->epoch;
    return DEPSYNC_OK;
}

// Does the chain fit the policy's workspace?
int check_limits(const sync_policy* pol, const Plan& p) {
    const WsLayout& l = pol ? pol->lay : HEAP_LAYOUT;
    const bool fixed = pol && pol->fixed_scratch;
    if (p.n_sems > l.max_sems || p.n_arrive > l.max_arrive) return fixed ? DEPSYNC_ELIMIT : DEPSYNC_ENOMEM;
    if (fixed && p.partial_floats > pol->scratch_floats) return DEPSYNC_ELIMIT;
    return DEPSYNC_OK;
}

// Make the policy's scratch buffer large enough for the chain's split-K partial tiles.
int ensure_scratch(sync_policy* pol, const Plan& p) {
    if (p.partial_floats <= pol->scratch_floats) return DEPSYNC_OK;
    if (pol->fixed_scratch) return DEPSYNC_ELIMIT;   // a fixed part of the static array: never grown
    HIP_TRY(hipDeviceSynchronize());               // earlier chains may still use the old buffer
    if (pol->scratch) (void)hipFree(pol->scratch);
    pol->scratch = nullptr;
    pol->scratch_floats = 0;
    float* buf = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&buf), p.partial_floats * sizeof(float));
    if (e != hipSuccess) return e == hipErrorOutOfMemory ? DEPSYNC_ENOMEM : hip_fail(e);
    pol->scratch = buf;
    pol->scratch_floats = p.partial_floats;
    return DEPSYNC_OK;
}

// Grid, split and dependency geometry of stage s (everything the index arithmetic of
// dep_map.hpp reads); pointers and epoch-dependent values are filled in by fill_common.
void fill_stage_geometry(StageDesc& st, const Plan& p, int s) {
    st.grid_x = p.grid_x[s];
    st.grid_y = p.grid_y[s];
    st.queue_by_col = p.grid_x[s] >= 8 ? 1u : 0u;
    st.ksplit = p.ksplit[s];
    st.dep_kind = s > 0 ? p.dep_kind[s] : DEP_NONE;
    if (s > 0) {
        st.sem_value = p.sem_value[s];
        st.prod_tm = p.out_tm[s - 1];
        st.prod_tn = p.out_tn[s - 1];
        st.prod_grid_x = p.grid_x[s - 1];
        st.prod_grid_y = p.grid_y[s - 1];
        st.stride = p.stride[s];
    }
    if (s + 1 < p.n_stages) {
        st.post_kind = p.dep_kind[s + 1];
        st.post_stride = p.stride[s + 1];
    } else {
        st.post_kind = DEP_NONE;
    }
}

void fill_common(ChainArgs& a, sync_policy* pol, const Plan& p, uint32_t epoch) {
    a.n_stages = p.n_stages;
    uint32_t t = 0;
    for (int s = 0; s < 5; ++s) {
        a.first_ticket[s] = t;
        if (s < p.n_stages) t += p.n_tiles[s];
    }
    a.ticket = pol->ws + WS_TICKET;
    a.epoch = epoch;
    a.queue_epoch = pol->queue_epoch;
    a.block_offset = 0;
    a.flags = pol->params.flags;
    // 0 selects a generous default bound (seconds), so that a dependency that can never be
    // satisfied ends in DEPSYNC_ETIMEOUT instead of a hung GPU; 0xffffffff waits without bound
    a.spin_limit = pol->params.spin_limit == 0 ? (1u << 22)
                   : pol->params.spin_limit == 0xffffffffu ? 0u : pol->params.spin_limit;
    a.delay_tile = pol->params.delay_tile;
    a.delay_iters = pol->params.delay_iters;
    a.status = reinterpret_cast<StatusBlock*>(pol->ws + WS_STATUS);
    a.trace = pol->lay.trace_cap ? reinterpret_cast<TraceRec*>(pol->ws + pol->lay.trace) : nullptr;
    a.trace_cap = pol->lay.trace_cap;
    for (int s = 0; s < p.n_stages; ++s) {
        StageDesc& st = a.st[s];
        fill_stage_geometry(st, p, s);
        st.partials = pol->scratch ? pol->scratch + p.partial_off[s] : nullptr;
        st.arrive = pol->ws + pol->lay.arrive + p.arrive_off[s] * SYNC_WORD_STRIDE;
        st.zero_page = pol->ws + WS_ZERO_PAGE;
        if (s > 0) {
            st.sems = pol->ws + WS_SEMS + p.sem_off[s] * SYNC_WORD_STRIDE;
            st.sem_target_base = epoch * p.sem_value[s];
        }
        if (s + 1 < p.n_stages) st.post_sems = pol->ws + WS_SEMS + p.sem_off[s + 1] * SYNC_WORD_STRIDE;
    }
}

int launch_chain(sync_policy* pol, const Plan& p, ChainArgs& a, depsync_mode mode, void* sp_, void* sc_) {
    hipStream_t sp = static_cast<hipStream_t>(sp_);
    const bool sync = mode != DEPSYNC_MODE_PLAIN;
    uint32_t total = 0;
    for (int s = 0; s < p.n_stages; ++s) total += p.n_tiles[s];
    // Tile order of a one-dispatch launch.  Drawn from the dispatch queues, producer tiles are
    // always handed out before consumer tiles, whatever order the hardware starts workgroups in
    // (Section III-B).  Named by the block index (Section IV-C, "avoid custom tile order"), a chain
    // of more tiles than resident workgroups progresses only if every XCD starts the workgroups of
    // a dispatch in index order, which HIP does not promise; so the library chooses that order on
    // its own only when every tile's workgroup is resident at once (any start order is then safe),
    // or when the autotuner measured it for such a chain; beyond that it is the caller's explicit
    // choice (DEPSYNC_FLAG_HW_ORDER), backed by the bounded wait.
    const bool want_queues = (pol->params.flags & (DEPSYNC_FLAG_QUEUE_ORDER | DEPSYNC_FLAG_REVERSE_ORDER)) != 0;
    const bool caller_hw = (pol->params.flags & DEPSYNC_FLAG_HW_ORDER) != 0;
    bool mixed = false;   // stages of differing macro-tile shapes: one launch (one kernel) per stage
    for (int s = 1; s < p.n_stages; ++s) mixed = mixed || p.tile[s] != p.tile[0];
    const bool all_resident = !mixed && total <= (uint32_t)p.slots;
    if (pol->force_order == 1 && !all_resident && !caller_hw) return DEPSYNC_EINVAL;   // not a candidate for the autotuner
    bool hw;
    if (pol->force_order >= 0) hw = pol->force_order == 1;
    else if (want_queues) hw = false;
    else if (caller_hw) hw = true;
    else hw = all_resident && p.order_pref != 0;
    if (sync && mode == DEPSYNC_MODE_FUSED && hw) a.flags |= DEPSYNC_FLAG_HW_ORDER;
    if (sync && (a.flags & DEPSYNC_FLAG_HW_ORDER) && mode == DEPSYNC_MODE_FINE && !all_resident)
        return DEPSYNC_EINVAL;

    // With the dispatch queues a launch needs no more workgroups than fit on the chip at once:
    // each keeps drawing tiles.  With tiles named by the block index (PLAIN, HW_ORDER) a launch
    // has one workgroup per tile.
    const bool queues = sync && !(a.flags & DEPSYNC_FLAG_HW_ORDER);
    auto blocks = [&](uint32_t tiles, int s = 0) { return queues ? std::min<uint32_t>(tiles, (uint32_t)p.stage_slots[s]) : tiles; };
    const int last = p.n_stages - 1;
    if (mode == DEPSYNC_MODE_FUSED) {
        // all stages in one dispatch; needs one macro-tile shape for the whole chain
        if (mixed) return DEPSYNC_ENOTIMPL;
        a.block_offset = 0;
        a.stage_lo = 0; a.stage_hi = (uint32_t)last;
        HIP_TRY(launch_chain_kernel(p.tile[0], p.dtype, p.amode, true, blocks(total), sp, a));
    } else if (mode == DEPSYNC_MODE_FINE) {
        // Section III-A: the stages are launched on different streams and overlap.  The LAST stage
        // goes on the caller's stream, the earlier ones on side streams forked off it with one
        // event.  Nothing is joined back: every tile of an earlier stage is waited for by some
        // tile of the stage after it, so the end of the last stage's launch is the end of the chain,
        // and the caller's stream carries no wait for another stream (a cross-stream wait costs
        // some 20 us here).  A launch works on its own stage and first helps with whatever earlier
        // stages have not been handed out yet, so the chain completes even if a side stream's
        // launch starts late: it then finds its tiles taken and ends.  Because it may run that
        // late (into a later chain), a side launch draws with compare-and-swap on a value it has
        // seen to lie in its own epoch, and never moves a counter otherwise.
        if (!pol->ev_fork) return DEPSYNC_EINVAL;          // a policy without streams of its own
        hipStream_t side[3] = {sc_ ? static_cast<hipStream_t>(sc_) : pol->own_stream, pol->third_stream, pol->fourth_stream};
        if (sc_) pol->last_side = static_cast<hipStream_t>(sc_);
        if (mixed) {
            // Two stages of differing tile shapes are two kernels, and neither launch can run the
            // other's tiles.  The producer goes on the side stream, the consumer on the caller's,
            // behind Section III-B's wait kernel: the consumer's workgroups are not started before
            // the producer's persistent workgroups hold their slots, so consumers that then fill
            // the rest of the chip wait for tiles that resident workgroups are working through.
            if (!queues || p.n_stages != 2) return DEPSYNC_EINVAL;
            HIP_TRY(hipEventRecord(pol->ev_fork, sp));
            HIP_TRY(hipStreamWaitEvent(side[0], pol->ev_fork, 0));
            const uint32_t nb0 = blocks(p.n_tiles[0], 0);
            a.block_offset = 0u; a.stage_lo = a.stage_hi = 0u; a.draw_cas = 1u;
            HIP_TRY(launch_chain_kernel(p.tile[0], p.dtype, p.amode, true, nb0, side[0], a));
            a.draw_cas = 0u;
            HIP_TRY(launch_wait_draws(a, 0u, nb0, sp));
            a.block_offset = p.n_tiles[0]; a.stage_lo = a.stage_hi = 1u;
            HIP_TRY(launch_chain_kernel(p.tile[1], p.dtype, p.amode, true, blocks(p.n_tiles[1], 1), sp, a));
            pol->side_used = true;
            pol->epoch += 1;
            pol->queue_epoch += 1;
            pol->launches += 1;
            return DEPSYNC_OK;
        }
        // When the last stage's launch has a workgroup of its own for every tile of the chain, all
        // of them resident at once, a side launch could only ever find its tiles taken (it starts
        // when the event has crossed streams, later than the caller's launch): it is left out, as
        // the paper leaves out its wait kernel when both kernels fit the GPU together (Section IV-C).
        const bool side_useful = !(queues && total <= (uint32_t)p.slots);
        if (side_useful) HIP_TRY(hipEventRecord(pol->ev_fork, sp));
        uint32_t off = 0;
        for (int s = 0; s < p.n_stages; ++s) {
            hipStream_t st = s == last ? sp : side[s];
            if (s != last && !side_useful) { off += p.n_tiles[s]; continue; }
            if (s != last) HIP_TRY(hipStreamWaitEvent(st, pol->ev_fork, 0));
            // (drawing from the queues, the last stage's launch covers the whole chain from its first
            // block on, so its first blocks go straight for the first stage's queues)
            a.block_offset = (s == last && queues) ? 0u : off;
            a.stage_lo = 0u;
            a.stage_hi = (uint32_t)s;
            a.draw_cas = s == last ? 0u : 1u;
            // (the last stage's launch may have to run the whole chain: as many workgroups as all of it
            // could use; the side launches together take at most half of the slots, so that whichever
            // launch starts first, the caller's finds room next to them)
            uint32_t nb = blocks(s == last && queues ? total : p.n_tiles[s]);
            if (s != last && queues) nb = std::min<uint32_t>(nb, std::max<uint32_t>(1u, (uint32_t)p.slots / (2u * (uint32_t)last)));
            HIP_TRY(launch_chain_kernel(p.tile[s], p.dtype, p.amode, true, nb, st, a));
            off += p.n_tiles[s];
        }
        a.draw_cas = 0u;
        if (side_useful) pol->side_used = true;
    } else {
        uint32_t off = 0;
        for (int s = 0; s < p.n_stages; ++s) {   // one launch per stage on the caller's stream
            a.block_offset = off;
            a.stage_lo = a.stage_hi = (uint32_t)s;
            HIP_TRY(launch_chain_kernel(p.tile[s], p.dtype, p.amode, sync, blocks(p.n_tiles[s], s), sp, a));
            off += p.n_tiles[s];
        }
    }
    if (sync) {
        pol->epoch += 1;
        if (queues) pol->queue_epoch += 1;   // every queue counter has advanced by its length
    }
    pol->launches += 1;
    return DEPSYNC_OK;
}

// Operand pointers, shapes and epilogues of a GeMM chain's stages (what does not depend on the plan).
void fill_gemm_stages(ChainArgs& a, const depsync_gemm_chain_desc* d) {
    const bool gate_up = d->mid == DEPSYNC_MID_SWIGLU;
    StageDesc& s0 = a.st[0];
    s0.A = d->X; s0.B = d->W1t; s0.C = d->H;
    s0.M = d->M; s0.N = d->N1; s0.K = d->K1;
    s0.lda = (uint32_t)d->ldx; s0.ldb = (uint32_t)d->ldw1; s0.ldc = (uint32_t)d->ldh;
    const bool kblocked = d->w_layout == DEPSYNC_W_KBLOCKED;
    s0.b_row_bytes = kblocked ? 128u : 2u * (uint32_t)d->ldw1;
    s0.b_kstep_bytes = kblocked ? 128u * (uint32_t)(gate_up ? 2 * d->N1 : d->N1) : 128u;
    s0.op = OP_GEMM; s0.amode = A_DENSE; s0.bmode = gate_up ? B_GATE_UP : B_DENSE;
    s0.act = d->mid == DEPSYNC_MID_GELU ? ACT_GELU : d->mid == DEPSYNC_MID_RELU ? ACT_RELU
             : gate_up ? ACT_SWIGLU : ACT_NONE;
    const bool attn = d->mid == DEPSYNC_MID_CAUSAL_ATTN;
    if (attn) {
        StageDesc& sa = a.st[1];
        sa.A = d->H; sa.C = d->T;
        sa.M = d->M; sa.N = d->heads * 128; sa.K = 128;
        sa.lda = (uint32_t)d->ldh; sa.ldc = (uint32_t)d->ldt;
        sa.op = OP_ATTN; sa.amode = A_DENSE; sa.bmode = B_DENSE; sa.act = ACT_NONE;
        sa.batch = d->batch; sa.seq = d->seq; sa.heads = d->heads; sa.head_dim = 128;
        sa.kcache = d->cached > 0 ? d->k_cache : nullptr; sa.vcache = d->cached > 0 ? d->v_cache : nullptr;
        sa.cached = (uint32_t)d->cached; sa.ld_cache = (uint32_t)d->ld_cache;
    }
    StageDesc& s1 = a.st[attn ? 2 : 1];
    s1.A = attn ? d->T : d->H; s1.B = d->W2t; s1.C = d->Y;
    s1.M = d->M; s1.N = d->N2; s1.K = attn ? d->heads * 128 : d->N1;
    s1.lda = (uint32_t)(attn ? d->ldt : d->ldh); s1.ldb = (uint32_t)d->ldw2; s1.ldc = (uint32_t)d->ldy;
    s1.b_row_bytes = kblocked ? 128u : 2u * (uint32_t)d->ldw2;
    s1.b_kstep_bytes = kblocked ? 128u * (uint32_t)d->N2 : 128u;
    s1.op = OP_GEMM; s1.amode = A_DENSE; s1.bmode = B_DENSE; s1.act = ACT_NONE;
}

void fill_conv_stages(ChainArgs& a, const depsync_conv_chain_n_desc* d) {
    const uint32_t M = (uint32_t)d->B * d->H * d->W;
    for (int i = 0; i < d->n; ++i) {
        const uint32_t cin = i == 0 ? (uint32_t)d->C : (uint32_t)d->K[i - 1];
        StageDesc& st = a.st[i];
        st.A = i == 0 ? d->in : d->out[i - 1]; st.B = d->w[i]; st.C = d->out[i];
        st.M = M; st.N = d->K[i]; st.K = 9u * cin;
        st.lda = cin; st.ldb = 9u * cin; st.ldc = d->K[i];
        st.b_row_bytes = 18u * cin; st.b_kstep_bytes = 128u;
        st.op = OP_GEMM; st.amode = A_CONV3X3; st.bmode = B_DENSE;
        st.act = i == d->n - 1 ? ACT_NONE : ACT_RELU;
        st.H = d->H; st.W = d->W; st.Cin = cin;
    }
}

int gemm_chain_impl(const depsync_gemm_chain_desc* d, sync_policy* pol, depsync_mode mode, void* stream_producer,
                    void* stream_consumer) {
    if (!pol) return DEPSYNC_EINVAL;
    if (mode != DEPSYNC_MODE_FINE && mode != DEPSYNC_MODE_STREAMSYNC && mode != DEPSYNC_MODE_PLAIN &&
        mode != DEPSYNC_MODE_FUSED)
        return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_gemm(d, pol, 0, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    uint32_t epoch = 0;
    if (mode != DEPSYNC_MODE_PLAIN) {
        rc = prepare_epoch(pol, p, static_cast<hipStream_t>(stream_producer), &epoch);
        if (rc != DEPSYNC_OK) return rc;
    }
    ChainArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_gemm_stages(a, d);
    if (int rs = ensure_scratch(pol, p); rs != DEPSYNC_OK) return rs;
    fill_common(a, pol, p, epoch);
    return launch_chain(pol, p, a, mode, stream_producer, stream_consumer);
}

}  // namespace

extern "C" {

int sync_policy_create(depsync_policy_kind kind, const depsync_policy_params* params, sync_policy_t** out) {
    if (!out) return DEPSYNC_EINVAL;
    *out = nullptr;
    if (kind != DEPSYNC_ROWSYNC && kind != DEPSYNC_TILESYNC && kind != DEPSYNC_STRIDEDSYNC && kind != DEPSYNC_AUTOSYNC)
        return DEPSYNC_EINVAL;
    sync_policy* p = new (std::nothrow) sync_policy();
    if (!p) return DEPSYNC_ENOMEM;
    p->kind = kind;
    if (params) p->params = *params; else std::memset(&p->params, 0, sizeof(p->params));
    hipError_t e = hipGetDevice(&p->device);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->ws), HEAP_LAYOUT.words * sizeof(uint32_t));
    if (e != hipSuccess) { delete p; return e == hipErrorOutOfMemory ? DEPSYNC_ENOMEM : hip_fail(e); }
    e = hipMemset(p->ws, 0, HEAP_LAYOUT.words * sizeof(uint32_t));
    if (e == hipSuccess) {
        StatusBlock sb{};
        sb.first_timeout = -1;
        e = hipMemcpy(p->ws + WS_STATUS, &sb, sizeof(sb), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&p->own_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&p->third_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&p->fourth_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_side, hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipFree(p->ws); delete p; return hip_fail(e); }
    p->epoch = 0;
    p->queue_epoch = 0;
    p->side_used = false;
    p->last_side = nullptr;
    p->force_order = -1;
    p->geom_sig = 0;
    p->launches = 0;
    p->sems_dirty = 0;
    p->scratch = nullptr;
    p->scratch_floats = 0;
    p->need_reset = false;
    p->lay = HEAP_LAYOUT;
    p->fixed_scratch = false;
    *out = p;
    return DEPSYNC_OK;
}

int sync_policy_destroy(sync_policy_t* pol) {
    if (!pol) return DEPSYNC_EINVAL;
    (void)hipDeviceSynchronize();
    (void)hipEventDestroy(pol->ev_fork);
    (void)hipEventDestroy(pol->ev_side);
    (void)hipStreamDestroy(pol->fourth_stream);
    (void)hipStreamDestroy(pol->own_stream);
    (void)hipStreamDestroy(pol->third_stream);
    (void)hipFree(pol->ws);
    if (pol->scratch) (void)hipFree(pol->scratch);
    delete pol;
    return DEPSYNC_OK;
}

int dep_chain_reset(sync_policy_t* pol, void* stream) {
    if (!pol) return DEPSYNC_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int rc = settle_side_launches(pol, st); rc != DEPSYNC_OK) return rc;
    HIP_TRY(launch_fill_u32(pol->ws + WS_TICKET, 0u, WS_TICKET_WORDS, st));
    HIP_TRY(launch_fill_u32(pol->ws + pol->lay.arrive, 0u, pol->lay.max_arrive * SYNC_WORD_STRIDE, st));
    HIP_TRY(launch_fill_u32(pol->ws + WS_STATUS, 0u, 8, st));
    HIP_TRY(launch_fill_u32(pol->ws + WS_STATUS + 1, 0xffffffffu, 1, st));   // first_timeout = -1
    HIP_TRY(launch_fill_u32(pol->ws + WS_SEMS, 0u, pol->sems_dirty * SYNC_WORD_STRIDE, st));
    pol->sems_dirty = 0;
    pol->epoch = 0;
    pol->queue_epoch = 0;
    pol->launches = 0;
    pol->need_reset = false;
    return DEPSYNC_OK;
}

int depsync_last_status(sync_policy_t* pol, depsync_status* out) {
    if (!pol || !out) return DEPSYNC_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    StatusBlock sb;
    HIP_TRY(hipMemcpy(&sb, pol->ws + WS_STATUS, sizeof(sb), hipMemcpyDeviceToHost));
    out->timed_out = sb.timed_out;
    out->first_timeout = sb.first_timeout;
    out->posts = sb.posts;
    out->waits = sb.waits;
    out->polling_waits = sb.polling_waits;
    out->launches = pol->launches;
    if (sb.timed_out > 0) { pol->need_reset = true; return DEPSYNC_ETIMEOUT; }
    return DEPSYNC_OK;
}

int depsync_read_trace(sync_policy_t* pol, depsync_trace_rec* out, int max_records) {
    if (!pol || !out || max_records < 0) return DEPSYNC_EINVAL;
    static_assert(sizeof(depsync_trace_rec) == sizeof(TraceRec), "trace record layout");
    HIP_TRY(hipDeviceSynchronize());
    const size_t n = std::min<size_t>((size_t)max_records, pol->lay.trace_cap);
    if (n == 0) return 0;
    HIP_TRY(hipMemcpy(out, pol->ws + pol->lay.trace, n * sizeof(TraceRec), hipMemcpyDeviceToHost));
    return (int)n;
}

int depsync_gemm_chain_plan(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int n_cu,
                            depsync_plan_info* out) {
    if (!out) return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_gemm(d, pol, n_cu, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    fill_plan_info(p, out);
    return DEPSYNC_OK;
}

int depsync_conv_chain_plan(const depsync_conv_chain_desc* d, const sync_policy_t* pol, int n_cu,
                            depsync_plan_info* out) {
    if (!out) return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_conv(d, pol, n_cu, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    fill_plan_info(p, out);
    return DEPSYNC_OK;
}

int dep_gemm_chain(const depsync_gemm_chain_desc* d, sync_policy_t* pol, depsync_mode mode, void* stream_producer,
                   void* stream_consumer) {
    return gemm_chain_impl(d, pol, mode, stream_producer, stream_consumer);
}

int dep_conv_chain_n(const depsync_conv_chain_n_desc* d, sync_policy_t* pol, depsync_mode mode, void* stream_producer,
                     void* stream_consumer) {
    if (!pol) return DEPSYNC_EINVAL;
    if (mode != DEPSYNC_MODE_FINE && mode != DEPSYNC_MODE_STREAMSYNC && mode != DEPSYNC_MODE_PLAIN &&
        mode != DEPSYNC_MODE_FUSED)
        return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_conv_n(d, pol, 0, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    uint32_t epoch = 0;
    if (mode != DEPSYNC_MODE_PLAIN) {
        rc = prepare_epoch(pol, p, static_cast<hipStream_t>(stream_producer), &epoch);
        if (rc != DEPSYNC_OK) return rc;
    }
    ChainArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_conv_stages(a, d);
    if (int rs = ensure_scratch(pol, p); rs != DEPSYNC_OK) return rs;
    fill_common(a, pol, p, epoch);
    return launch_chain(pol, p, a, mode, stream_producer, stream_consumer);
}

int dep_conv_chain(const depsync_conv_chain_desc* d, sync_policy_t* pol, depsync_mode mode, void* stream_producer,
                   void* stream_consumer) {
    if (!d) return DEPSYNC_EINVAL;
    const depsync_conv_chain_n_desc c = as_chain_n(*d);
    return dep_conv_chain_n(&c, pol, mode, stream_producer, stream_consumer);
}

int depsync_conv_chain_n_plan(const depsync_conv_chain_n_desc* d, const sync_policy_t* pol, int n_cu, depsync_plan_info* out) {
    if (!out) return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_conv_n(d, pol, n_cu, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    fill_plan_info(p, out);
    return DEPSYNC_OK;
}

int depsync_copy_chain_plan(const depsync_copy_chain_desc* d, const sync_policy_t* pol, int n_cu, depsync_plan_info* out) {
    if (!out) return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_copy(d, pol, n_cu, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    fill_plan_info(p, out);
    return DEPSYNC_OK;
}

int dep_copy_chain(const depsync_copy_chain_desc* d, sync_policy_t* pol, depsync_mode mode, void* stream_producer,
                   void* stream_consumer) {
    if (!pol) return DEPSYNC_EINVAL;
    if (mode != DEPSYNC_MODE_FINE && mode != DEPSYNC_MODE_STREAMSYNC && mode != DEPSYNC_MODE_PLAIN &&
        mode != DEPSYNC_MODE_FUSED)
        return DEPSYNC_EINVAL;
    Plan p;
    int rc = plan_copy(d, pol, 0, p);
    if (rc == DEPSYNC_OK) rc = check_limits(pol, p);
    if (rc != DEPSYNC_OK) return rc;
    uint32_t epoch = 0;
    if (mode != DEPSYNC_MODE_PLAIN) {
        rc = prepare_epoch(pol, p, static_cast<hipStream_t>(stream_producer), &epoch);
        if (rc != DEPSYNC_OK) return rc;
    }
    ChainArgs a;
    std::memset(&a, 0, sizeof(a));
    const uint32_t tb = d->tile_bytes ? d->tile_bytes : 65536u;
    StageDesc& s0 = a.st[0];
    s0.A = d->src; s0.C = d->mid;
    StageDesc& s1 = a.st[1];
    s1.A = d->mid; s1.C = d->dst;
    for (int s = 0; s < 2; ++s) {
        a.st[s].N = (uint32_t)(d->bytes >> 4);   // 16-byte units in all
        a.st[s].K = tb >> 4;                     // and per tile
        a.st[s].amode = A_COPY;
    }
    fill_common(a, pol, p, epoch);
    return launch_chain(pol, p, a, mode, stream_producer, stream_consumer);
}

}  // extern "C"

namespace {
// Time every macro-tile shape the chain can run with, each with and without the library's split
// along K and with tiles drawn from the dispatch queues or named by the block index (one-dispatch mode, HIP events on the caller's stream, two passes, blocks long enough
// to time), and remember the fastest combination.
template <class Desc, class Run>
int autotune(const Desc* d, sync_policy* pol, hipStream_t sp, int reps, int* tile_out, Run run, float* best_ms_out = nullptr) {
    if (!d || !pol) return DEPSYNC_EINVAL;
    if (pol->kind == DEPSYNC_AUTOSYNC) return DEPSYNC_EINVAL;   // per kind: see autotune_policy
    if (reps <= 0) reps = 3;
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipError_t e = hipEventCreate(&e1); e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e); }
    const uint32_t user_split = pol->params.ksplit;
    int best = 0, rc = DEPSYNC_OK;
    float best_ms = 0.f;
    auto time_block = [&](const Desc* dd, int n, float* per_run) -> int {
        int r = DEPSYNC_OK;
        hipError_t e = hipEventRecord(e0, sp);
        for (int i = 0; i < n && r == DEPSYNC_OK; ++i) r = run(dd);
        if (e == hipSuccess) e = hipEventRecord(e1, sp);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) return hip_fail(e);
        *per_run = ms / (float)n;
        return r;
    };
    for (int pass = 0; pass < 2 && rc == DEPSYNC_OK; ++pass) {
        for (int t = 1; t < DEPSYNC_TILE__COUNT && rc == DEPSYNC_OK; ++t) {
            for (int var = 0; var < (user_split == 0 ? 4 : 2) && rc == DEPSYNC_OK; ++var) {
                const int off = var >> 1, hw = var & 1;
                if (hw && (pol->params.flags & DEPSYNC_FLAG_HW_ORDER)) continue;   // already the caller's choice
                pol->params.ksplit = off ? 1u : user_split;
                pol->force_order = hw;
                Desc dd = *d;
                dd.tile_prod = dd.tile_cons = t;
                int r = run(&dd);                   // warm-up; also tells whether this shape is usable
                if (r == DEPSYNC_EINVAL || r == DEPSYNC_ENOTIMPL || r == DEPSYNC_ENOMEM) continue;
                if (r != DEPSYNC_OK) { rc = r; break; }
                float ms = 0.f;
                r = time_block(&dd, reps, &ms);
                if (r == DEPSYNC_OK && ms * reps < 1.0f)   // too short to compare: about 2 ms worth
                    r = time_block(&dd, (int)(2.0f / std::max(ms, 0.005f)) + 1, &ms);
                if (r != DEPSYNC_OK) { rc = r; break; }
                const int cand = t | (off ? 0x100 : 0) | (hw ? 0x200 : 0);
                if (best == 0 || ms < best_ms) { best = cand; best_ms = ms; }
            }
        }
    }
    pol->params.ksplit = user_split;
    pol->force_order = -1;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != DEPSYNC_OK) return rc;
    if (best == 0) return DEPSYNC_EINVAL;
    {
        std::lock_guard<std::mutex> g(g_tuned_mutex);
        g_tuned[tune_key(d, pol->kind)] = best;
    }
    if (tile_out) *tile_out = best & 0xff;
    if (best_ms_out) *best_ms_out = best_ms;
    return DEPSYNC_OK;
}
// flags of a remembered choice: bit 0 no split along K, bit 1 tiles in hardware order
template <class Desc>
int get_tuned(const Desc* d, const sync_policy* pol, int* tile, int* flags) {
    if (!d || !pol || !tile || !flags) return DEPSYNC_EINVAL;
    const int v = tuned_tile(tune_key(d, effective_kind(d, pol, -1)));
    *tile = v & 0xff;
    *flags = (v >> 8) & 3;
    return DEPSYNC_OK;
}
template <class Desc>
int set_tuned(const Desc* d, const sync_policy* pol, int tile, int flags) {
    if (!d || !pol || tile < 0 || tile >= DEPSYNC_TILE__COUNT || (flags & ~3)) return DEPSYNC_EINVAL;
    std::lock_guard<std::mutex> g(g_tuned_mutex);
    if (pol->kind == DEPSYNC_AUTOSYNC) return DEPSYNC_EINVAL;
    if (tile == 0) g_tuned.erase(tune_key(d, pol->kind));
    else g_tuned[tune_key(d, pol->kind)] = tile | (flags << 8);
    return DEPSYNC_OK;
}


// The policy part of the search of Section IV-A: autotune the chain under every policy kind it can
// run with and remember the kind of the fastest for the chain's shape (what DEPSYNC_AUTOSYNC
// policies then resolve to).  `pol` lends its workspace and parameters; its kind is restored.
template <class Desc, class Run>
int autotune_policy(const Desc* d, sync_policy* pol, hipStream_t sp, int reps, int* kind_out, int* tile_out, float* us_out, Run run) {
    if (!d || !pol) return DEPSYNC_EINVAL;
    const int own_kind = pol->kind;
    int best_kind = -1, best_tile = 0, rc = DEPSYNC_OK;
    float best_ms = 0.f;
    for (int kind = DEPSYNC_ROWSYNC; kind <= DEPSYNC_STRIDEDSYNC; ++kind) {
        pol->kind = kind;
        int tile = 0;
        float ms = 0.f;
        const int r = autotune(d, pol, sp, reps, &tile, run, &ms);
        if (us_out) us_out[kind] = r == DEPSYNC_OK ? ms * 1e3f : -1.f;
        if (r == DEPSYNC_EINVAL || r == DEPSYNC_ENOTIMPL) continue;     // the chain cannot run under this kind
        if (r != DEPSYNC_OK) { rc = r; break; }
        if (best_kind < 0 || ms < best_ms) { best_kind = kind; best_ms = ms; best_tile = tile; }
    }
    pol->kind = own_kind;
    if (rc != DEPSYNC_OK) return rc;
    if (best_kind < 0) return DEPSYNC_EINVAL;
    {
        std::lock_guard<std::mutex> g(g_tuned_mutex);
        g_tuned[tune_key(d, -2)] = best_kind + 1;
    }
    if (kind_out) *kind_out = best_kind;
    if (tile_out) *tile_out = best_tile;
    return DEPSYNC_OK;
}

}  // namespace

extern "C" {

int depsync_gemm_chain_autotune_policy(const depsync_gemm_chain_desc* d, sync_policy_t* pol, void* stream, int reps,
                                       int* kind_out, int* tile_out, float* us_out) {
    return autotune_policy(d, pol, static_cast<hipStream_t>(stream), reps, kind_out, tile_out, us_out,
                           [&](const depsync_gemm_chain_desc* dd) { return dep_gemm_chain(dd, pol, DEPSYNC_MODE_FUSED, stream, nullptr); });
}

int depsync_conv_chain_n_autotune_policy(const depsync_conv_chain_n_desc* d, sync_policy_t* pol, void* stream, int reps,
                                         int* kind_out, int* tile_out, float* us_out) {
    return autotune_policy(d, pol, static_cast<hipStream_t>(stream), reps, kind_out, tile_out, us_out,
                           [&](const depsync_conv_chain_n_desc* dd) { return dep_conv_chain_n(dd, pol, DEPSYNC_MODE_FUSED, stream, nullptr); });
}

int depsync_gemm_chain_policy(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int* kind) {
    if (!d || !pol || !kind) return DEPSYNC_EINVAL;
    *kind = effective_kind(d, pol, default_kind(d));
    return DEPSYNC_OK;
}

int depsync_conv_chain_n_policy(const depsync_conv_chain_n_desc* d, const sync_policy_t* pol, int* kind) {
    if (!d || !pol || !kind) return DEPSYNC_EINVAL;
    *kind = effective_kind(d, pol, DEPSYNC_STRIDEDSYNC);
    return DEPSYNC_OK;
}

int depsync_gemm_chain_autotune(const depsync_gemm_chain_desc* d, sync_policy_t* pol, void* stream, int reps,
                                int* tile_out) {
    return autotune(d, pol, static_cast<hipStream_t>(stream), reps, tile_out, [&](const depsync_gemm_chain_desc* dd) {
        return dep_gemm_chain(dd, pol, DEPSYNC_MODE_FUSED, stream, nullptr);
    });
}

int depsync_conv_chain_n_autotune(const depsync_conv_chain_n_desc* d, sync_policy_t* pol, void* stream, int reps,
                                  int* tile_out) {
    return autotune(d, pol, static_cast<hipStream_t>(stream), reps, tile_out, [&](const depsync_conv_chain_n_desc* dd) {
        return dep_conv_chain_n(dd, pol, DEPSYNC_MODE_FUSED, stream, nullptr);
    });
}

int depsync_conv_chain_autotune(const depsync_conv_chain_desc* d, sync_policy_t* pol, void* stream, int reps,
                                int* tile_out) {
    return autotune(d, pol, static_cast<hipStream_t>(stream), reps, tile_out, [&](const depsync_conv_chain_desc* dd) {
        return dep_conv_chain(dd, pol, DEPSYNC_MODE_FUSED, stream, nullptr);
    });
}

int depsync_gemm_chain_tuned(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int* tile, int* flags) {
    return get_tuned(d, pol, tile, flags);
}
int depsync_conv_chain_tuned(const depsync_conv_chain_desc* d, const sync_policy_t* pol, int* tile, int* flags) {
    return get_tuned(d, pol, tile, flags);
}
int depsync_gemm_chain_set_tuned(const depsync_gemm_chain_desc* d, const sync_policy_t* pol, int tile, int flags) {
    return set_tuned(d, pol, tile, flags);
}
int depsync_conv_chain_set_tuned(const depsync_conv_chain_desc* d, const sync_policy_t* pol, int tile, int flags) {
    return set_tuned(d, pol, tile, flags);
}

const char* depsync_strerror(int status) {
    switch (status) {
        case DEPSYNC_OK: return "ok";
        case DEPSYNC_EINVAL: return "invalid argument (null pointer, shape, alignment or enum)";
        case DEPSYNC_ENOMEM: return "out of memory or too many semaphores";
        case DEPSYNC_EHIP: return "a HIP call failed (see depsync_last_hip_error)";
        case DEPSYNC_ETIMEOUT: return "a bounded semaphore wait expired";
        case DEPSYNC_ENOTIMPL: return "not implemented in this build";
        case DEPSYNC_ELIMIT: return "the chain needs more semaphores, arrival counters or split-K scratch than the fixed static workspace holds";
        default: return "unknown status";
    }
}

int depsync_last_hip_error(void) { return g_last_hip_error; }

int depsync_tile_shape(int tile, int* rows, int* cols) {
    const TileShape* ts = tile_shape(tile);
    if (!ts || !rows || !cols) return DEPSYNC_EINVAL;
    *rows = ts->rows;
    *cols = ts->cols;
    return DEPSYNC_OK;
}

int depsync_mfma_calibration(int zero_operands, int milliseconds, double* tflops) {
    if (!tflops || milliseconds <= 0 || milliseconds > 2000) return DEPSYNC_EINVAL;
    int dev = 0, cus = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int n_blocks = 2 * cus;                      // two workgroups per CU: two waves per SIMD
    constexpr size_t SRC_BYTES = 1u << 20;
    std::vector<uint16_t> host(SRC_BYTES / 2, 0);
    if (!zero_operands) {
        // bf16 bit patterns with random sign and mantissa and exponents 124..128 (|x| in [1/8, 4))
        uint64_t x = 0x9e3779b97f4a7c15ull;
        for (auto& h : host) {
            x = x * 6364136223846793005ull + 1442695040888963407ull;
            const uint32_t r = (uint32_t)(x >> 33);
            h = (uint16_t)(((r & 1u) << 15) | ((124u + (r >> 1) % 5u) << 7) | ((r >> 8) & 127u));
        }
    }
    void* src = nullptr;
    float* out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = DEPSYNC_OK;
    auto fail = [&](hipError_t e) { if (e != hipSuccess && rc == DEPSYNC_OK) rc = hip_fail(e); return e != hipSuccess; };
    if (fail(hipMalloc(&src, SRC_BYTES)) || fail(hipMalloc(reinterpret_cast<void**>(&out), (size_t)n_blocks * 256 * sizeof(float))) ||
        fail(hipMemcpy(src, host.data(), SRC_BYTES, hipMemcpyHostToDevice)) || fail(hipEventCreate(&e0)) ||
        fail(hipEventCreate(&e1))) {
        // fall through to the clean-up
    } else {
        // a short launch sizes the loop; then launches of about 10 ms each until the time is used
        // up, so that the clock has settled under the power cap; the last launch is reported
        const double flops_per_iter = (double)n_blocks * 4 * 8 * 2.0 * 32 * 32 * 16;
        float ms = 0.f;
        int iters = 2000;
        double spent = 0.0;
        while (rc == DEPSYNC_OK) {
            if (fail(hipEventRecord(e0, nullptr)) || fail(launch_mfma_calibration(src, out, n_blocks, iters, nullptr)) ||
                fail(hipEventRecord(e1, nullptr)) || fail(hipEventSynchronize(e1)) || fail(hipEventElapsedTime(&ms, e0, e1)))
                break;
            *tflops = flops_per_iter * iters / (ms * 1e-3) * 1e-12;
            spent += ms;
            if (spent >= milliseconds) break;
            iters = (int)std::min(2.0e6, std::max(2000.0, iters * 10.0 / std::max(ms, 0.01f)));
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (src) (void)hipFree(src);
    if (out) (void)hipFree(out);
    return rc;
}

size_t depsync_workspace_bytes(void) { return (size_t)HEAP_LAYOUT.words * sizeof(uint32_t); }

int depsync_device_info(int* n_cu, int* clock_khz) {
    if (!n_cu || !clock_khz) return DEPSYNC_EINVAL;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    HIP_TRY(hipDeviceGetAttribute(clock_khz, hipDeviceAttributeClockRate, dev));
    return DEPSYNC_OK;
}

}  // extern "C"

// ---- allocation-free entry point -----------------------------------------------------------

// Workspace of dep_gemm_chain_static: dispatch counters, status, zero page, semaphores and
// arrival counters (STATIC_LAYOUT), then the split-K partial tiles.  In host code this name is
// only a handle for hipGetSymbolAddress; the device address it returns (one per GPU) is what
// kernels and fills are given.
static __device__ __align__(256) uint32_t scratch[STATIC_WORDS];

namespace {

constexpr int STATIC_MAX_DEVICES = 64;
struct StaticState {
    sync_policy pol;
    bool ready;
};
StaticState g_static[STATIC_MAX_DEVICES];
std::mutex g_static_mutex;

// The static policy of the current device, set up on first use (device address of the array,
// status block).  Called with g_static_mutex held.
int static_policy(hipStream_t st, sync_policy** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return DEPSYNC_EINVAL;
    StaticState& S = g_static[dev];
    if (!S.ready) {
        uint32_t* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return DEPSYNC_EHIP;
        // the array is zero when the library's code is loaded onto the device; only the status
        // block's "no time-out yet" marker is not zero
        HIP_TRY(launch_fill_u32(ptr + WS_STATUS + 1, 0xffffffffu, 1, st));
        std::memset(&S.pol, 0, sizeof(S.pol));
        S.pol.device = dev;
        S.pol.ws = ptr;
        S.pol.lay = STATIC_LAYOUT;
        S.pol.fixed_scratch = true;
        S.pol.scratch = reinterpret_cast<float*>(ptr + STATIC_LAYOUT.words);
        S.pol.scratch_floats = STATIC_PARTIAL_FLOATS;
        S.pol.force_order = -1;
        S.ready = true;
    }
    *out = &S.pol;
    return DEPSYNC_OK;
}

// Consumer tiles (row tile, K part) of stage s whose operand slices are not all covered by a
// wait issued at or before the K step that loads them.
int64_t uncovered_waits(const Plan& p, const ChainArgs& a, int s) {
    const StageDesc& st = a.st[s];
    const TileShape* ts = tile_shape(p.tile[s]);
    if (!ts || st.dep_kind == DEP_NONE || st.op != OP_GEMM) return 0;
    const uint32_t TM = (uint32_t)ts->rows;
    const uint32_t KT = st.K / 64, S = st.ksplit;
    const uint32_t seg_steps = dep_seg_steps(st);
    int64_t bad = 0;
    std::vector<uint8_t> waited(p.sem_count[s]);
    for (uint32_t ty = 0; ty < st.grid_y; ++ty) {
        const uint32_t m0 = ty * TM, m_last = std::min(m0 + TM, st.M) - 1;
        for (uint32_t kz = 0; kz < S; ++kz) {
            std::fill(waited.begin(), waited.end(), 0);
            const uint32_t kb = kz * (KT / S), ke = kb + KT / S;
            uint32_t seg_next = kb;
            bool ok = true;
            for (uint32_t k = kb; k < ke && ok; ++k) {
                if (k == seg_next) {
                    seg_next = seg_steps ? seg_next + seg_steps : 0xffffffffu;
                    DepRange r;
                    if (dep_segment(st, m0, TM, k, kb, r))
                        for (uint32_t y = r.y0; y <= r.y1; ++y) waited[policy_sem(st.dep_kind, r.x, y, st.prod_grid_y, st.stride)] = 1;
                }
                // producer tiles whose output this K step's slice of A is read from
                const uint32_t k0 = k * 64;
                auto need = [&](uint32_t row, uint32_t col) {
                    const uint32_t x = col / st.prod_tn, y = row / st.prod_tm;
                    if (x >= st.prod_grid_x || y >= st.prod_grid_y || !waited[policy_sem(st.dep_kind, x, y, st.prod_grid_y, st.stride)]) ok = false;
                };
                if (st.amode == A_CONV3X3) {
                    const uint32_t tap = k0 / st.Cin, c0 = k0 % st.Cin;
                    const int fr = (int)(tap / 3) - 1, fs = (int)(tap % 3) - 1;
                    for (uint32_t m = m0; m <= m_last; ++m) {
                        const uint32_t rem = m % (st.H * st.W);
                        const int y = (int)(rem / st.W) + fr, x = (int)(rem % st.W) + fs;
                        if (y < 0 || y >= (int)st.H || x < 0 || x >= (int)st.W) continue;   // padding: nothing is read
                        const uint32_t row = (uint32_t)((int)m + fr * (int)st.W + fs);
                        need(row, c0); need(row, c0 + 63);
                    }
                } else {
                    need(m0, k0); need(m0, k0 + 63); need(m_last, k0); need(m_last, k0 + 63);
                    for (uint32_t y = m0 / st.prod_tm; y <= m_last / st.prod_tm; ++y) need(y * st.prod_tm, k0);
                }
            }
            if (!ok) ++bad;
        }
    }
    return bad;
}

// A policy object that exists on the host only (kind and parameters for the planner).
sync_policy host_policy(int kind, const depsync_policy_params* params) {
    sync_policy hp;
    std::memset(&hp, 0, sizeof(hp));
    hp.kind = kind;
    if (params) hp.params = *params;
    hp.lay = HEAP_LAYOUT;
    hp.force_order = -1;
    return hp;
}

bool valid_kind(int kind) { return kind == DEPSYNC_ROWSYNC || kind == DEPSYNC_TILESYNC || kind == DEPSYNC_STRIDEDSYNC || kind == DEPSYNC_AUTOSYNC; }

}  // namespace

extern "C" {

int dep_gemm_chain_static(const depsync_gemm_chain_desc* d, depsync_policy_kind kind, const depsync_policy_params* params,
                          void* stream) {
    if (!valid_kind(kind)) return DEPSYNC_EINVAL;
    if (params && (params->flags & DEPSYNC_FLAG_TRACE)) return DEPSYNC_EINVAL;   // the static workspace has no trace area
    std::lock_guard<std::mutex> g(g_static_mutex);
    sync_policy* pol = nullptr;
    if (int rc = static_policy(static_cast<hipStream_t>(stream), &pol); rc != DEPSYNC_OK) return rc;
    pol->kind = kind;
    if (params) pol->params = *params; else std::memset(&pol->params, 0, sizeof(pol->params));
    return gemm_chain_impl(d, pol, DEPSYNC_MODE_FUSED, stream, nullptr);
}

int depsync_gemm_chain_check_waits(const depsync_gemm_chain_desc* d, depsync_policy_kind kind,
                                   const depsync_policy_params* params, int n_cu, int64_t* uncovered) {
    if (!uncovered || !valid_kind(kind)) return DEPSYNC_EINVAL;
    const sync_policy hp = host_policy(kind, params);
    Plan p;
    if (int rc = plan_gemm(d, &hp, n_cu, p); rc != DEPSYNC_OK) return rc;
    ChainArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_gemm_stages(a, d);
    for (int s = 0; s < p.n_stages; ++s) fill_stage_geometry(a.st[s], p, s);
    *uncovered = 0;
    for (int s = 1; s < p.n_stages; ++s) *uncovered += uncovered_waits(p, a, s);
    return DEPSYNC_OK;
}

int depsync_conv_chain_n_check_waits(const depsync_conv_chain_n_desc* d, depsync_policy_kind kind,
                                     const depsync_policy_params* params, int n_cu, int64_t* uncovered) {
    if (!uncovered || !valid_kind(kind)) return DEPSYNC_EINVAL;
    const sync_policy hp = host_policy(kind, params);
    Plan p;
    if (int rc = plan_conv_n(d, &hp, n_cu, p); rc != DEPSYNC_OK) return rc;
    ChainArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_conv_stages(a, d);
    for (int s = 0; s < p.n_stages; ++s) fill_stage_geometry(a.st[s], p, s);
    *uncovered = 0;
    for (int s = 1; s < p.n_stages; ++s) *uncovered += uncovered_waits(p, a, s);
    return DEPSYNC_OK;
}

}  // extern "C"
