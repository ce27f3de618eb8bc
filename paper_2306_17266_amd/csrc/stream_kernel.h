// The stream kernel: one launch runs a whole SubNet query (all layers) on a fixed grid of
// workgroups that synchronise between layers with a grid barrier, instead of one launch per layer.
//
// Activations written by one layer are read by other workgroups (on other XCDs, whose L2s are not
// coherent with each other) in the next layer.  They are therefore stored write-through and loaded
// around the L2 (agent-scope "sc1" accesses); weights, which never change, use ordinary cached
// loads.  The barrier is two-level (groups of 16 workgroups, then the group leaders) on 64-bit
// monotonic counters; every wait is bounded by a spin limit, after which the kernel raises an abort
// flag and all workgroups leave.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <vector>

#include "kernels.h"
#include "model.h"

namespace sushi {

constexpr int STREAM_THREADS = 512;  // 8 waves per workgroup
constexpr int STREAM_WAVES = STREAM_THREADS / 64;
constexpr int BARRIER_GROUP = 16;    // workgroups per first-level barrier group
constexpr int SYNC_WORDS = 512 * 16;  // 64-bit words in the barrier area (128-byte spacing)

// A whole squeeze-excite block as one op of a team program (DEV_SE): average over the pixels, the two FC layers
// (activation `act1` after the first, hard sigmoid after the second), and the map times the resulting gate.
// Every vector between the steps stays in LDS as float32.
struct SeArgs {
    const void *x;            // [B][C / 8][HW][8] bf16, the map to gate (read only)
    void *y;                  // gated map, same shape, another buffer
    const void *reserved;     // null (x, y and this word lie where ConvArgs has x, y, res: the team kernel turns
                              // those three from arena offsets into addresses for every kind of op)
    const void *w1, *w2;      // packed weights of the FC layers: [channel group of 8][filter < Kpad][8]
    const float *sc1, *sh1;   // per filter of FC 1 (sc1 may be null = 1)
    const float *sc2, *sh2;   // per filter of FC 2 (sc2 may be null = 1)
    int B, HW, C, mid;        // images, pixels per image, channels of the map, filters of FC 1
    int Kpad1, Kpad2;         // padded filter counts of the two weight tensors
    int act1;                 // sushi_act after FC 1
    int pad;
};
constexpr int SE_MAX_C = 1024, SE_MAX_MID = 256;  // what the op's LDS layout has room for

// Kinds of a team program beyond OpKind (model.h): a fused squeeze-excite block, and the slots of the ops it
// replaced (skipped without a barrier, so a program keeps one slot per op of the plan).
constexpr int DEV_SE = 6, DEV_NONE = 7;

struct DevOp {
    int kind;      // OpKind (model.h), DEV_SE or DEV_NONE
    int pt, wk;    // dense conv: pixel tiles per unit (1, 2, 4) and waves sharing one unit (1, 2, 4, 8);
                   // wk = 0: tiled units (ft x pt tiles per wave); wk = -1: stem units (pt output rows per band); wk = -2: depthwise through LDS; wk = -3: tiled units with the weights held in LDS; wk = -4: depthwise straight from memory, neighbouring outputs per thread
    int n_units;   // dense conv: filter groups x pixel groups
    int n_p;       // dense conv: pixel groups
    int in_patch;  // input pointer is the caller's input buffer
    int out_patch; // output pointer is the caller's logits buffer
    int relative;  // activation pointers hold (offset into the team's arena) + 1
    int layer;     // SuperNet layer of a conv / FC op, -1 otherwise
    int ft;        // dense conv: filter tiles per unit (1, 2, 4); ft * pt <= 4
    union {
        ConvArgs conv;
        SeArgs se;  // kind == DEV_SE
    };
    PoolArgs pool;
};
static_assert(sizeof(SeArgs) <= sizeof(ConvArgs) && offsetof(SeArgs, x) == offsetof(ConvArgs, x) &&
                  offsetof(SeArgs, y) == offsetof(ConvArgs, y) && offsetof(SeArgs, reserved) == offsetof(ConvArgs, res),
              "the squeeze-excite arguments share the conv arguments' words, activation pointers in the same places");

struct StreamArgs {
    const DevOp *prog;  // DEVICE
    int n_ops;
    const void *input;  // DEVICE, caller's
    void *logits;       // DEVICE, caller's
    unsigned long long *sync;       // DEVICE barrier area, SYNC_WORDS words, zero before first use
    unsigned long long epoch_base;  // barriers already counted on `sync`
    int spin_limit;
    unsigned *abort_flag;  // pinned HOST memory, set to 1 when a wait ran out
};

// ---------------------------------------------------------------------------------------------
// The team kernel: a persistent kernel in which the workgroups running on one XCD form one to sixteen teams.
// A team serves one query at a time, entirely inside its XCD: activations go through that XCD's L2
// (ordinary stores; loads that skip the vector L1, which is emptied once per query), layers are separated by a
// team barrier (2 to 32 arrivals instead of 256), and 8 to 128 queries are in flight on the chip.  Queries arrive through per-team mailboxes in
// pinned host memory; a team leader that finds no post for `idle_ticks` (or sees `stop`) makes its
// team leave, so the kernel always ends by itself.
constexpr int MAX_XCDS = 8;
constexpr int MAX_TEAMS = 128;  // up to sixteen teams per XCD (two workgroups each; with one each the stream runs a third slower)
enum TeamCmd { TEAM_RUN = 0, TEAM_STOP = 1 };

// SubGraph residency inside the team kernel (the persistent buffer of the paper, Section 4.2.2, kept
// in LDS): every workgroup of a team owns RES_STORE_BYTES of LDS that survive from query to query.
// The store is cut into slabs, one per 16-filter tile of a layer:
// [tap][channel group < cg_stride][16 filters][8 channels] bf16, i.e. 256 bytes per (tap, group).  Slab f
// of a layer lives in the LDS of workgroup `owner` at byte offset `lds_off`; that workgroup computes
// filter tile f of the layer for every query and reads those weights from LDS instead of memory.
// Which slab sits where (the geometry) is fixed for as long as the cached SubGraphs fit it: a layer's
// slabs are as wide (cg_stride) and as many as the largest SubGraph cached so far asked for.  A new
// SubGraph then only changes how much of every slab is valid (tiles below n_res, channel groups below
// cg_res), and a team copies just the cells its stores do not hold yet.
// Every team holds the same slabs.  Only layers that run as a single pixel group (at most 64 output
// pixels per query: the late stages, squeeze-excite and classifier layers, which hold most of the
// weights) use their slabs.
constexpr int RES_STORE_BYTES = 120 * 1024;
constexpr int RED_BYTES = STREAM_WAVES * 4 * 256 * 4;  // partial-sum scratch in front of the store

struct ResEntry {
    int owner;    // rank inside the team, -1 = the geometry has no slab for this tile
    int lds_off;  // byte offset inside the owner's store
};

struct ResLayer {
    const void *w;  // packed weights of the layer (DEVICE)
    int Kpad, CG, taps;
    int cg_res;      // valid channel groups of every valid tile (cached SubGraph's channels, at most cg_stride)
    int n_res;       // filter tiles 0 .. n_res-1 are valid where the geometry has a slab for them (see entries)
    int first_entry; // index of tile 0's entry in ResTable::entries
    int cg_stride;   // channel groups a slab of this layer has room for
    int pad;
};

// The host writes a table into pinned HOST memory; a team copies it into device memory of its own
// before it uses it (see TeamArgs::team_mem), with `layers` and `entries` pointing into that copy.
struct ResTable {
    int n_layers, team_size;  // team size the owners were assigned for
    int n_entries, geometry;  // tables with the same geometry number place every slab alike
    const ResLayer *layers;   // one per SuperNet layer
    const ResEntry *entries;
};
constexpr int RES_MAX_LAYERS = 256, RES_MAX_ENTRIES = 16384;
static_assert(sizeof(ResTable) == 32 && sizeof(ResLayer) % 8 == 0 && sizeof(ResEntry) == 8, "tables are copied in 8-byte words");

// Device memory of one team: the program of the query it is running and its copy of the residency table.
constexpr int TEAM_PROG_MAX_OPS = 512;

struct TeamPost {  // written by the host
    unsigned long long seq;  // the post's number (1, 2, ...)
    int cmd, n_ops;
    const DevOp *prog;  // pinned HOST; activation pointers are arena offsets + 1
    const void *input;  // DEVICE
    void *logits;       // DEVICE
    // The residency table the query runs under (pinned HOST, null: nothing cached) and its number.  A team
    // that holds another number brings its LDS stores up to this table before it runs the query, so a team
    // pays for a change of the cached SubGraph once per query at most, however many changes went by
    // since its last query.
    const ResTable *table;
    unsigned long long table_seq;  // > 0
    unsigned long long pad;
};
static_assert(sizeof(TeamPost) == 64, "a post is eight 8-byte words");

constexpr int POST_RING = 32;  // posts a team's mailbox holds (post number s sits in slot s % POST_RING)

struct TeamHostState {  // pinned HOST memory, device-visible
    TeamPost post[MAX_TEAMS][POST_RING];
    unsigned long long posted[MAX_TEAMS * 8];  // posted[8 t]: number of posts written for team t (host)
    unsigned long long done[MAX_TEAMS * 8];    // done[8 t]: number of posts team t has finished (kernel)
    unsigned team_size[MAX_TEAMS];
    unsigned ready;       // kernel: teams are formed, sizes valid
    unsigned stop;        // host: leave as soon as idle
    unsigned abort_flag;  // kernel: a bounded wait ran out
};

struct TeamArgs {
    TeamHostState *host;
    unsigned long long *sync;  // DEVICE, SYNC_WORDS words, zero at launch
    char *arena;               // DEVICE, MAX_TEAMS arenas
    long arena_bytes;          // bytes per team arena
    unsigned long long last_seq[MAX_TEAMS];  // posts each team has already finished
    long idle_ticks;           // 100 MHz ticks a leader waits for a post before its team leaves
    int teams_per_xcd;         // 1: the workgroups of an XCD form one team; 2, 4, 8, 16: that many teams, each a share of them
    int spin_limit;
    char *team_mem;            // DEVICE, MAX_TEAMS areas of TEAM_MEM_BYTES: [program][residency table][slab words]
    unsigned long long *trace;  // DEVICE or null: [MAX_TEAMS][TRACE_SLOTS] 100 MHz timestamps, one after each op
};
constexpr int TRACE_SLOTS = 256;
// [program][residency table][one word per table entry: what of the slab the owner's LDS store holds]
constexpr long TEAM_TABLE_OFFSET = (long)TEAM_PROG_MAX_OPS * sizeof(DevOp);
constexpr long TEAM_TABLE_BYTES = 64 + (long)RES_MAX_LAYERS * sizeof(ResLayer) + (long)RES_MAX_ENTRIES * sizeof(ResEntry);
constexpr long TEAM_MEM_BYTES = TEAM_TABLE_OFFSET + TEAM_TABLE_BYTES + (long)RES_MAX_ENTRIES * 4;
static_assert(sizeof(DevOp) % 8 == 0, "programs are copied in 8-byte words");

// Two team kernels: one for networks without depthwise layers (dense convs, max-pool, pooling, FC) and one for the
// inverted-residual families (depthwise, gating and squeeze-excite ops instead of the max-pool).  A kernel has one
// register allocation for all the units in it, so each holds only the units its networks use.
hipError_t launch_team_kernel(const TeamArgs &a, int nwg, hipStream_t s);
hipError_t launch_team_kernel_mobile(const TeamArgs &a, int nwg, hipStream_t s);
// Sets the kernel's dynamic LDS limit; call once per device before the first launch.
hipError_t prepare_team_kernel();
hipError_t prepare_team_kernel_mobile();
// Workgroups of the team kernel that fit on one compute unit at the same time.
hipError_t team_kernel_blocks_per_cu(int *n);
hipError_t team_kernel_mobile_blocks_per_cu(int *n);

// The matrix-core paths of both kernels keep one table entry per reduction step (tap x 32 channels)
// of the running op in LDS and one bit per tap in a 32-bit mask.
constexpr int STEP_TABLE_MAX = 256;
inline bool dense_op_fits(const ConvArgs &a) {
    return a.R * a.R <= 32 && a.R * a.R * ((a.C + 31) / 32) + 1 <= STEP_TABLE_MAX;
}

// Bytes of the 32 KiB LDS scratch (RED_BYTES) the unit variant chosen for `op` uses, from the kernels' layouts.
long dev_op_lds_bytes(const DevOp &op);

// Chooses pt / wk / unit counts of a dense conv or FC op for a grid of nwg workgroups.
void tile_dev_op(DevOp &op, int nwg, bool team);
// A dense conv with few input channels (the stem): sets wk = -1 and the band height in pt if the
// layer qualifies for the matrix-core stem path, else leaves the op alone and returns false.
bool tile_stem_op(DevOp &op, int nwg);
// A depthwise conv: sets wk = -2, the channel groups per unit in ft and the band height in pt if the layer fits
// the LDS-staged path, else leaves the op alone and returns false.
bool tile_dw_op(DevOp &op, int nwg);

// Team programs: turns every squeeze-excite block of the plan whose dimensions fit (pooling, FC, FC, gating in
// four consecutive slots, the gated map in a buffer of its own) into one DEV_SE op in the first slot and DEV_NONE
// in the other three.  `prog` has one op per op of `plan`.  Returns the number of blocks fused.
int fuse_se_blocks(std::vector<DevOp> &prog, const Plan &plan);

// Number of grid barriers the kernel executes for a program of n_ops ops.
inline int stream_barriers(int n_ops) { return n_ops > 0 ? n_ops - 1 : 0; }

hipError_t launch_stream_kernel(const StreamArgs &a, int nwg, hipStream_t s);

}  // namespace sushi
