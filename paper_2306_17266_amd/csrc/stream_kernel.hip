// The stream kernel (see stream_kernel.h): a whole SubNet query in one launch; the team kernel for networks
// without depthwise layers; and the host side of both (tilings, fused ops, LDS accounting).
#include "stream_units.h"

namespace sushi {

// ------------------------------------------------------------------ the kernel

// (two waves per SIMD: see sushi_team_kernel)
__global__ __launch_bounds__(STREAM_THREADS, 2) void sushi_stream_kernel(StreamArgs sa) {
    __shared__ float lds[STREAM_WAVES * 4 * 256];  // conv partial sums; 64x8x9 floats for pooling fit too
    __shared__ int barrier_ok;
    __shared__ DevOp op;
    __shared__ u32x4_t step_entries[STEP_TABLE_MAX];
    __shared__ u32x2_t slab_entries[STEP_TABLE_MAX];
    const StepTables tb{step_entries, slab_entries};
    unsigned long long epoch = sa.epoch_base;
    for (int i = 0; i < sa.n_ops; ++i) {
        // every thread needs the op's fields: stage the descriptor in LDS once per workgroup
        {
            const int *src = reinterpret_cast<const int *>(sa.prog + i);
            int *dst = reinterpret_cast<int *>(&op);
            for (int k = threadIdx.x; k < (int)(sizeof(DevOp) / sizeof(int)); k += STREAM_THREADS) dst[k] = src[k];
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            if (op.in_patch) op.conv.x = sa.input;
            if (op.out_patch) op.conv.y = sa.logits;
        }
        __syncthreads();
        run_op<AUX_SC1, AUX_SC1, false, OPS_ALL>(uniform_op(op), lds, (int)blockIdx.x, (int)gridDim.x,
                                        ResView{nullptr, nullptr, nullptr, nullptr}, tb);
        if (i + 1 < sa.n_ops) {
            epoch += 1;
            if (!grid_barrier(sa, epoch, &barrier_ok)) return;
        }
    }
}

// ------------------------------------------------------------------ the team kernel, dense networks
hipError_t prepare_team_kernel() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(sushi_team_kernel<OPS_DENSE>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, RED_BYTES + RES_STORE_BYTES);
}

hipError_t team_kernel_blocks_per_cu(int *n) {
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, sushi_team_kernel<OPS_DENSE>, STREAM_THREADS,
                                                        RED_BYTES + RES_STORE_BYTES);
}

hipError_t launch_team_kernel(const TeamArgs &a, int nwg, hipStream_t s) {
    hipLaunchKernelGGL(sushi_team_kernel<OPS_DENSE>, dim3(nwg), dim3(STREAM_THREADS), RED_BYTES + RES_STORE_BYTES, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ host side

// Picks the unit shape (ft x pt tiles of 16 x 16) and the waves per unit (wk) of a dense conv / FC op
// for nwg cooperating workgroups from a small cost model, in units of one load round trip: a
// workgroup runs ceil(groups / nwg) unit groups one after the other; a group costs one round trip
// per batch of U reduction steps, plus the LDS reduction when waves share a unit, plus the epilogue.
void tile_dev_op(DevOp &op, int nwg, bool team) {
    const ConvArgs &a = op.conv;
    const long M = (long)a.B * a.P * a.Q;
    const long ptiles = (M + 15) / 16, ftiles = (a.K + 15) / 16;
    const int nsteps = a.R * a.R * ((a.C + 31) / 32);
    // In microseconds, a least-squares fit to timings of the layer shapes of a ResNet50-like SuperNet with
    // every team of the chip busy: a group of units (one per slot) has a fixed cost (first loads, reduction
    // across waves) plus an epilogue per tile, and a cost per reduction step of a wave that grows mostly
    // with the activation tiles it loads.
    static const int shapes[7][2] = {{2, 4}, {1, 4}, {2, 2}, {1, 2}, {4, 1}, {2, 1}, {1, 1}};
    auto shape_cost = [&](int ft, int pt, int wk) {
        const long n_f = (ftiles + ft - 1) / ft, n_p = (ptiles + pt - 1) / pt;
        const long units = n_f * n_p;
        const int slots = STREAM_WAVES / wk;
        const long iters = ((units + slots - 1) / slots + nwg - 1) / nwg;
        const int per_wave = (nsteps + wk - 1) / wk;
        const double step = 0.047 + 0.1275 * pt + 0.038 * ft;
        const double fixed = 2.84 + 0.56 * ft * pt;
        return 2.87 + iters * (fixed + per_wave * step);
    };
    // team kernel, at most 64 output pixels: units of at most two filter tiles can take their weights
    // from resident slabs
    const bool slab_shapes_only = team && ptiles <= 4;
    double best = 1e30;
    int bft = 1, bpt = 1, bwk = 1;
    for (const auto &sh : shapes)
        for (int wk = 1; wk <= STREAM_WAVES; wk *= 2) {
            // eight tiles: one wave per unit (nothing to add up) or all waves on one unit (the partial sums of
            // one filter tile at a time fit the scratch)
            if (sh[0] * sh[1] > 4 && wk != STREAM_WAVES && wk != 1) continue;
            if (slab_shapes_only && sh[0] > 2) continue;
            if (a.in_f32 && sh[1] != 1) continue;  // float32 vector input: units of one pixel tile
            if (sh[1] > ptiles && !(sh[1] == 4 && ptiles == 3)) continue;
            const double cost = shape_cost(sh[0], sh[1], wk);
            if (cost < best - 1e-9) best = cost, bft = sh[0], bpt = sh[1], bwk = wk;
        }
    // tiled units (wk = 0): at filter tiles x 8 waves x bt pixel tiles, the weight tile shared in LDS
    bool tiled = false;
    if ((a.C & 7) == 0 && ptiles >= STREAM_WAVES && !a.in_f32) {
        static const int tile_shapes[10][2] = {{2, 1}, {2, 2}, {3, 1}, {3, 2}, {3, 4}, {4, 1}, {4, 2}, {4, 4}, {6, 1}, {6, 2}};
        for (const auto &tsh : tile_shapes) {
            const int at = tsh[0], bt = tsh[1];
            {
                const long n_f = (ftiles + at - 1) / at, n_p = (ptiles + STREAM_WAVES * bt - 1) / (STREAM_WAVES * bt);
                const long iters = (n_f * n_p + nwg - 1) / nwg;
                // least-squares fit to timings of the layer shapes of a ResNet50-like SuperNet with every
                // team of the chip busy (teams of 8, 16 and 32 workgroups): a step costs mostly what the
                // activation tiles of a wave cost to load, a unit has a fixed cost for set-up and first
                // loads plus the epilogue of its at x bt tiles per wave, the op a constant.  In microseconds.
                const int round = tile_ks(bt) * TILE_SETS;
                const int steps_pad = (nsteps + round - 1) / round * round;
                // LDS: two weight stages, the epilogue constants, one 16-byte entry per step (the loads
                // run one round past the last step)
                if (2 * tile_ks(bt) * at * 1024 + at * 128 + (steps_pad + round) * 16 > RED_BYTES) continue;
                const double step_cost = 0.034 + 0.0234 * at + 0.0847 * bt - 0.0035 * at * bt;
                const double unit_cost = 1.54 + at * bt * (a.res ? 0.346 : 0.327) + steps_pad * step_cost;
                const double cost = 2.14 + iters * unit_cost;
                if (cost < best - 1e-9) best = cost, bft = at, bpt = bt, bwk = 0, tiled = true;
            }
        }
    }
    // the same units with the filter group's weights held in LDS (wk = -3): short reductions only
    bool ares = false;
    if ((a.C & 7) == 0 && ptiles >= STREAM_WAVES && !a.in_f32) {
        static const int shapes_r[5][2] = {{2, 1}, {2, 2}, {4, 1}, {4, 2}, {6, 1}};
        const int steps_pad = (nsteps + ARES_D - 1) / ARES_D * ARES_D;
        for (const auto &sh : shapes_r) {
            const int at = sh[0], bt = sh[1];
            if ((long)nsteps * at * 1024 + at * 128 + steps_pad * 16 > RED_BYTES) continue;
            const long n_f = (ftiles + at - 1) / at, n_p = (ptiles + STREAM_WAVES * bt - 1) / (STREAM_WAVES * bt);
            const long iters = (n_f * n_p + nwg - 1) / nwg;
            // filter groups a workgroup meets on its way through units rank, rank + nwg, ...
            const long reloads = std::min<long>(iters, n_p >= nwg ? (iters * nwg + n_p - 1) / n_p + 1 : iters);
            (void)reloads;  // (the fitted unit cost includes the reloads the timed shapes had)
            const double step_cost = 0.0735 - 0.0053 * at + 0.0522 * bt + 0.0009 * at * bt;
            const double unit_cost = 0.99 + at * bt * (a.res ? 0.453 : 0.358) + steps_pad * step_cost;
            const double cost = 3.99 + iters * unit_cost;
            if (cost < best - 1e-9) best = cost, bft = at, bpt = bt, bwk = -3, ares = true;
        }
    }
    if (ares) {
        op.ft = bft, op.pt = bpt, op.wk = -3;
        op.n_p = (int)((ptiles + STREAM_WAVES * bpt - 1) / (STREAM_WAVES * bpt));
        op.n_units = (int)(((ftiles + bft - 1) / bft) * op.n_p);
        return;
    }
    if (tiled) {
        op.ft = bft, op.pt = bpt, op.wk = 0;
        op.n_p = (int)((ptiles + STREAM_WAVES * bpt - 1) / (STREAM_WAVES * bpt));
        op.n_units = (int)(((ftiles + bft - 1) / bft) * op.n_p);
        return;
    }
    op.ft = bft, op.pt = bpt, op.wk = bwk;
    op.n_p = (int)((ptiles + bpt - 1) / bpt);
    op.n_units = (int)(((ftiles + bft - 1) / bft) * op.n_p);
}

bool tile_dw_op(DevOp &op, int nwg) {
    const ConvArgs &a = op.conv;
    const int cgs = a.K / 8;
    if ((a.K & 7) != 0 || a.C != a.K) return false;
    if ((a.R != 3 && a.R != 5 && a.R != 7) || (a.stride != 1 && a.stride != 2)) return false;
    const int Wp = dw_padded_width(a.W, a.Q, a.R, a.stride);
    const int qblocks = (a.Q + DW_ITEMS - 1) / DW_ITEMS;
    const int ncol = (DW_ITEMS - 1) * a.stride + a.R;
    auto lds_bytes = [&](int rows, int cb) {
        return (long)a.R * a.R * cb * 32 + (long)((rows - 1) * a.stride + a.R) * Wp * cb * 16;
    };
    // clocks ~ rounds x (items per thread x instructions of an item, two waves per SIMD taking turns,
    // plus the batches of four loads that copy the input rows and a fixed part for weights and barriers)
    int best_cb = 0, best_rows = 0;
    double best = 1e30;
    for (int cb = 1; cb <= 4; cb *= 2) {
        const int cblocks = (cgs + cb - 1) / cb;
        for (int rows = 1; rows <= a.P; ++rows) {
            if (lds_bytes(rows, cb) > RED_BYTES) break;
            const long units = (long)a.B * cblocks * ((a.P + rows - 1) / rows);
            const long rounds = (units + nwg - 1) / nwg;
            const long passes = ((long)rows * qblocks * cb + STREAM_THREADS - 1) / STREAM_THREADS;
            const double item = a.R * (ncol * 10.0 + DW_ITEMS * a.R * 8.0 + 30.0) + DW_ITEMS * 40.0;
            const long cells = (long)((rows - 1) * a.stride + a.R) * Wp * cb;
            const double copy = (double)((cells + 4 * STREAM_THREADS - 1) / (4 * STREAM_THREADS)) * 900.0;
            const double cost = rounds * (passes * item * 8.0 + copy + 3000.0);
            if (cost < best) best = cost, best_cb = cb, best_rows = rows;
        }
    }
    // straight from memory: every thread of the team takes items in turn; a tap row costs a load round trip
    // (no other wave of the SIMD may be there to hide it) plus its instructions
    {
        const long items = (long)a.B * cgs * ((a.P + DW_ITEMS - 1) / DW_ITEMS) * a.Q;
        const long per_thread = (items + (long)nwg * STREAM_THREADS - 1) / ((long)nwg * STREAM_THREADS);
        const double row = 2500.0 + (ncol * 10.0 + DW_ITEMS * a.R * 8.0 + a.R * 10.0 + 30.0) * 8.0;
        const double direct = per_thread * (a.R * row + DW_ITEMS * 40.0 * 8.0) + 1000.0;
        if (direct < best) {
            op.wk = -4, op.ft = 1, op.pt = 1, op.n_p = 1, op.n_units = 1;
            return true;
        }
    }
    if (best_cb == 0) return false;
    const int cblocks = (cgs + best_cb - 1) / best_cb;
    op.wk = -2, op.ft = best_cb, op.pt = best_rows;
    op.n_p = (a.P + best_rows - 1) / best_rows;
    op.n_units = a.B * cblocks * op.n_p;
    return true;
}

int fuse_se_blocks(std::vector<DevOp> &prog, const Plan &plan) {
    int fused = 0;
    for (size_t i = 0; i + 3 < prog.size() && i + 3 < plan.ops.size(); ++i) {
        const Op &p = plan.ops[i], &f1 = plan.ops[i + 1], &f2 = plan.ops[i + 2], &g = plan.ops[i + 3];
        if (p.kind != OP_GAP || f1.kind != OP_FC || f2.kind != OP_FC || g.kind != OP_GATE) continue;
        const bool chain = p.out_small && p.out_f32 && f1.in_small && f1.in_buf == p.out_buf && f1.out_small &&
                           f2.in_small && f2.in_buf == f1.out_buf && f2.out_small && f2.hsigmoid &&
                           g.gate_buf == f2.out_buf && g.in_buf == p.in_buf && g.out_buf != g.in_buf && g.out_buf >= 0;
        const bool dims = (p.C & 7) == 0 && p.C <= SE_MAX_C && (f1.K & 7) == 0 && f1.K <= SE_MAX_MID && f1.C == p.C &&
                          f2.C == f1.K && f2.K == p.C && g.C == p.C && g.H == p.H && g.W == p.W && g.B == p.B;
        if (!chain || !dims) continue;
        const DevOp &d0 = prog[i], &d1 = prog[i + 1], &d2 = prog[i + 2], &d3 = prog[i + 3];
        DevOp f{};
        f.kind = DEV_SE;
        f.pt = f.wk = f.ft = 1;
        f.n_units = std::min(p.B, 1 << 30), f.n_p = 1;
        f.relative = d0.relative, f.layer = -1;
        SeArgs &a = f.se;
        a.x = d0.pool.x, a.y = d3.pool.y, a.reserved = nullptr;
        a.w1 = d1.conv.w, a.sc1 = d1.conv.scale, a.sh1 = d1.conv.shift, a.Kpad1 = d1.conv.Kpad;
        a.w2 = d2.conv.w, a.sc2 = d2.conv.scale, a.sh2 = d2.conv.shift, a.Kpad2 = d2.conv.Kpad;
        a.B = p.B, a.HW = p.H * p.W, a.C = p.C, a.mid = f1.K, a.act1 = f1.act;
        f.pool.B = p.B, f.pool.H = p.H, f.pool.W = p.W, f.pool.C = p.C, f.pool.P = p.H, f.pool.Q = p.W;
        prog[i] = f;
        for (int k = 1; k <= 3; ++k) {
            DevOp none{};
            none.kind = DEV_NONE, none.layer = -1, none.pt = none.wk = none.ft = 1;
            prog[i + k] = none;
        }
        fused += 1;
        i += 3;
    }
    return fused;
}

long dev_op_lds_bytes(const DevOp &op) {
    if (op.kind == DEV_SE) return (long)(SE_PART + SE_MAX_C + SE_MAX_MID + SE_MAX_C) * 4;  // partials, averages, hidden, gate
    if (op.kind == DEV_NONE) return 0;
    const ConvArgs &a = op.conv;
    if (op.kind == OP_DW) {
        if (op.wk != -2) return 0;
        const long rows_in = (long)(op.pt - 1) * a.stride + a.R;
        return (long)a.R * a.R * op.ft * 32 + rows_in * dw_padded_width(a.W, a.Q, a.R, a.stride) * op.ft * 16;
    }
    if (op.kind != OP_CONV && op.kind != OP_FC) return 0;
    const long nsteps = (long)a.R * a.R * ((a.C + 31) / 32);
    if (op.wk == -1) return ((long)(op.pt - 1) * a.stride + a.R) * a.W * a.C * 2;  // the band's input rows
    if (op.wk == 0) {  // two weight stages, epilogue constants, step table (one round past the end)
        const int ks = tile_ks(op.pt), round = ks * TILE_SETS;
        const long steps_pad = (nsteps + round - 1) / round * round;
        return 2L * ks * op.ft * 1024 + op.ft * 128 + (steps_pad + round) * 16;
    }
    if (op.wk == -3) {  // the filter group's weights for every step, epilogue constants, step table
        const long steps_pad = (nsteps + ARES_D - 1) / ARES_D * ARES_D;
        return nsteps * op.ft * 1024 + op.ft * 128 + steps_pad * 16;
    }
    if (op.wk > 1) {  // partial sums of the waves: all tiles of a unit, or one filter tile at a time
        const int nt = op.ft * op.pt;
        return (long)STREAM_WAVES * (nt <= 4 ? nt : op.pt) * 1024;
    }
    return 0;
}

bool tile_stem_op(DevOp &op, int nwg) {
    const ConvArgs &a = op.conv;
    if ((a.C & 7) == 0 || a.R * a.R * a.C > 32 * STEM_MAX_KS || a.K > 16 * STEM_MAX_FT || (a.K & 3) != 0 ||
        ((a.W * a.C) & 1) != 0 || a.res != nullptr || a.out_f32)
        return false;
    // rows per band: as many as keep every workgroup busy, within the LDS the input rows may take
    const int bands_wanted = std::max(1, nwg / std::max(1, a.B));
    int rows = (a.P + bands_wanted - 1) / bands_wanted;
    while (rows > 1 && (long)((rows - 1) * a.stride + a.R) * a.W * a.C * 2 > RED_BYTES) --rows;
    if ((long)((rows - 1) * a.stride + a.R) * a.W * a.C * 2 > RED_BYTES) return false;
    op.wk = -1, op.ft = (a.K + 15) / 16, op.pt = rows;
    op.n_p = (a.P + rows - 1) / rows;
    op.n_units = a.B * op.n_p;
    return true;
}

hipError_t launch_stream_kernel(const StreamArgs &a, int nwg, hipStream_t s) {
    hipLaunchKernelGGL(sushi_stream_kernel, dim3(nwg), dim3(STREAM_THREADS), 0, s, a);
    return hipGetLastError();
}

}  // namespace sushi
