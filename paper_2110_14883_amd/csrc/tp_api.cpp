// C ABI of libtplinear (see include/tp_linear.h): argument validation, the partition map
// (paper Section 2.2: chunk shapes [P/q, Q/q], N = S^2 D, [P/p^2, Q/p]; device-count rule),
// launch planning (macro-tile, split of K across workgroups, tile order) and kernel launches.
// Everything is checked before the first launch; nothing is allocated or synchronised here.
#include <algorithm>
#include <atomic>
#include <cstring>

#include "tp_internal.h"

using namespace tpl;

namespace {

constexpr int kCUs = 256;                       // MI355X compute units (8 XCDs x 32): the tile order and the plan assume it
constexpr int64_t kMaxLd = (int64_t)1 << 21;    // keeps every in-tile byte offset below 2^31

// Launch-plan options of one call, resolved from the caller's tp_plan_opts_t (NULL = automatic).
// rotate: -1 automatic (on for the eight-wave kernel, off for the four-wave stream kernel: its workgroups
// of one XCD share operand panels through the L2 only while they walk K in step), 0 off, 1 on.
struct Opts { int tile, split, group, rotate, trim; bool eight_wave; };
int resolve_opts(const tp_plan_opts_t* o, Opts* r) {
    *r = Opts{0, 0, 0, -1, 1, false};
    if (!o) return TP_OK;
    if (o->tile < 0 || o->tile > 5 || o->split_k < 0 || o->split_k > 8 || o->group_m < 0 || o->group_m > 64 ||
        o->rotate < 0 || o->rotate > 2 || o->trim < 0 || o->trim > 2)
        return TP_ERR_MODE;
    r->tile = o->tile == 5 ? (int)TILE_256x256 : o->tile;
    r->eight_wave = o->tile == 5;
    r->split = o->split_k; r->group = o->group_m;
    r->rotate = o->rotate == 0 ? -1 : (o->rotate == 1); r->trim = o->trim != 2;
    return TP_OK;
}

// The device must be the one the kernels are laid out for: checked once per device.
int check_device() {
    static std::atomic<uint64_t> ok_mask{0}, bad_mask{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TP_ERR_HIP;
    const uint64_t bit = 1ull << (dev & 63);
    if (ok_mask.load(std::memory_order_relaxed) & bit) return TP_OK;
    if (bad_mask.load(std::memory_order_relaxed) & bit) return TP_ERR_HIP;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return TP_ERR_HIP;
    (cus == kCUs ? ok_mask : bad_mask).fetch_or(bit, std::memory_order_relaxed);
    return cus == kCUs ? TP_OK : TP_ERR_HIP;
}

struct Chunks { int rc, kc, cc; };              // row chunks of X/Y, col chunks of X (= row chunks of W), col chunks of W/Y

int check_grid(const tp_grid_t* g, Chunks* c) {
    if (g->q < 1 || g->d < 1 || g->p < 1) return TP_ERR_GRID;
    int li = 1, lj = 1, lk = 1;
    switch (g->mode) {
        case TP_MODE_1D_COL: li = g->p; *c = {1, 1, g->p}; if (g->q != 1 || g->d != 1) return TP_ERR_GRID; break;
        case TP_MODE_1D_ROW: li = g->p; *c = {1, g->p, 1}; if (g->q != 1 || g->d != 1) return TP_ERR_GRID; break;
        case TP_MODE_2D:     li = lj = g->q; *c = {g->q, g->q, g->q}; if (g->p != 1 || g->d != 1) return TP_ERR_GRID; break;
        case TP_MODE_2P5D:   li = lj = g->q; lk = g->d; *c = {g->q * g->d, g->q, g->q}; if (g->p != 1) return TP_ERR_GRID; break;
        case TP_MODE_3D:     li = lj = lk = g->p; *c = {g->p * g->p, g->p, g->p}; if (g->q != 1 || g->d != 1) return TP_ERR_GRID; break;
        case TP_MODE_3D_GATHERED: li = lj = lk = g->p; *c = {g->p, g->p, g->p}; if (g->q != 1 || g->d != 1) return TP_ERR_GRID; break;
        default: return TP_ERR_MODE;
    }
    if (g->ri < 0 || g->ri >= li || g->rj < 0 || g->rj >= lj || g->rk < 0 || g->rk >= lk) return TP_ERR_GRID;
    return TP_OK;
}

struct Share {           // one pass of one rank
    int n_steps; int64_t m, n, k;
    int a_row[TP_MAX_STEPS], a_col[TP_MAX_STEPS], b_row[TP_MAX_STEPS], b_col[TP_MAX_STEPS];
    int out_row, out_col, partial;
};

int build_share(const tp_grid_t* g, const tp_dims_t* d, int pass, Share* s) {
    if (!g || !d || !s) return TP_ERR_NULL;
    if (pass != TP_PASS_FWD && pass != TP_PASS_DX && pass != TP_PASS_DW) return TP_ERR_MODE;
    Chunks c;
    if (int e = check_grid(g, &c)) return e;
    if (d->M < 1 || d->H < 1 || d->F < 1) return TP_ERR_SHAPE;
    if (d->M % c.rc || d->H % c.kc || d->F % c.cc) return TP_ERR_SHAPE;
    // the gathered slabs are made of p stored chunks [M/p^2, .]
    if (g->mode == TP_MODE_3D_GATHERED && d->M % ((int64_t)g->p * g->p)) return TP_ERR_SHAPE;
    const int64_t mb = d->M / c.rc, hb = d->H / c.kc, fb = d->F / c.cc;
    std::memset(s, 0, sizeof(*s));
    if (g->mode == TP_MODE_3D_GATHERED) {
        const int i = g->ri, j = g->rj, l = g->rk;
        s->n_steps = 1; s->partial = g->p > 1;
        if (pass == TP_PASS_FWD)     { s->m = mb; s->n = fb; s->k = hb; s->a_row[0] = i; s->a_col[0] = l; s->b_row[0] = l; s->b_col[0] = j; s->out_row = i; s->out_col = j; }
        else if (pass == TP_PASS_DX) { s->m = mb; s->n = hb; s->k = fb; s->a_row[0] = i; s->a_col[0] = j; s->b_row[0] = l; s->b_col[0] = j; s->out_row = i; s->out_col = l; }
        else                         { s->m = hb; s->n = fb; s->k = mb; s->a_row[0] = i; s->a_col[0] = l; s->b_row[0] = i; s->b_col[0] = j; s->out_row = l; s->out_col = j; }
        return TP_OK;
    }
    int steps = 1, row = 0, col = 0, wrow = 0;     // own row chunk, own column index, dW's row chunk
    int first_row = 0;                             // first row chunk of the group dW sums over
    switch (g->mode) {
        case TP_MODE_1D_COL: case TP_MODE_1D_ROW: steps = 1; break;
        case TP_MODE_2D:   steps = g->q; row = g->ri; col = g->rj; wrow = g->ri; first_row = 0; break;
        case TP_MODE_2P5D: steps = g->q; row = g->rk * g->q + g->ri; col = g->rj; wrow = g->ri; first_row = g->rk * g->q; break;
        case TP_MODE_3D:   steps = g->p; row = g->ri * g->p + g->rk; col = g->rj; wrow = g->rk; first_row = g->ri * g->p; break;
    }
    if (steps > TP_MAX_STEPS) return TP_ERR_GRID;
    s->n_steps = steps;
    if (g->mode == TP_MODE_1D_COL) {
        const int r = g->ri;
        if (pass == TP_PASS_FWD)      { s->m = mb; s->n = fb; s->k = hb; s->a_col[0] = 0; s->b_col[0] = r; s->out_col = r; }
        else if (pass == TP_PASS_DX)  { s->m = mb; s->n = hb; s->k = fb; s->a_col[0] = r; s->b_col[0] = r; s->partial = g->p > 1; }
        else                          { s->m = hb; s->n = fb; s->k = mb; s->b_col[0] = r; s->out_col = r; }
        return TP_OK;
    }
    if (g->mode == TP_MODE_1D_ROW) {
        const int r = g->ri;
        if (pass == TP_PASS_FWD)      { s->m = mb; s->n = fb; s->k = hb; s->a_col[0] = r; s->b_row[0] = r; s->partial = g->p > 1; }
        else if (pass == TP_PASS_DX)  { s->m = mb; s->n = hb; s->k = fb; s->b_row[0] = r; s->out_col = r; }
        else                          { s->m = hb; s->n = fb; s->k = mb; s->a_col[0] = r; s->out_row = r; }
        return TP_OK;
    }
    for (int k = 0; k < steps; ++k) {
        if (pass == TP_PASS_FWD)     { s->a_row[k] = row; s->a_col[k] = k; s->b_row[k] = k; s->b_col[k] = col; }
        else if (pass == TP_PASS_DX) { s->a_row[k] = row; s->a_col[k] = k; s->b_row[k] = col; s->b_col[k] = k; }
        else                         { s->a_row[k] = first_row + k; s->a_col[k] = wrow; s->b_row[k] = first_row + k; s->b_col[k] = col; }
    }
    if (pass == TP_PASS_FWD)     { s->m = mb; s->n = fb; s->k = hb; s->out_row = row; s->out_col = col; }
    else if (pass == TP_PASS_DX) { s->m = mb; s->n = hb; s->k = fb; s->out_row = row; s->out_col = col; }
    else {
        s->m = hb; s->n = fb; s->k = mb; s->out_row = wrow; s->out_col = col;
        s->partial = (g->mode == TP_MODE_2P5D && g->d > 1) || (g->mode == TP_MODE_3D && g->p > 1);
    }
    return TP_OK;
}

struct PartialsShare {   // the backward products as partials for other owners (2D, 2.5D)
    int n_steps; int64_t m, n, k;
    int own_row, own_col;
    int other_row[TP_MAX_STEPS], other_col[TP_MAX_STEPS], out_row[TP_MAX_STEPS], out_col[TP_MAX_STEPS];
};

int build_partials(const tp_grid_t* g, const tp_dims_t* d, int pass, PartialsShare* s) {
    if (!g || !d || !s) return TP_ERR_NULL;
    if (pass != TP_PASS_DX_PARTIALS && pass != TP_PASS_DW_PARTIALS) return TP_ERR_MODE;
    if (g->mode != TP_MODE_2D && g->mode != TP_MODE_2P5D) return TP_ERR_MODE;
    Chunks c;
    if (int e = check_grid(g, &c)) return e;
    if (d->M < 1 || d->H < 1 || d->F < 1) return TP_ERR_SHAPE;
    if (d->M % c.rc || d->H % c.kc || d->F % c.cc) return TP_ERR_SHAPE;
    if (g->q > TP_MAX_STEPS) return TP_ERR_GRID;
    const int64_t mb = d->M / c.rc, hb = d->H / c.kc, fb = d->F / c.cc;
    std::memset(s, 0, sizeof(*s));
    const int row = (g->mode == TP_MODE_2P5D ? g->rk * g->q : 0) + g->ri, col = g->rj;
    s->n_steps = g->q; s->own_row = row; s->own_col = col;
    for (int k = 0; k < g->q; ++k) {
        if (pass == TP_PASS_DX_PARTIALS) { s->other_row[k] = k; s->other_col[k] = col; s->out_row[k] = row; s->out_col[k] = k; }
        else                             { s->other_row[k] = row; s->other_col[k] = k; s->out_row[k] = k; s->out_col[k] = col; }
    }
    if (pass == TP_PASS_DX_PARTIALS) { s->m = mb; s->n = hb; s->k = fb; }
    else                             { s->m = hb; s->n = fb; s->k = mb; }
    return TP_OK;
}

struct Plan {
    int tile_id, bm, bn, tiles_m, tiles_n, split_k, group_m, groups;
    // Tail trimming: when the tile count is a little more than a whole number of rounds of the 256
    // persistent workgroups, the last tile rows are cut off and run as a second, small launch with a
    // plan of their own, so that the main launch ends on a full round.  m_main = rows of the main launch
    // (0 = not trimmed); the tail covers rows [m_main, m).
    int64_t m_main;
    int tail_tile_id, tail_tiles_m, tail_tiles_n, tail_split;
};

// Measured costs in shader cycles.  One 64-deep K tile of one workgroup: the four-wave stream kernel
// (256 x 256) takes 2500 - 2900 against 2048 of pure MFMA issue; the eight-wave kernel's half and
// quarter tiles move more bytes per flop and take ~2200 and ~1400.  On top of that every C tile has
// a fixed cost: the epilogue alone for the stream kernel (its K tiles keep flowing across C tiles),
// epilogue plus pipeline refill for the others.
double k_tile_cycles(int bm, int bn) { return bm * bn == 65536 ? 2730.0 : (bm * bn == 32768 ? 2220.0 : 1410.0); }
double c_tile_cycles(int bm, int bn) { return bm * bn == 65536 ? 12000.0 : 20000.0; }

// Pick the macro-tile and the split of K so that the launch fills whole waves of the 256 CUs.
// Cost model: (waves of workgroups) x (K tiles per workgroup) x (tile area), plus the fp32
// round trip of the partials when K is split.
// groups > 1: that many products of the same extents share one launch (tiles_m, tiles_n stay per product).
Plan plan_whole(const Opts& o, int64_t m, int64_t n, int64_t k, int n_steps, int groups, double* cost_out) {
    const int64_t T = (int64_t)n_steps * ((k + 63) / 64);
    Plan best{};
    double best_cost = 1e300;
    const int tile_ids[4] = {TILE_256x256, TILE_128x256, TILE_256x128, TILE_128x128};
    const int forced_split = o.split, forced_tile = o.tile;
    for (int ti = 0; ti < 4; ++ti) {
        if (forced_tile && tile_ids[ti] != forced_tile) continue;
        int bm, bn;
        tile_shape(tile_ids[ti], &bm, &bn);
        const int64_t tm = (m + bm - 1) / bm, tn = (n + bn - 1) / bn;
        const int64_t tiles = tm * tn * groups;
        const double tile_cycles = k_tile_cycles(bm, bn);
        const double per_tile = c_tile_cycles(bm, bn);
        for (int z = 1; z <= 8; ++z) {
            if (forced_split && z != forced_split) continue;
            if (z > T) break;
            const int64_t waves = (tiles * z + kCUs - 1) / kCUs;
            const double main_cost = (double)waves * ((double)((T + z - 1) / z) * tile_cycles + per_tile);
            // partials: z fp32 planes written and read back at ~1.6 KB/clk, plus one more launch
            const double fix = z > 1 ? ((double)m * n * 8.0 * z / 1667.0 + 12000.0) * groups : 0.0;
            const double cost = main_cost + fix;
            if (cost < best_cost) {
                best_cost = cost;
                best = Plan{tile_ids[ti], bm, bn, (int)tm, (int)tn, z, 4, groups, 0, 0, 0, 0, 0};
            }
        }
    }
    if (best.tile_id == 0) {           // overrides left nothing admissible: fall back to the safe default
        best = Plan{TILE_256x256, 256, 256, (int)((m + 255) / 256), (int)((n + 255) / 256), 1, 4, groups, 0, 0, 0, 0, 0};
    }
    best.group_m = o.group > 0 ? o.group : 4;
    if (cost_out) *cost_out = best_cost;
    return best;
}

// cycles of one C tile of the given shape over T K tiles (the cost model's unit, see plan_whole)
double tile_cost(int bm, int bn, int64_t T) { return (double)T * k_tile_cycles(bm, bn) + c_tile_cycles(bm, bn); }

Plan make_plan(const Opts& o, int64_t m, int64_t n, int64_t k, int n_steps, int groups = 1) {
    double whole_cost = 0.0;
    Plan best = plan_whole(o, m, n, k, n_steps, groups, &whole_cost);
    if (groups != 1 || !o.trim || o.split > 1) return best;
    const int64_t T = (int64_t)n_steps * ((k + 63) / 64);
    const int tile_ids[4] = {TILE_256x256, TILE_128x256, TILE_256x128, TILE_128x128};
    const int forced_tile = o.tile;
    double best_cost = whole_cost;
    for (int ti = 0; ti < 4; ++ti) {
        if (forced_tile && tile_ids[ti] != forced_tile) continue;
        int bm, bn;
        tile_shape(tile_ids[ti], &bm, &bn);
        const int64_t tm = (m + bm - 1) / bm, tn = (n + bn - 1) / bn;
        const int64_t tiles = tm * tn, rem = tiles % kCUs;
        if (tiles <= kCUs || rem == 0 || rem % tn != 0) continue;      // the tail must be whole tile rows
        const int64_t tail_rows_tiles = rem / tn;
        if (tail_rows_tiles >= tm) continue;
        const int64_t m_main = (tm - tail_rows_tiles) * bm;
        double tail_cost = 0.0;
        const Plan tail = plan_whole(o, m - m_main, n, k, n_steps, 1, &tail_cost);
        const double cost = (double)((tiles - rem) / kCUs) * tile_cost(bm, bn, T) + tail_cost + 15000.0;   // + one more launch
        if (cost < best_cost) {
            best_cost = cost;
            best = Plan{tile_ids[ti], bm, bn, (int)(tm - tail_rows_tiles), (int)tn, 1, best.group_m, 1,
                        m_main, tail.tile_id, tail.tiles_m, tail.tiles_n, tail.split_k};
        }
    }
    return best;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_cblk(const tp_cblk_t& b, int64_t cols) {
    if (!b.ptr) return TP_ERR_NULL;
    if (!aligned16(b.ptr) || (b.ld & 7) || (cols & 7)) return TP_ERR_ALIGN;
    if (b.ld < cols || b.ld > kMaxLd) return TP_ERR_SHAPE;
    return TP_OK;
}
int check_oblk(const tp_oblk_t& b, int64_t cols, bool f32_only) {
    if (!b.ptr) return TP_ERR_NULL;
    if (b.dtype != TP_BF16 && b.dtype != TP_F32) return TP_ERR_DTYPE;
    if (f32_only && b.dtype != TP_F32) return TP_ERR_DTYPE;
    if (!aligned16(b.ptr) || (b.ld & 7) || (cols & 7)) return TP_ERR_ALIGN;
    if (b.ld < cols) return TP_ERR_SHAPE;
    return TP_OK;
}

size_t ws_bytes_for(const Plan& p, int64_t m, int64_t n) {
    if (p.m_main > 0)              // the main launch never splits K; the tail may
        return p.tail_split > 1 ? (size_t)p.tail_split * (size_t)(m - p.m_main) * (size_t)n * sizeof(float) : 0;
    return p.split_k > 1 ? (size_t)p.split_k * (size_t)p.groups * (size_t)m * (size_t)n * sizeof(float) : 0;
}

struct Product {                 // one validated GEMM ready to launch
    int form; Plan plan; GemmArgs args; bool active;
};

// The four-wave stream kernel keeps one buffer descriptor per (C tile, step) and moves 32-bit lane
// offsets along K: every offset it can form must stay below 2^31.
bool w4_eligible(int form, const GemmArgs& a) {
    const bool a_kc = form != FORM_TN, b_kc = form == FORM_NT;
    const int slots = a.n_groups > 1 ? a.n_groups : a.n_steps;
    for (int s = 0; s < slots; ++s) {
        const int64_t lda = a.lda[s], ldb = a.ldb[s], K = a.K;
        if (a_kc ? (255 * lda + K) * 2 >= ((int64_t)1 << 31) : (K * lda + 256) * 2 >= ((int64_t)1 << 31)) return false;
        if (b_kc ? (255 * ldb + K) * 2 >= ((int64_t)1 << 31) : (K * ldb + 256) * 2 >= ((int64_t)1 << 31)) return false;
    }
    // its epilogue addresses a wave's 128 rows of every output (and of the GeLU' operand) the same way
    const int64_t lim = (int64_t)1 << 31, N = a.N;
    const int groups = a.n_groups > 1 ? a.n_groups : 1;
    for (int g = 0; g < groups; ++g) {
        const int64_t ldo = a.n_groups > 1 ? a.ldos[g] : a.ldo;
        if ((128 * ldo + N) * 4 >= lim) return false;
    }
    if (a.pre && (128 * a.ldp + N) * 2 >= lim) return false;
    if (a.dg && (128 * a.lddg + N) * 2 >= lim) return false;
    if (129 * N * 4 >= lim) return false;          // split-K planes
    return true;
}

int run_one(const Opts& o, int form, int tile_id, int split_k, const GemmArgs& a, hipStream_t stream) {
    // 256 x 256 tiles run on the four-wave stream kernel unless the eight-wave one is asked for
    if (tile_id == TILE_256x256 && !o.eight_wave && w4_eligible(form, a)) tile_id = TILE_256x256_W4;
    GemmArgs la = a;
    la.rotate = o.rotate < 0 ? (tile_id != TILE_256x256_W4) : o.rotate;
    if (launch_gemm(form, tile_id, la, stream) != hipSuccess) return TP_ERR_HIP;
    if (split_k > 1) {
        const int groups = a.n_groups > 1 ? a.n_groups : 1;
        const int64_t mn = (int64_t)a.M * a.N;
        for (int g = 0; g < groups; ++g) {
            void* out = groups > 1 ? a.outs[g] : a.out;
            const int64_t ldo = groups > 1 ? a.ldos[g] : a.ldo;
            ReduceArgs r{a.ws + g * mn, mn * groups, a.split_k, a.M, a.N, out, ldo, a.out_f32, a.pre, a.ldp, a.bias, a.gelu, a.dg, a.lddg};
            if (launch_reduce(r, stream) != hipSuccess) return TP_ERR_HIP;
        }
    }
    return TP_OK;
}

int run_product(const Opts& o, const Product& pr, void* workspace, hipStream_t stream) {
    GemmArgs a = pr.args;
    a.ws = static_cast<float*>(workspace);
    const Plan& pl = pr.plan;
    if (pl.m_main <= 0) return run_one(o, pr.form, pl.tile_id, pl.split_k, a, stream);
    // main launch: rows [0, m_main), a whole number of rounds
    const int64_t m = a.M, m0 = pl.m_main;
    GemmArgs mainp = a;
    mainp.M = (int32_t)m0;
    if (int e = run_one(o, pr.form, pl.tile_id, 1, mainp, stream)) return e;
    // tail launch: rows [m_main, m) through shifted pointers, with its own tile shape and K split
    GemmArgs tail = a;
    tail.M = (int32_t)(m - m0);
    tail.tiles_m = pl.tail_tiles_m; tail.tiles_n = pl.tail_tiles_n; tail.split_k = pl.tail_split;
    for (int k = 0; k < a.n_steps; ++k) {
        const char* ap = static_cast<const char*>(a.a[k]);
        tail.a[k] = pr.form == FORM_TN ? ap + m0 * 2 : ap + m0 * (int64_t)a.lda[k] * 2;    // TN: A is [k][m], else [m][k]
    }
    tail.out = static_cast<char*>(a.out) + m0 * a.ldo * (a.out_f32 ? 4 : 2);
    if (a.pre) tail.pre = static_cast<char*>(a.pre) + m0 * a.ldp * 2;
    if (a.dg) tail.dg = static_cast<const char*>(a.dg) + m0 * a.lddg * 2;
    return run_one(o, pr.form, pl.tail_tile_id, pl.tail_split, tail, stream);
}

void fill_common(const Opts& o, GemmArgs& a, const Plan& p, int64_t m, int64_t n, int64_t k, int n_steps) {
    std::memset(&a, 0, sizeof(a));
    a.M = (int32_t)m; a.N = (int32_t)n; a.K = (int32_t)k; a.n_steps = n_steps;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.split_k = p.split_k; a.group_m = p.group_m;
    a.max_workgroups = kCUs;
    a.rotate = o.rotate;                       // (run_one resolves "automatic" once it knows the kernel)
}

bool ws_ok(size_t need, const void* workspace, size_t bytes) {
    return need == 0 || (workspace && bytes >= need && aligned16(workspace));
}

// byte range of an fp32 output block [rows, cols] with leading dimension ld
struct Range { uintptr_t lo, hi; };
Range out_range(const tp_oblk_t& b, int64_t rows, int64_t cols) {
    const uintptr_t lo = reinterpret_cast<uintptr_t>(b.ptr);
    return Range{lo, lo + (uintptr_t)(((rows - 1) * b.ld + cols) * 4)};
}
bool overlap(const Range& a, const Range& b) { return a.lo < b.hi && b.lo < a.hi; }

// ---------------------------------------------------------------------------------------------
// Built-in scratch for tp_linear_fwd_static: a fixed array in device memory (every GPU the library
// runs on holds its own copy until the process ends).  Host code never uses the array's name as an
// address: the address on the current device is asked for once per device and kept.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TP_ERR_HIP;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TP_ERR_HIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);      // (two threads racing here store the same address)
    }
    *out = ptr;
    return TP_OK;
}

int linear_fwd(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps, const tp_cblk_t* x_blocks,
               const tp_cblk_t* w_blocks, const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
               void* workspace, size_t workspace_bytes, void* hip_stream, const tp_plan_opts_t* opts,
               bool use_static_scratch) {
    Opts o;

    if (int e = resolve_opts(opts, &o)) return e;
    Share s;
    if (int e = build_share(grid, dims, TP_PASS_FWD, &s)) return e;
    if (!x_blocks || !w_blocks) return TP_ERR_NULL;
    if (n_steps < 1 || n_steps > s.n_steps) return TP_ERR_SHAPE;
    if (epi != TP_EPI_NONE && epi != TP_EPI_BIAS && epi != TP_EPI_BIAS_GELU) return TP_ERR_MODE;
    if (epi != TP_EPI_NONE && !bias) return TP_ERR_NULL;
    if (bias && !aligned16(bias)) return TP_ERR_ALIGN;
    if (s.partial) {                    // an additive partial: bias and GeLU come after the summation
        if (epi != TP_EPI_NONE || preact.ptr) return TP_ERR_MODE;
        if (y.ptr && y.dtype != TP_F32) return TP_ERR_DTYPE;
    }
    if (s.m > INT32_MAX || s.n > INT32_MAX || s.k > INT32_MAX) return TP_ERR_SHAPE;
    for (int k = 0; k < n_steps; ++k) {
        if (int e = check_cblk(x_blocks[k], s.k)) return e;
        if (int e = check_cblk(w_blocks[k], s.n)) return e;
    }
    if (int e = check_oblk(y, s.n, false)) return e;
    if (preact.ptr) {
        if (int e = check_oblk(preact, s.n, false)) return e;
        if (preact.dtype != TP_BF16) return TP_ERR_DTYPE;
    }
    Plan p = make_plan(o, s.m, s.n, s.k, n_steps);
    if (use_static_scratch) {
        if (ws_bytes_for(p, s.m, s.n) > kStaticScratchBytes) return TP_ERR_SCRATCH;
    } else if (!ws_ok(ws_bytes_for(p, s.m, s.n), workspace, workspace_bytes)) {
        return TP_ERR_WORKSPACE;
    }
    if (int e = check_device()) return e;
    if (use_static_scratch) {
        if (int e = static_scratch(&workspace)) return e;
    }

    Product pr{};
    pr.form = FORM_NN; pr.plan = p;
    fill_common(o, pr.args, p, s.m, s.n, s.k, n_steps);
    for (int k = 0; k < n_steps; ++k) {
        pr.args.a[k] = x_blocks[k].ptr; pr.args.lda[k] = (int32_t)x_blocks[k].ld;
        pr.args.b[k] = w_blocks[k].ptr; pr.args.ldb[k] = (int32_t)w_blocks[k].ld;
    }
    pr.args.out = y.ptr; pr.args.ldo = y.ld; pr.args.out_f32 = y.dtype == TP_F32;
    pr.args.pre = preact.ptr; pr.args.ldp = preact.ld;
    pr.args.bias = epi == TP_EPI_NONE ? nullptr : bias;
    pr.args.gelu = epi == TP_EPI_BIAS_GELU;
    return run_product(o, pr, workspace, static_cast<hipStream_t>(hip_stream));
}

}  // namespace

extern "C" {

int tp_block_map(const tp_grid_t* grid, const tp_dims_t* dims, int pass, int* n_steps, int64_t* m, int64_t* n,
                 int64_t* k_per_step, int* a_row, int* a_col, int* b_row, int* b_col, int* out_row, int* out_col,
                 int* is_partial) {
    Share s;
    if (int e = build_share(grid, dims, pass, &s)) return e;
    if (n_steps) *n_steps = s.n_steps;
    if (m) *m = s.m;
    if (n) *n = s.n;
    if (k_per_step) *k_per_step = s.k;
    for (int i = 0; i < TP_MAX_STEPS; ++i) {
        if (a_row) a_row[i] = s.a_row[i];
        if (a_col) a_col[i] = s.a_col[i];
        if (b_row) b_row[i] = s.b_row[i];
        if (b_col) b_col[i] = s.b_col[i];
    }
    if (out_row) *out_row = s.out_row;
    if (out_col) *out_col = s.out_col;
    if (is_partial) *is_partial = s.partial;
    return TP_OK;
}

size_t tp_linear_workspace_size_ex(const tp_grid_t* grid, const tp_dims_t* dims, int pass, const tp_plan_opts_t* opts) {
    Opts o;
    if (resolve_opts(opts, &o) != TP_OK) return 0;
    if (pass == TP_PASS_DX_PARTIALS || pass == TP_PASS_DW_PARTIALS) {
        PartialsShare ps;
        if (build_partials(grid, dims, pass, &ps) != TP_OK) return 0;
        size_t worst = 0;               // any number of products 1 .. n_steps may be asked for
        for (int groups = 1; groups <= ps.n_steps; ++groups)
            worst = std::max(worst, ws_bytes_for(make_plan(o, ps.m, ps.n, ps.k, 1, groups), ps.m, ps.n));
        return worst;
    }
    Share s;
    if (build_share(grid, dims, pass, &s) != TP_OK) return 0;
    size_t worst = 0;                   // any prefix 1 .. n_steps of the steps may be asked for
    for (int steps = 1; steps <= s.n_steps; ++steps)
        worst = std::max(worst, ws_bytes_for(make_plan(o, s.m, s.n, s.k, steps), s.m, s.n));
    Share sf;                           // the bias gradient of tp_linear_bwd sums the forward block's columns in two passes
    if (pass != TP_PASS_FWD && build_share(grid, dims, TP_PASS_FWD, &sf) == TP_OK)
        worst = std::max(worst, colsum_ws_bytes(sf.m, sf.n));
    return worst;
}

size_t tp_linear_workspace_size(const tp_grid_t* grid, const tp_dims_t* dims, int pass) {
    return tp_linear_workspace_size_ex(grid, dims, pass, nullptr);
}

int tp_linear_fwd_ex(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps, const tp_cblk_t* x_blocks,
                     const tp_cblk_t* w_blocks, const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
                     void* workspace, size_t workspace_bytes, void* hip_stream, const tp_plan_opts_t* opts) {
    return linear_fwd(grid, dims, n_steps, x_blocks, w_blocks, bias, epi, y, preact, workspace, workspace_bytes, hip_stream,
                      opts, false);
}

int tp_linear_fwd_static(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps, const tp_cblk_t* x_blocks,
                         const tp_cblk_t* w_blocks, const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
                         void* hip_stream) {
    return linear_fwd(grid, dims, n_steps, x_blocks, w_blocks, bias, epi, y, preact, nullptr, 0, hip_stream, nullptr, true);
}

size_t tp_static_scratch_bytes(void) { return kStaticScratchBytes; }

int tp_linear_fwd(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps, const tp_cblk_t* x_blocks,
                  const tp_cblk_t* w_blocks, const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
                  void* workspace, size_t workspace_bytes, void* hip_stream) {
    return tp_linear_fwd_ex(grid, dims, n_steps, x_blocks, w_blocks, bias, epi, y, preact, workspace, workspace_bytes,
                            hip_stream, nullptr);
}

int tp_linear_bwd_ex(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps_dx, int n_steps_dw,
                     const tp_cblk_t* dy_own, const tp_cblk_t* preact_own, const tp_cblk_t* da_row_blocks,
                     const tp_cblk_t* w_blocks_dx, const tp_cblk_t* x_blocks_dw, const tp_cblk_t* da_col_blocks,
                     int own_slot_dx, int own_slot_dw, const tp_cblk_t* dgelu_preact, tp_oblk_t dx, tp_oblk_t dw,
                     tp_oblk_t da_own_out, void* db_f32, void* workspace, size_t workspace_bytes, void* hip_stream,
                     const tp_plan_opts_t* opts) {
    Opts o;
    if (int e = resolve_opts(opts, &o)) return e;
    Share sf, sx, sw;
    if (int e = build_share(grid, dims, TP_PASS_FWD, &sf)) return e;
    if (int e = build_share(grid, dims, TP_PASS_DX, &sx)) return e;
    if (int e = build_share(grid, dims, TP_PASS_DW, &sw)) return e;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (sf.m > INT32_MAX || sf.n > INT32_MAX || sf.k > INT32_MAX) return TP_ERR_SHAPE;

    // ---- (1) own dA
    const bool want_da = da_own_out.ptr != nullptr;
    if (want_da) {
        if (!dy_own || !preact_own) return TP_ERR_NULL;
        if (int e = check_cblk(*dy_own, sf.n)) return e;
        if (int e = check_cblk(*preact_own, sf.n)) return e;
        if (int e = check_oblk(da_own_out, sf.n, false)) return e;
        if (da_own_out.dtype != TP_BF16) return TP_ERR_DTYPE;
        if (da_own_out.ld > kMaxLd) return TP_ERR_SHAPE;
    } else if (db_f32 || own_slot_dx >= 0 || own_slot_dw >= 0) {
        return TP_ERR_NULL;                      // both need the dA that only part (1) produces
    }
    if (db_f32 && !aligned16(db_f32)) return TP_ERR_ALIGN;
    const tp_cblk_t own_blk{da_own_out.ptr, da_own_out.ld};

    // ---- (2) dX
    Product px{}; px.active = dx.ptr != nullptr;
    if (px.active) {
        if (!da_row_blocks || !w_blocks_dx) return TP_ERR_NULL;
        if (n_steps_dx < 1 || n_steps_dx > sx.n_steps) return TP_ERR_SHAPE;
        if (own_slot_dx >= n_steps_dx) return TP_ERR_SHAPE;
        if (sx.partial) {               // a summand of a reduction: fp32, and GeLU' belongs after the sum
            if (dgelu_preact) return TP_ERR_MODE;
            if (dx.dtype != TP_F32) return TP_ERR_DTYPE;
        }
        Plan p = make_plan(o, sx.m, sx.n, sx.k, n_steps_dx);
        fill_common(o, px.args, p, sx.m, sx.n, sx.k, n_steps_dx);
        for (int k = 0; k < n_steps_dx; ++k) {
            const tp_cblk_t& a = (k == own_slot_dx) ? own_blk : da_row_blocks[k];
            if (int e = check_cblk(a, sx.k)) return e;
            if (int e = check_cblk(w_blocks_dx[k], sx.k)) return e;       // W block is [n = H_blk][k = F_blk]
            px.args.a[k] = a.ptr; px.args.lda[k] = (int32_t)a.ld;
            px.args.b[k] = w_blocks_dx[k].ptr; px.args.ldb[k] = (int32_t)w_blocks_dx[k].ld;
        }
        if (int e = check_oblk(dx, sx.n, false)) return e;
        if (dgelu_preact) {
            if (int e = check_cblk(*dgelu_preact, sx.n)) return e;
            px.args.dg = dgelu_preact->ptr; px.args.lddg = dgelu_preact->ld;
        }
        px.args.out = dx.ptr; px.args.ldo = dx.ld; px.args.out_f32 = dx.dtype == TP_F32;
        px.form = FORM_NT; px.plan = p;
    }
    // ---- (3) dW
    Product pw{}; pw.active = dw.ptr != nullptr;
    if (pw.active) {
        if (!x_blocks_dw || !da_col_blocks) return TP_ERR_NULL;
        if (n_steps_dw < 1 || n_steps_dw > sw.n_steps) return TP_ERR_SHAPE;
        if (own_slot_dw >= n_steps_dw) return TP_ERR_SHAPE;
        Plan p = make_plan(o, sw.m, sw.n, sw.k, n_steps_dw);
        fill_common(o, pw.args, p, sw.m, sw.n, sw.k, n_steps_dw);
        for (int k = 0; k < n_steps_dw; ++k) {
            const tp_cblk_t& b = (k == own_slot_dw) ? own_blk : da_col_blocks[k];
            if (int e = check_cblk(x_blocks_dw[k], sw.m)) return e;       // X block is [k = tokens][m = H_blk]
            if (int e = check_cblk(b, sw.n)) return e;
            pw.args.a[k] = x_blocks_dw[k].ptr; pw.args.lda[k] = (int32_t)x_blocks_dw[k].ld;
            pw.args.b[k] = b.ptr; pw.args.ldb[k] = (int32_t)b.ld;
        }
        if (int e = check_oblk(dw, sw.n, true)) return e;
        pw.args.out = dw.ptr; pw.args.ldo = dw.ld; pw.args.out_f32 = 1;
        pw.form = FORM_TN; pw.plan = p;
    }
    size_t need = 0;
    if (px.active) need = std::max(need, ws_bytes_for(px.plan, sx.m, sx.n));
    if (pw.active) need = std::max(need, ws_bytes_for(pw.plan, sw.m, sw.n));
    if (!ws_ok(need, workspace, workspace_bytes)) return TP_ERR_WORKSPACE;
    if (want_da || px.active || pw.active)
        if (int e = check_device()) return e;

    // ---- launches (stream order: dA, db, dX, dW)
    if (want_da) {
        if (launch_dgelu(dy_own->ptr, dy_own->ld, preact_own->ptr, preact_own->ld, da_own_out.ptr, da_own_out.ld,
                         sf.m, sf.n, stream) != hipSuccess) return TP_ERR_HIP;
        // (two passes over row slabs when the workspace holds the slab sums, else one workgroup per 64 columns)
        float* const cws = (workspace && aligned16(workspace) && workspace_bytes >= colsum_ws_bytes(sf.m, sf.n))
                               ? static_cast<float*>(workspace) : nullptr;
        if (db_f32 && launch_colsum(da_own_out.ptr, da_own_out.ld, sf.m, sf.n, static_cast<float*>(db_f32), cws, stream) != hipSuccess)
            return TP_ERR_HIP;
    }
    if (px.active) if (int e = run_product(o, px, workspace, stream)) return e;
    if (pw.active) if (int e = run_product(o, pw, workspace, stream)) return e;
    return TP_OK;
}

int tp_linear_bwd(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps_dx, int n_steps_dw,
                  const tp_cblk_t* dy_own, const tp_cblk_t* preact_own, const tp_cblk_t* da_row_blocks,
                  const tp_cblk_t* w_blocks_dx, const tp_cblk_t* x_blocks_dw, const tp_cblk_t* da_col_blocks,
                  int own_slot_dx, int own_slot_dw, const tp_cblk_t* dgelu_preact, tp_oblk_t dx, tp_oblk_t dw,
                  tp_oblk_t da_own_out, void* db_f32, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return tp_linear_bwd_ex(grid, dims, n_steps_dx, n_steps_dw, dy_own, preact_own, da_row_blocks, w_blocks_dx,
                            x_blocks_dw, da_col_blocks, own_slot_dx, own_slot_dw, dgelu_preact, dx, dw, da_own_out,
                            db_f32, workspace, workspace_bytes, hip_stream, nullptr);
}

int tp_partials_map(const tp_grid_t* grid, const tp_dims_t* dims, int pass, int* n_steps, int64_t* m, int64_t* n,
                    int64_t* k, int* own_row, int* own_col, int* other_row, int* other_col, int* out_row, int* out_col) {
    PartialsShare s;
    if (int e = build_partials(grid, dims, pass, &s)) return e;
    if (n_steps) *n_steps = s.n_steps;
    if (m) *m = s.m;
    if (n) *n = s.n;
    if (k) *k = s.k;
    if (own_row) *own_row = s.own_row;
    if (own_col) *own_col = s.own_col;
    for (int i = 0; i < TP_MAX_STEPS; ++i) {
        if (other_row) other_row[i] = s.other_row[i];
        if (other_col) other_col[i] = s.other_col[i];
        if (out_row) out_row[i] = s.out_row[i];
        if (out_col) out_col[i] = s.out_col[i];
    }
    return TP_OK;
}

int tp_linear_bwd_partials_ex(const tp_grid_t* grid, const tp_dims_t* dims, int n_dx, int n_dw, const tp_cblk_t* da_own,
                              const tp_cblk_t* w_blocks_dx, const tp_oblk_t* dx_partials, const tp_cblk_t* x_blocks_dw,
                              const tp_oblk_t* dw_partials, void* workspace, size_t workspace_bytes, void* hip_stream,
                              const tp_plan_opts_t* opts) {
    Opts o;
    if (int e = resolve_opts(opts, &o)) return e;
    PartialsShare sx, sw;
    if (int e = build_partials(grid, dims, TP_PASS_DX_PARTIALS, &sx)) return e;
    if (int e = build_partials(grid, dims, TP_PASS_DW_PARTIALS, &sw)) return e;
    if (n_dx < 0 || n_dx > sx.n_steps || n_dw < 0 || n_dw > sw.n_steps) return TP_ERR_SHAPE;
    if (sx.m > INT32_MAX || sx.n > INT32_MAX || sx.k > INT32_MAX) return TP_ERR_SHAPE;
    if (n_dx == 0 && n_dw == 0) return TP_OK;
    if (!da_own) return TP_ERR_NULL;
    if (int e = check_cblk(*da_own, sx.k)) return e;                  // [M_blk, F_blk]
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    Range ranges[2 * TP_MAX_STEPS];
    int n_ranges = 0;
    Product px{}; px.active = n_dx > 0;
    if (px.active) {
        if (!w_blocks_dx || !dx_partials) return TP_ERR_NULL;
        Plan p = make_plan(o, sx.m, sx.n, sx.k, 1, n_dx);
        fill_common(o, px.args, p, sx.m, sx.n, sx.k, 1);
        for (int k = 0; k < n_dx; ++k) {
            if (int e = check_cblk(w_blocks_dx[k], sx.k)) return e;    // W block [H_blk][F_blk]: n x k
            if (int e = check_oblk(dx_partials[k], sx.n, true)) return e;
            ranges[n_ranges++] = out_range(dx_partials[k], sx.m, sx.n);
            px.args.a[k] = da_own->ptr; px.args.lda[k] = (int32_t)da_own->ld;
            px.args.b[k] = w_blocks_dx[k].ptr; px.args.ldb[k] = (int32_t)w_blocks_dx[k].ld;
            px.args.outs[k] = dx_partials[k].ptr; px.args.ldos[k] = dx_partials[k].ld;
        }
        px.args.out = dx_partials[0].ptr; px.args.ldo = dx_partials[0].ld; px.args.out_f32 = 1;
        px.args.n_groups = n_dx; px.args.group_along_n = 1; px.args.group_tiles = p.tiles_n;
        px.args.tiles_n = p.tiles_n * n_dx;                            // the products side by side along N
        px.form = FORM_NT; px.plan = p;
    }
    Product pw{}; pw.active = n_dw > 0;
    if (pw.active) {
        if (!x_blocks_dw || !dw_partials) return TP_ERR_NULL;
        Plan p = make_plan(o, sw.m, sw.n, sw.k, 1, n_dw);
        fill_common(o, pw.args, p, sw.m, sw.n, sw.k, 1);
        for (int k = 0; k < n_dw; ++k) {
            if (int e = check_cblk(x_blocks_dw[k], sw.m)) return e;    // X block [M_blk][H_blk]: k x m
            if (int e = check_oblk(dw_partials[k], sw.n, true)) return e;
            ranges[n_ranges++] = out_range(dw_partials[k], sw.m, sw.n);
            pw.args.a[k] = x_blocks_dw[k].ptr; pw.args.lda[k] = (int32_t)x_blocks_dw[k].ld;
            pw.args.b[k] = da_own->ptr; pw.args.ldb[k] = (int32_t)da_own->ld;
            pw.args.outs[k] = dw_partials[k].ptr; pw.args.ldos[k] = dw_partials[k].ld;
        }
        pw.args.out = dw_partials[0].ptr; pw.args.ldo = dw_partials[0].ld; pw.args.out_f32 = 1;
        pw.args.n_groups = n_dw; pw.args.group_along_n = 0; pw.args.group_tiles = p.tiles_m;
        pw.args.tiles_m = p.tiles_m * n_dw;                            // the products stacked along M
        pw.form = FORM_TN; pw.plan = p;
    }
    for (int i = 0; i < n_ranges; ++i)
        for (int j = i + 1; j < n_ranges; ++j)
            if (overlap(ranges[i], ranges[j])) return TP_ERR_SHAPE;
    size_t need = 0;
    if (px.active) need = std::max(need, ws_bytes_for(px.plan, sx.m, sx.n));
    if (pw.active) need = std::max(need, ws_bytes_for(pw.plan, sw.m, sw.n));
    if (!ws_ok(need, workspace, workspace_bytes)) return TP_ERR_WORKSPACE;
    if (int e = check_device()) return e;
    if (px.active) if (int e = run_product(o, px, workspace, stream)) return e;
    if (pw.active) if (int e = run_product(o, pw, workspace, stream)) return e;
    return TP_OK;
}

int tp_linear_bwd_partials(const tp_grid_t* grid, const tp_dims_t* dims, int n_dx, int n_dw, const tp_cblk_t* da_own,
                           const tp_cblk_t* w_blocks_dx, const tp_oblk_t* dx_partials, const tp_cblk_t* x_blocks_dw,
                           const tp_oblk_t* dw_partials, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return tp_linear_bwd_partials_ex(grid, dims, n_dx, n_dw, da_own, w_blocks_dx, dx_partials, x_blocks_dw, dw_partials,
                                     workspace, workspace_bytes, hip_stream, nullptr);
}

int tp_bias_act(const void* c, int64_t ld_c, const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact, int64_t rows,
                int64_t cols, void* hip_stream) {
    if (!c || !y.ptr) return TP_ERR_NULL;
    if (epi != TP_EPI_NONE && epi != TP_EPI_BIAS && epi != TP_EPI_BIAS_GELU) return TP_ERR_MODE;
    if (epi != TP_EPI_NONE && !bias) return TP_ERR_NULL;
    if (rows < 0 || cols < 0) return TP_ERR_SHAPE;
    if (!aligned16(c) || (bias && !aligned16(bias)) || (ld_c & 7)) return TP_ERR_ALIGN;
    if (ld_c < cols) return TP_ERR_SHAPE;
    if (int e = check_oblk(y, cols, false)) return e;
    if (preact.ptr) {
        if (int e = check_oblk(preact, cols, false)) return e;
        if (preact.dtype != TP_BF16) return TP_ERR_DTYPE;
    }
    if (launch_bias_act(static_cast<const float*>(c), ld_c, epi == TP_EPI_NONE ? nullptr : bias, epi == TP_EPI_BIAS_GELU,
                        y.ptr, y.ld, y.dtype == TP_F32, preact.ptr, preact.ld, rows, cols,
                        static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return TP_ERR_HIP;
    return TP_OK;
}

int tp_dgelu(const void* dy, int64_t ld_dy, const void* preact, int64_t ld_pre, void* da, int64_t ld_da,
             int64_t rows, int64_t cols, void* hip_stream) {
    if (!dy || !preact || !da) return TP_ERR_NULL;
    if (rows < 0 || cols < 0) return TP_ERR_SHAPE;
    if (!aligned16(dy) || !aligned16(preact) || !aligned16(da) || (cols & 7) || (ld_dy & 7) || (ld_pre & 7) || (ld_da & 7))
        return TP_ERR_ALIGN;
    if (ld_dy < cols || ld_pre < cols || ld_da < cols) return TP_ERR_SHAPE;
    if (launch_dgelu(dy, ld_dy, preact, ld_pre, da, ld_da, rows, cols, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return TP_ERR_HIP;
    return TP_OK;
}

size_t tp_bias_grad_workspace_size(int64_t rows, int64_t cols) {
    return rows > 0 && cols > 0 ? colsum_ws_bytes(rows, cols) : 0;
}

int tp_bias_grad(const void* da, int64_t ld_da, int64_t rows, int64_t cols, void* db_f32, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
    if (!da || !db_f32) return TP_ERR_NULL;
    if (rows < 0 || cols < 0) return TP_ERR_SHAPE;
    if (!aligned16(da) || !aligned16(db_f32) || (cols & 7) || (ld_da & 7)) return TP_ERR_ALIGN;
    if (ld_da < cols) return TP_ERR_SHAPE;
    if (workspace && (!aligned16(workspace) || workspace_bytes < colsum_ws_bytes(rows, cols))) return TP_ERR_WORKSPACE;
    if (cols == 0) return TP_OK;
    if (launch_colsum(da, ld_da, rows, cols, static_cast<float*>(db_f32), static_cast<float*>(workspace),
                      static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return TP_ERR_HIP;
    return TP_OK;
}

const char* tp_strerror(int status) {
    switch (status) {
        case TP_OK: return "ok";
        case TP_ERR_NULL: return "a required pointer is NULL";
        case TP_ERR_MODE: return "unknown mode, pass, epilogue or option, or an epilogue asked of an additive partial";
        case TP_ERR_GRID: return "grid size or rank coordinate out of range";
        case TP_ERR_SHAPE: return "layer dimensions, leading dimension or step count do not fit the grid, or outputs overlap";
        case TP_ERR_ALIGN: return "pointer not 16-byte aligned, or a column extent / leading dimension not a multiple of 8";
        case TP_ERR_DTYPE: return "output dtype not supported here";
        case TP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case TP_ERR_HIP: return "a HIP call failed, or the device is not a 256-CU MI355X";
        case TP_ERR_SCRATCH: return "the product needs more than the library's built-in scratch: call tp_linear_fwd with a workspace";
        default: return "unknown status";
    }
}

}  // extern "C"
