// C ABI of the library: argument validation, shape -> tile-configuration lookup, launches.
// Host code only; every step of the computation runs in the kernels of gemm_kernel.h and
// aux_kernels.hip.
#include "../../include/fact.h"
#include "launch.h"

#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

namespace fact {

static const ConfigDesc g_configs[] = {
#define FACT_CFG(id, bm, bn, wm, wn, bk, st) {id, bm, bn, wm, wn, bk, st, fact_launch_cfg##id},
#include "configs.def"
#undef FACT_CFG
};
static constexpr int kNumConfigs = (int)(sizeof(g_configs) / sizeof(g_configs[0]));

static constexpr int kNumCU = 256;
static constexpr int kLdsPerCU = 160 * 1024;
static constexpr int kMaxGridZ = 65535;

static thread_local char g_last_error[256] = "";

static int hip_fail(hipError_t e, const char *what)
{
    std::snprintf(g_last_error, sizeof g_last_error, "%s: %s", what, hipGetErrorString(e));
    return FACT_ERR_HIP;
}
int record_hip_failure(hipError_t e, const char *what) { return hip_fail(e, what); }    // for the other translation units

// ---- the per-shape table (filled by the on-device sweep) and the model behind it -----------

struct TableRow {
    int64_t batch, M, N, K;
    int trans_b, gated;
    int cfg, split, group_m;
};
static const TableRow g_table[] = {
#include "tile_table.inc"
    {0, 0, 0, 0, 0, 0, -1, 0, 0}   // sentinel
};

// Rows loaded at run time from a registry file (fact_registry_load): consulted before the
// compiled-in table, newest load first.  Readers and the loader share one mutex: a lookup is a
// short scan on the host and launches are asynchronous, so it is never held across GPU work.
static std::mutex g_registry_mutex;
static std::vector<TableRow> g_registry;

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Tail split hand-over: flags and the status word carry a launch-unique 64-bit value (a process-wide
// counter that starts at a clock-derived value), so a workspace never needs clearing and a stale
// word from another process or another use of the memory is not mistaken for one of ours.
static const unsigned long long g_tail_epoch_first =
    (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() * 0x9E3779B97F4A7C15ull;
static std::atomic<unsigned long long> g_tail_epoch{g_tail_epoch_first};
static std::atomic<int> g_persistent{0};                  // fact_tune_persistent (off unless asked for: measured 0.5-3 % slower than ordinary launches)
static std::atomic<int> g_tail_budget{1 << 20};           // polls (about 0.3 us each) a collecting work-group waits: a third of a second

// Can the MFMA kernel take these operands at all?  (Dimensions only; pointer alignment is
// checked separately at launch.)
static bool fast_dims_ok(int64_t M, int64_t N, int64_t K, int trans_b)
{
    if (K % 8) return false;
    if (!trans_b && N % 8) return false;
    if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX - 64) return false;
    return true;
}

static int wgs_per_cu(const ConfigDesc &c)
{
    int by_lds = kLdsPerCU / c.lds_bytes();
    // accumulators per lane + staging/fragment registers, out of 512 per lane at one wave per SIMD
    int acc = (c.bm / c.wm / 32) * (c.bn / c.wn / 32) * 16;
    int by_regs = 512 / (acc + 128);
    int occ = by_lds < by_regs ? by_lds : by_regs;
    return occ < 1 ? 1 : occ;
}

// Relative K-loop throughput of a compute unit running this tile, 256 x 256 = 1 (larger tiles reuse
// operands more).  Measured on a full chip at long K; the formula serves shapes of tile not listed.
static double tile_rate(const ConfigDesc &c)
{
    const int hi = c.bm > c.bn ? c.bm : c.bn, lo = c.bm > c.bn ? c.bn : c.bm;
    if (hi == 256 && lo == 256) return 1.0;
    if (hi == 256 && lo == 192) return 0.92;
    if (hi == 256 && lo == 128) return 0.85;
    if (hi == 192 && lo == 128) return 0.78;
    if (hi == 128 && lo == 128) return 0.74;
    if (hi == 64 && lo == 64) return 0.40;
    const double per_k = (double)(c.bm + c.bn) / ((double)c.bm * c.bn);   // operand bytes per MAC
    return (1.0 + 48.0 * 512.0 / 65536.0) / (1.0 + 48.0 * per_k);
}

// Work-groups of a persistent launch of `items` tiles (times batch entries) with K whole, or 0 when the
// launch is an ordinary one: every item fits at once, an 8-wave configuration (see the kernel), or
// switched off.  A multiple of 8, so a work-group stays on its XCD's part of the tile order.
static int persistent_grid(const ConfigDesc &c, int64_t items)
{
    if (c.wm * c.wn > 4 || !g_persistent.load(std::memory_order_relaxed)) return 0;
    const int64_t slots = (int64_t)kNumCU * wgs_per_cu(c);
    return items > slots && items <= INT32_MAX / 2 ? (int)slots : 0;
}

struct Plan {
    int cfg = -1;      // -1: fallback kernel
    int split = 1;
    int group_m = 4;
};

// Estimated microseconds of a launch, for shapes the registry does not list.  A 64-deep K step of a
// 256 x 256 tile takes 1.4 us on a busy chip; a tile costs 1.5 us + 1.5 us per 256 x 256 of area
// besides its K loop (first loads, epilogue); a partly filled last round runs its tiles up to a
// fifth faster (the chip is power-limited: fewer busy compute units, higher clock).  Checked against
// exhaustive timing of every configuration on 24 unlisted shapes: the choice costs 0.6 % on average
// and at most 8 % (the model it replaces, which counted the fixed cost in K steps and priced small
// tiles by a formula: 5.4 % and 30 %).
static double model_time(const ConfigDesc &c, int64_t batch, int64_t M, int64_t nout, int64_t K, bool gated, int split)
{
    const int64_t bn_out = gated ? c.bn / 2 : c.bn;
    const int64_t tiles = ((M + c.bm - 1) / c.bm) * ((nout + bn_out - 1) / bn_out) * batch * split;
    const int occ = wgs_per_cu(c);
    const int64_t slots = (int64_t)kNumCU * occ;
    const int64_t rounds = (tiles + slots - 1) / slots;
    const double area = (double)c.bm * c.bn / 65536.0;
    const double step_us = 1.40 * area / tile_rate(c);
    const int64_t ksteps = ((K + split - 1) / split + 63) / 64;
    const double tile_us = (double)occ * (double)ksteps * step_us + 1.5 + 1.5 * area;
    const double last = (double)(tiles - (rounds - 1) * slots) / (double)slots;     // how full the last round is
    return (double)(rounds - 1) * tile_us + tile_us * (1.0 - 0.2 * (1.0 - last));
}

static Plan make_plan(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b, int act, bool allow_split)
{
    Plan pl;
    const bool gated = act == FACT_ACT_SILU_GATE;
    if (!fast_dims_ok(M, N, K, trans_b)) return pl;
    auto matches = [&](const TableRow &r) {
        return r.batch == batch && r.M == M && r.N == N && r.K == K && r.trans_b == trans_b &&
               r.gated == (int)gated && (allow_split || (r.split >= 0 && r.split <= 1));
    };
    auto take = [&](const TableRow &r) {
        pl.cfg = r.cfg;
        pl.split = r.split == 0 ? 1 : r.split;             // negative: a tail split, which needs a workspace as well
        pl.group_m = r.group_m > 0 ? r.group_m : 4;
    };
    {
        std::lock_guard<std::mutex> lock(g_registry_mutex);
        for (const TableRow &r : g_registry)
            if (matches(r)) { take(r); return pl; }
    }
    for (const TableRow *r = g_table; r->cfg >= 0; ++r)
        if (matches(*r)) { take(*r); return pl; }
    const int64_t nout = gated ? N / 2 : N;
    double best = 0;
    for (int i = 0; i < kNumConfigs; ++i) {
        const ConfigDesc &c = g_configs[i];
        if (gated && !c.gate_capable()) continue;
        if (!c.serves(trans_b)) continue;
        int max_split = 1;
        if (allow_split && batch == 1) {
            max_split = (int)(K / 1024);
            if (max_split > 256) max_split = 256;
            if (max_split < 1) max_split = 1;
        }
        for (int s = 1; s <= max_split; s *= 2) {
            double t = model_time(c, batch, M, nout, K, gated, s);
            if (s > 1) t += 4.0 + 2.0 * s * (double)M * N * 4.0 / 4.0e6;     // the reduction launch; partials written and read back at ~4 TB/s
            if (pl.cfg < 0 || t < best) { best = t; pl.cfg = i; pl.split = s; }
        }
    }
    pl.group_m = 4;
    return pl;
}

// ---- validation -----------------------------------------------------------------------------

struct Problem {
    int64_t batch, M, N, K;
    const void *A; int64_t lda, stride_a;
    const void *B; int64_t ldb, stride_b; int trans_b;
    const void *B_up;     // gated with separate weights, else nullptr
    void *C; int64_t ldc, stride_c;
    fact_epilogue ep;
};

static int validate(const Problem &q)
{
    if (!q.A || !q.B || !q.C) return FACT_ERR_NULL;
    if (q.batch <= 0 || q.M <= 0 || q.N <= 0 || q.K <= 0) return FACT_ERR_DIM;
    if (q.batch > kMaxGridZ) return FACT_ERR_DIM;
    if (q.trans_b != 0 && q.trans_b != 1) return FACT_ERR_LAYOUT;
    const int act = q.ep.act;
    if (act != FACT_ACT_NONE && act != FACT_ACT_GELU_TANH && act != FACT_ACT_SILU_GATE) return FACT_ERR_EPILOGUE;
    const bool gated = act == FACT_ACT_SILU_GATE;
    if (gated) {
        if (q.ep.bias) return FACT_ERR_EPILOGUE;
        if (q.N % 2) return FACT_ERR_EPILOGUE;
        if (!q.trans_b) return FACT_ERR_LAYOUT;
    }
    const int64_t nout = gated ? q.N / 2 : q.N;
    if (q.lda < q.K) return FACT_ERR_DIM;
    if (q.ldb < (q.trans_b ? q.K : q.N)) return FACT_ERR_DIM;
    if (q.ldc < nout) return FACT_ERR_DIM;
    if (q.ep.residual && q.ep.ldr < nout) return FACT_ERR_DIM;
    if (q.stride_a < 0 || q.stride_b < 0 || q.stride_c < 0 || q.ep.stride_r < 0) return FACT_ERR_DIM;
    if (q.batch > 1 && q.stride_c < (q.M - 1) * q.ldc + nout) return FACT_ERR_DIM;
    if (q.M > INT32_MAX || q.N > INT32_MAX || q.K > INT32_MAX) return FACT_ERR_DIM;
    const uintptr_t two = (uintptr_t)q.A | (uintptr_t)q.B | (uintptr_t)q.C | (uintptr_t)q.ep.bias |
                          (uintptr_t)q.ep.residual | (uintptr_t)q.B_up;
    if (two & 1u) return FACT_ERR_ALIGN;
    if (q.ep.out_f32 != 0 && q.ep.out_f32 != 1) return FACT_ERR_EPILOGUE;
    if (q.ep.f16 != 0 && q.ep.f16 != 1) return FACT_ERR_EPILOGUE;
    if (q.ep.out_f32 && ((uintptr_t)q.C & 3u)) return FACT_ERR_ALIGN;
    return FACT_OK;
}

static size_t splitk_ws_bytes(int64_t M, int64_t N, int split)
{
    return split > 1 ? (size_t)split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

// Tail split: the tiles of the last, partly filled round are shared by g work-groups each.
struct TailPlan {
    int64_t first = 0;      // tiles computed whole
    int64_t rem = 0;        // tiles in the tail
    int g = 0;              // K ranges per tail tile (0: no tail split)
    // workspace: a status block (its first word: see fact_tail_timeouts), the fp32 partial tiles, one flag per partial
    static constexpr size_t kStatusBytes = 256;
    size_t bytes() const { return g > 1 ? kStatusBytes + (size_t)rem * (g - 1) * sizeof(float) * tile_floats + (size_t)rem * (g - 1) * 8 : 0; }
    size_t partials_offset() const { return kStatusBytes; }
    size_t flags_offset() const { return kStatusBytes + (size_t)rem * (g - 1) * sizeof(float) * tile_floats; }
    size_t tile_floats = 0;
};

static TailPlan tail_plan(const ConfigDesc &c, int64_t tiles, int64_t K, int g)
{
    TailPlan t;
    t.tile_floats = (size_t)c.bm * c.bn;
    const int64_t slots = (int64_t)kNumCU * wgs_per_cu(c);
    const int64_t ksteps = (K + 63) / 64;
    if (g < 2 || ksteps / g < 4) return t;            // too little K per range to be worth a hand-over
    if (!c.has_prefetch()) return t;                  // (no sink behind the ring: the collector has nowhere to pass its verdict)
    t.first = tiles / slots * slots;
    t.rem = tiles - t.first;
    if (t.rem == 0) { t.first = 0; return t; }
    t.g = g;
    return t;
}

// ---- the one launch path every entry point goes through ----------------------------------------

static int run(const Problem &q, int cfg_id, int split, int group_m, bool allow_table_split,
               void *ws, size_t ws_bytes, hipStream_t stream)
{
    int rc = validate(q);
    if (rc != FACT_OK) return rc;
    const bool gated = q.ep.act == FACT_ACT_SILU_GATE;
    const int64_t nout = gated ? q.N / 2 : q.N;

    Plan pl = make_plan(q.batch, q.M, q.N, q.K, q.trans_b, q.ep.act, allow_table_split);
    if (cfg_id == FACT_CONFIG_GUARDED) {              // the guarded kernel on request: the sweep's reference result
        if (split > 1 || split < 0 || q.ep.out_f32) return FACT_ERR_UNSUPPORTED;
        pl.cfg = -1; pl.split = 1;
    }
    if (cfg_id >= 0) {
        if (cfg_id >= kNumConfigs) return FACT_ERR_UNSUPPORTED;
        if (!fast_dims_ok(q.M, q.N, q.K, q.trans_b)) return FACT_ERR_UNSUPPORTED;
        if (gated && !g_configs[cfg_id].gate_capable()) return FACT_ERR_UNSUPPORTED;
        if (!g_configs[cfg_id].serves(q.trans_b)) return FACT_ERR_UNSUPPORTED;
        pl.cfg = cfg_id;
        if (split <= 0) pl.split = 1;
    }
    if (split > 0) pl.split = split;
    if (split < 0) pl.split = split;                  // forced tail split, -split ranges per tail tile
    if (group_m > 0) pl.group_m = group_m;
    int tail_g = 0;                                   // a negative split in a plan is a tail split
    if (pl.split < 0) { tail_g = -pl.split; pl.split = 1; }
    if (tail_g > 1 && q.batch != 1) { if (split < 0) return FACT_ERR_UNSUPPORTED; tail_g = 0; }
    if (pl.split > 1 && q.batch != 1) return FACT_ERR_UNSUPPORTED;
    if (pl.split > kMaxGridZ) return FACT_ERR_UNSUPPORTED;

    // operands the MFMA kernel reads with 16-byte loads
    // (leading dimensions are bounded so that per-lane byte offsets inside one tile panel fit 31 bits)
    const bool ptr_ok = aligned16(q.A) && aligned16(q.B) && (!q.B_up || aligned16(q.B_up)) &&
                        q.lda % 8 == 0 && q.ldb % 8 == 0 && q.stride_a % 8 == 0 && q.stride_b % 8 == 0 &&
                        q.lda <= (1 << 21) && q.ldb <= (1 << 21);
    if (pl.cfg >= 0 && !ptr_ok) {
        if (cfg_id >= 0) return FACT_ERR_UNSUPPORTED;
        pl.cfg = -1;
    }
    if (pl.cfg < 0) pl.split = 1;     // the fallback never splits
    // fp32 output: with K whole the main kernel's epilogue writes it, unrounded; with K split the
    // reduction pass does (no batch then, as for any split).  No tail split, no fallback kernel.
    bool out_f32 = q.ep.out_f32 != 0, c_f32 = false;
    if (out_f32) {
        if (pl.cfg < 0) return FACT_ERR_UNSUPPORTED;
        tail_g = 0;
        if (pl.split < 1) pl.split = 1;
        if (pl.split == 1) { c_f32 = true; out_f32 = false; }
        else if (q.batch != 1 || !allow_table_split) return FACT_ERR_UNSUPPORTED;
    }

    GemmArgs a;
    std::memset(&a, 0, sizeof a);
    a.A = (const __bf16 *)q.A;
    a.B = (const __bf16 *)q.B;
    a.B_up = gated ? (q.B_up ? (const __bf16 *)q.B_up : (const __bf16 *)q.B + nout * q.ldb) : nullptr;
    a.C = (__bf16 *)q.C;
    a.bias = (const __bf16 *)q.ep.bias;
    a.res = (const __bf16 *)q.ep.residual;
    a.lda = q.lda; a.ldb = q.ldb; a.ldc = q.ldc; a.ldr = q.ep.ldr;
    a.stride_a = q.stride_a; a.stride_b = q.stride_b; a.stride_c = q.stride_c; a.stride_r = q.ep.stride_r;
    a.M = (int)q.M; a.N = (int)q.N; a.K = (int)q.K;
    a.act = q.ep.act;
    a.splits = 1;
    a.group_m = pl.group_m;
    // 16-byte vector access to C / residual / bias in the epilogue
    a.out_f32 = out_f32 ? 1 : 0;
    a.c_f32 = c_f32 ? 1 : 0;
    a.f16 = q.ep.f16;
    // (an fp32 row of 8 columns is two 16-byte pieces: ldc and the batch stride in multiples of 4)
    a.vec_store = (nout % 8 == 0) && q.ldc % (c_f32 ? 4 : 8) == 0 && aligned16(q.C) && q.stride_c % (c_f32 ? 4 : 8) == 0 &&
                  (!q.ep.bias || aligned16(q.ep.bias)) &&
                  (!q.ep.residual || (aligned16(q.ep.residual) && q.ep.ldr % 8 == 0 && q.ep.stride_r % 8 == 0)) &&
                  q.ldc < ((int64_t)1 << 21) && q.ep.ldr < ((int64_t)1 << 21);     // a tile's rows within 2^31 bytes: 32-bit row offsets in the epilogue

    hipError_t e;
    if (pl.cfg < 0) {
        e = launch_fallback_gemm(a, q.trans_b != 0, (int)q.batch, stream);
        return e == hipSuccess ? FACT_OK : hip_fail(e, "fallback gemm launch");
    }

    const ConfigDesc &c = g_configs[pl.cfg];
    const int bn_out = gated ? c.bn / 2 : c.bn;
    const int64_t tiles_m = (q.M + c.bm - 1) / c.bm, tiles_n = (nout + bn_out - 1) / bn_out;
    if (tiles_m * tiles_n > INT32_MAX / 2) return FACT_ERR_DIM;
    a.tiles_m = (int)tiles_m; a.tiles_n = (int)tiles_n;

    a.pf_dist = 1;
    a.tail_first = (int)(tiles_m * tiles_n);
    if (tail_g > 1 && pl.split <= 1) {
        const TailPlan t = tail_plan(c, tiles_m * tiles_n, q.K, tail_g);
        if (t.g > 1 && ws && aligned16(ws) && ws_bytes >= t.bytes()) {
            // flags carry a launch-unique 64-bit value, so the workspace needs no clearing
            a.tail_first = (int)t.first;
            a.tail_g = t.g;
            a.tail_ws = (float *)((char *)ws + t.partials_offset());
            a.tail_flags = (unsigned long long *)((char *)ws + t.flags_offset());
            a.tail_status = (unsigned long long *)ws;
            a.tail_epoch = ++g_tail_epoch;
            a.tail_budget = g_tail_budget.load(std::memory_order_relaxed);
        } else if (split < 0) {
            return t.g > 1 ? FACT_ERR_WORKSPACE : FACT_ERR_UNSUPPORTED;
        }
    }
    if (pl.split > 1) {
        // K ranges are multiples of the 64-element staging step
        int64_t kps = (q.K + pl.split - 1) / pl.split;
        kps = (kps + 63) / 64 * 64;
        const int splits = (int)((q.K + kps - 1) / kps);
        if (splits <= 1) {
            pl.split = 1;
        } else {
            const size_t need = splitk_ws_bytes(q.M, q.N, pl.split);
            if (!ws) return FACT_ERR_WORKSPACE;
            if (!aligned16(ws)) return FACT_ERR_ALIGN;
            if (ws_bytes < need) return FACT_ERR_WORKSPACE;
            a.splits = splits;
            a.k_per_split = (int)kps;
            a.P = (float *)ws;
        }
    }
    // L2 prefetch (see the kernel).  Many work-groups: the ones resident on an XCD (32 CUs) form a
    // block of gsz tile rows x (resident / gsz) tile columns that share panels; each touches its
    // share one step ahead.  (With few work-groups, e.g. long split-K ranges streamed from HBM,
    // unshared prefetching several steps ahead was measured to be slower than none.)
    {
        const int64_t grid = tiles_m * tiles_n * (a.splits > 1 ? a.splits : q.batch);
        const bool soff_ok = q.trans_b || (q.K * q.ldb * 2 < ((int64_t)1 << 31));
        auto pow2_floor = [](int v) { int r = 1; while (r * 2 <= v) r *= 2; return r; };
        // Also with about one work-group per compute unit when K is long and not split: the panels then
        // come from HBM at least once per launch, and inside a transformer block (weights of several
        // layers between two uses) every time.  Measured with operands rotated out of the memory-side
        // cache: Llama QKV 1052 -> 1260 TFLOP/s, down projection 1130 -> 1235, 4096^3 1243 -> 1330;
        // no gain or a small loss for K = 768, for half-empty grids and for split-K ranges.
        const int64_t wgs = a.tail_g > 1 ? a.tail_first + (tiles_m * tiles_n - a.tail_first) * a.tail_g : grid;
        const bool one_round_long_k = pl.split <= 1 && wgs >= 3 * kNumCU / 4 && q.K >= 2048;
        if (soff_ok && c.has_prefetch()) {
            // (a round and a half of whole-K tiles counts as many: 8192 x 2304 x 768 on 384 tiles of 256 x 192,
            // operands from HBM, 48.0 -> 42.9 us with the prefetch, 37.4 -> 36.9 us from the memory-side cache)
            if (grid >= 2 * kNumCU || (a.splits <= 1 && grid >= 3 * kNumCU / 2) || one_round_long_k) {
                const int gsz = (int)(pl.group_m < tiles_m ? pl.group_m : tiles_m);
                const int resident = 32 * wgs_per_cu(c);
                int sb = pow2_floor(gsz), sa = pow2_floor(resident / gsz > 0 ? resident / gsz : 1);
                if (sa > tiles_n) sa = pow2_floor((int)tiles_n);
                a.pf_sa = sa > 32 ? 32 : sa; a.pf_sb = sb > 32 ? 32 : sb; a.pf_dist = 1;
            }
        }
    }
    if (out_f32 && a.splits <= 1) {                   // one fp32 plane
        const size_t need = (size_t)q.M * (size_t)q.N * sizeof(float);
        if (!ws) return FACT_ERR_WORKSPACE;
        if (!aligned16(ws)) return FACT_ERR_ALIGN;
        if (ws_bytes < need) return FACT_ERR_WORKSPACE;
        a.P = (float *)ws;
    }
    // Persistent launch: more work items than resident work-groups, K whole, no tail split.
    a.persist_items = 0; a.persist_z = 1; a.persist_grid = 0;
    if (a.tail_g <= 1 && a.splits <= 1 && !a.f16) {       // (the persistent form is instantiated for bf16 only)
        const int grid = persistent_grid(c, tiles_m * tiles_n * q.batch);
        if (grid > 0) { a.persist_items = (int)(tiles_m * tiles_n * q.batch); a.persist_z = (int)q.batch; a.persist_grid = grid; }
    }
    // (the kernel numbers (K range or batch entry, tile) pairs with 32-bit integers)
    if (tiles_m * tiles_n * (a.splits > 1 ? (int64_t)a.splits : q.batch) > INT32_MAX / 2) return FACT_ERR_DIM;
    e = c.launch(a, q.trans_b != 0, a.splits > 1 ? a.splits : (int)q.batch, stream);
    if (e != hipSuccess) return hip_fail(e, "gemm launch");
    if (a.splits > 1 || out_f32) {
        e = launch_splitk_reduce(a, stream);
        if (e != hipSuccess) return hip_fail(e, "split-K reduce launch");
    }
    return FACT_OK;
}

static fact_epilogue ep_or_none(const fact_epilogue *ep)
{
    fact_epilogue e;
    std::memset(&e, 0, sizeof e);
    if (ep) e = *ep;
    return e;
}

}  // namespace fact

using namespace fact;

extern "C" {

int fact_gemm(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
              int trans_b, void *C, int64_t ldc, const fact_epilogue *ep, void *stream)
{
    Problem q{1, M, N, K, A, lda, 0, B, ldb, 0, trans_b, nullptr, C, ldc, 0, ep_or_none(ep)};
    return run(q, -1, 1, 0, false, nullptr, 0, (hipStream_t)stream);
}

int fact_gemm_batched(int64_t batch, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, int64_t stride_a,
                      const void *B, int64_t ldb, int64_t stride_b, int trans_b,
                      void *C, int64_t ldc, int64_t stride_c,
                      const fact_epilogue *ep, void *stream)
{
    Problem q{batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, trans_b, nullptr, C, ldc, stride_c, ep_or_none(ep)};
    return run(q, -1, 1, 0, false, nullptr, 0, (hipStream_t)stream);
}

int fact_gemm_splitk(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                     int trans_b, void *C, int64_t ldc, const fact_epilogue *ep,
                     int split_k, void *ws, size_t ws_bytes, void *stream)
{
    if (split_k < 0) return FACT_ERR_UNSUPPORTED;
    Problem q{1, M, N, K, A, lda, 0, B, ldb, 0, trans_b, nullptr, C, ldc, 0, ep_or_none(ep)};
    return run(q, -1, split_k, 0, true, ws, ws_bytes, (hipStream_t)stream);
}

// workspace a plan needs: split-K partial planes, or the partial tiles and flags of a tail split
static size_t plan_ws_bytes(const Plan &pl, int64_t M, int64_t N, int64_t K, bool gated)
{
    if (pl.cfg < 0) return 0;
    if (pl.split > 1) return splitk_ws_bytes(M, N, pl.split);
    if (pl.split < -1) {
        const ConfigDesc &c = g_configs[pl.cfg];
        const int64_t nout = gated ? N / 2 : N, bn_out = gated ? c.bn / 2 : c.bn;
        const int64_t tiles = ((M + c.bm - 1) / c.bm) * ((nout + bn_out - 1) / bn_out);
        return tail_plan(c, tiles, K, -pl.split).bytes();
    }
    return 0;
}

size_t fact_gemm_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int split_k)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    if (split_k < 0) {
        // forced tail split (fact_gemm_ex): the largest need over the tile configurations
        size_t need = 0;
        for (int i = 0; i < kNumConfigs; ++i)
            for (int gated = 0; gated < 2; ++gated) {
                Plan pl; pl.cfg = i; pl.split = split_k;
                const size_t b = plan_ws_bytes(pl, M, N, K, gated != 0);
                if (b > need) need = b;
            }
        return need;
    }
    int s = split_k;
    size_t tail_need = 0;
    if (s == 0) {
        // the table's choice may depend on layout and epilogue; report the largest over them
        for (int tb = 0; tb < 2; ++tb)
            for (int act = 0; act < 3; ++act) {
                if (act == FACT_ACT_SILU_GATE && (!tb || N % 2)) continue;
                Plan pl = make_plan(1, M, N, K, tb, act, true);
                if (pl.cfg >= 0 && pl.split > s) s = pl.split;
                const size_t b = pl.split < -1 ? plan_ws_bytes(pl, M, N, K, act == FACT_ACT_SILU_GATE) : 0;
                if (b > tail_need) tail_need = b;
            }
    }
    const size_t sk = splitk_ws_bytes(M, N, s);
    return sk > tail_need ? sk : tail_need;
}

size_t fact_gemm_f32out_workspace_bytes(int64_t M, int64_t N, int64_t K, int split_k)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    int s = split_k < 0 ? 0 : split_k;
    if (s == 0)                                       // the table's split-K factor, over both layouts (tail splits do not apply)
        for (int tb = 0; tb < 2; ++tb) {
            const Plan pl = make_plan(1, M, N, K, tb, FACT_ACT_NONE, true);
            if (pl.cfg >= 0 && pl.split > s) s = pl.split;
        }
    return splitk_ws_bytes(M, N, s);                  // nothing when K stays whole: the main kernel writes the fp32 result
}

int fact_gemm_ex(int64_t batch, int64_t M, int64_t N, int64_t K,
                 const void *A, int64_t lda, int64_t stride_a,
                 const void *B, int64_t ldb, int64_t stride_b, int trans_b,
                 void *C, int64_t ldc, int64_t stride_c,
                 const fact_epilogue *ep, int config_id, int split_k, int group_m,
                 void *ws, size_t ws_bytes, void *stream)
{
    Problem q{batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, trans_b, nullptr, C, ldc, stride_c, ep_or_none(ep)};
    return run(q, config_id, split_k, group_m, true, ws, ws_bytes, (hipStream_t)stream);
}

size_t fact_block_mlp_workspace_bytes(int64_t T, int64_t d_model, int64_t d_ff, int act)
{
    if (T <= 0 || d_model <= 0 || d_ff <= 0) return 0;
    if (act < 0 || act > 2) return 0;
    const bool gated = act == FACT_ACT_SILU_GATE;
    const Plan p1 = make_plan(1, T, gated ? 2 * d_ff : d_ff, d_model, 1, act, true);
    const Plan p2 = make_plan(1, T, d_model, d_ff, 1, FACT_ACT_NONE, true);
    const size_t b1 = p1.split < -1 ? plan_ws_bytes(p1, T, gated ? 2 * d_ff : d_ff, d_model, gated) : 0;   // GEMM 1 never splits K
    const size_t b2 = plan_ws_bytes(p2, T, d_model, d_ff, false);
    return b1 > b2 ? b1 : b2;
}

static int block_mlp_impl(int f16, int64_t T, int64_t d_model, int64_t d_ff,
                          const void *X, const void *W1, const void *W1u, const void *b1, int act,
                          const void *W2, const void *b2, const void *R,
                          void *H, void *Y, void *ws, size_t ws_bytes, void *stream)
{
    if (!X || !W1 || !W2 || !H || !Y) return FACT_ERR_NULL;
    if (act != FACT_ACT_NONE && act != FACT_ACT_GELU_TANH && act != FACT_ACT_SILU_GATE) return FACT_ERR_EPILOGUE;
    const bool gated = act == FACT_ACT_SILU_GATE;
    if (gated && !W1u) return FACT_ERR_NULL;
    if (!gated && W1u) return FACT_ERR_EPILOGUE;
    if (gated && b1) return FACT_ERR_EPILOGUE;
    if (T <= 0 || d_model <= 0 || d_ff <= 0) return FACT_ERR_DIM;

    // GEMM 1: H = act(X W1^T + b1); gated: contraction over 2*d_ff columns, gate then up
    fact_epilogue e1;
    std::memset(&e1, 0, sizeof e1);
    e1.bias = b1;
    e1.act = act;
    e1.f16 = f16;
    Problem q1{1, T, gated ? 2 * d_ff : d_ff, d_model, X, d_model, 0, W1, d_model, 0, 1,
               gated ? W1u : nullptr, H, d_ff, 0, e1};
    // GEMM 2: Y = H W2^T + b2 + R  (may split K = d_ff when the table says so and ws allows)
    fact_epilogue e2;
    std::memset(&e2, 0, sizeof e2);
    e2.bias = b2;
    e2.residual = R;
    e2.ldr = d_model;
    e2.act = FACT_ACT_NONE;
    e2.f16 = f16;
    Problem q2{1, T, d_model, d_ff, H, d_ff, 0, W2, d_ff, 0, 1, nullptr, Y, d_model, 0, e2};
    // everything either launch could refuse is checked before the first one: on error nothing runs
    int rc = validate(q1);
    if (rc == FACT_OK) rc = validate(q2);
    if (rc != FACT_OK) return rc;
    const size_t need = fact_block_mlp_workspace_bytes(T, d_model, d_ff, act);
    if (need > 0 && (!ws || ws_bytes < need)) return FACT_ERR_WORKSPACE;
    if (need > 0 && !aligned16(ws)) return FACT_ERR_ALIGN;
    // (the first GEMM never splits K into planes, but its last round of tiles may be split)
    const Plan p1 = make_plan(1, T, gated ? 2 * d_ff : d_ff, d_model, 1, act, true);
    rc = run(q1, -1, p1.split < -1 ? 0 : 1, 0, p1.split < -1, ws, ws_bytes, (hipStream_t)stream);
    if (rc != FACT_OK) return rc;
    return run(q2, -1, 0, 0, need > 0, ws, ws_bytes, (hipStream_t)stream);
}

int fact_block_mlp(int64_t T, int64_t d_model, int64_t d_ff,
                   const void *X, const void *W1, const void *W1u, const void *b1, int act,
                   const void *W2, const void *b2, const void *R,
                   void *H, void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return block_mlp_impl(0, T, d_model, d_ff, X, W1, W1u, b1, act, W2, b2, R, H, Y, ws, ws_bytes, stream);
}

int fact_block_mlp_f16(int64_t T, int64_t d_model, int64_t d_ff,
                       const void *X, const void *W1, const void *W1u, const void *b1, int act,
                       const void *W2, const void *b2, const void *R,
                       void *H, void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return block_mlp_impl(1, T, d_model, d_ff, X, W1, W1u, b1, act, W2, b2, R, H, Y, ws, ws_bytes, stream);
}

int fact_num_configs(void) { return kNumConfigs; }

int fact_config_info(int id, int *tile_m, int *tile_n, int *waves_m, int *waves_n, int *lds_bytes)
{
    if (id < 0 || id >= kNumConfigs) return FACT_ERR_UNSUPPORTED;
    const ConfigDesc &c = g_configs[id];
    if (tile_m) *tile_m = c.bm;
    if (tile_n) *tile_n = c.bn;
    if (waves_m) *waves_m = c.wm;
    if (waves_n) *waves_n = c.wn;
    if (lds_bytes) *lds_bytes = c.lds_bytes();
    return FACT_OK;
}

int fact_select_config(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b, int act,
                       int *config_id, int *split_k)
{
    if (batch <= 0 || M <= 0 || N <= 0 || K <= 0) return FACT_ERR_DIM;
    if (trans_b != 0 && trans_b != 1) return FACT_ERR_LAYOUT;
    if (act < 0 || act > 2) return FACT_ERR_EPILOGUE;
    if (act == FACT_ACT_SILU_GATE && (N % 2 || !trans_b)) return FACT_ERR_EPILOGUE;
    Plan pl = make_plan(batch, M, N, K, trans_b, act, true);
    if (config_id) *config_id = pl.cfg;
    if (split_k) *split_k = pl.split;
    return FACT_OK;
}

int fact_persistent_grid(int64_t batch, int64_t M, int64_t N, int64_t K, int trans_b, int act, int config_id)
{
    if (batch <= 0 || M <= 0 || N <= 0 || K <= 0) return 0;
    if (config_id < 0) {
        Plan pl = make_plan(batch, M, N, K, trans_b, act, false);
        if (pl.split != 1) return 0;
        config_id = pl.cfg;
    }
    if (config_id < 0 || config_id >= kNumConfigs) return 0;
    const ConfigDesc &c = g_configs[config_id];
    const int64_t nout = act == FACT_ACT_SILU_GATE ? N / 2 : N;
    const int bn_out = act == FACT_ACT_SILU_GATE ? c.bn / 2 : c.bn;
    return persistent_grid(c, ((M + c.bm - 1) / c.bm) * ((nout + bn_out - 1) / bn_out) * batch);
}

const char *fact_status_string(int status)
{
    switch (status) {
    case FACT_OK: return "ok";
    case FACT_ERR_NULL: return "required pointer is NULL";
    case FACT_ERR_DIM: return "bad dimension, leading dimension or stride";
    case FACT_ERR_ALIGN: return "pointer alignment";
    case FACT_ERR_LAYOUT: return "bad layout flag";
    case FACT_ERR_EPILOGUE: return "bad epilogue";
    case FACT_ERR_WORKSPACE: return "workspace missing or too small";
    case FACT_ERR_UNSUPPORTED: return "unsupported configuration";
    case FACT_ERR_HIP: return "HIP error";
    default: return "unknown status";
    }
}

// ---- split-K without a caller's workspace: partials in a library-owned static device array --------
// For callers that cannot allocate (code under graph capture, serving loops, harnesses that forbid
// it).  The array lives in this library's device image: every GPU the library runs on holds its own
// copy, at its own address, until the process ends.  Host code never uses the array's name as an
// address (on the host it is a stand-in for the symbol): the address is asked for once per device,
// with that device current, and kept.
static constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

static int static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "static scratch: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return FACT_ERR_UNSUPPORTED;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));       // this device's copy (the current device)
        if (e != hipSuccess || !ptr) return hip_fail(e, "static scratch: hipGetSymbolAddress");
        g_scratch_ptr[dev].store(ptr, std::memory_order_release); // (two threads may both ask: they get the same address)
    }
    *out = ptr;
    return FACT_OK;
}

size_t fact_gemm_splitk_static_capacity(void) { return kStaticScratchBytes; }

int fact_gemm_splitk_static_init(void)
{
    void *ptr = nullptr;
    return static_scratch(&ptr);
}

int fact_gemm_splitk_static(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                            int trans_b, void *C, int64_t ldc, const fact_epilogue *ep, int split_k, void *stream)
{
    if (split_k < 0) return FACT_ERR_UNSUPPORTED;
    if (M <= 0 || N <= 0 || K <= 0) return FACT_ERR_DIM;
    // what fact_gemm_splitk would ask the caller for, for this very call (layout and epilogue known here)
    const fact_epilogue e0 = ep_or_none(ep);
    Plan pl = make_plan(1, M, N, K, trans_b, e0.act, true);
    if (split_k > 0) pl.split = split_k;
    const bool gated = e0.act == FACT_ACT_SILU_GATE;
    size_t need = pl.split > 1 && e0.out_f32 ? splitk_ws_bytes(M, N, pl.split) : plan_ws_bytes(pl, M, N, K, gated);
    if (need > kStaticScratchBytes) {
        std::snprintf(g_last_error, sizeof g_last_error,
                      "fact_gemm_splitk_static: this call needs %zu bytes of partial sums, the static array holds %zu "
                      "(use fact_gemm_splitk with a workspace, or a smaller split_k)", need, kStaticScratchBytes);
        return FACT_ERR_WORKSPACE;
    }
    void *ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != FACT_OK) return rc;
    Problem q{1, M, N, K, A, lda, 0, B, ldb, 0, trans_b, nullptr, C, ldc, 0, e0};
    return run(q, -1, split_k, 0, true, ptr, kStaticScratchBytes, (hipStream_t)stream);
}

int fact_tail_timeouts(const void *ws, void *stream, int *gave_up)
{
    if (!ws || !gave_up) return FACT_ERR_NULL;
    if ((uintptr_t)ws & 15u) return FACT_ERR_ALIGN;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "fact_tail_timeouts: stream synchronize");
    unsigned long long word = 0;
    e = hipMemcpy(&word, ws, sizeof word, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "fact_tail_timeouts: read of the status word");
    const unsigned long long last = g_tail_epoch.load();
    // epochs handed out by this process: (first, last], compared modulo 2^64
    *gave_up = (word - g_tail_epoch_first - 1) < (last - g_tail_epoch_first) ? 1 : 0;
    return FACT_OK;
}

void fact_test_tail_poll_budget(int polls) { g_tail_budget.store(polls, std::memory_order_relaxed); }
int fact_tune_persistent(int mode) { return fact::g_persistent.exchange(mode != 0 ? 1 : 0, std::memory_order_relaxed); }

// Registry file: text, one entry per line (see include/fact.h).  Entries of another rule, data type
// or architecture are skipped, as are entries naming a configuration this build does not have or
// one that does not serve the entry's layout.
int fact_registry_load(const char *path)
{
    if (!path) return FACT_ERR_NULL;
    std::FILE *f = std::fopen(path, "r");
    if (!f) return FACT_ERR_UNSUPPORTED;
    char line[1024];
    bool header = false;
    std::vector<TableRow> rows;
    while (std::fgets(line, sizeof line, f)) {
        if (line[0] == '#') {
            int ver = 0;
            if (std::sscanf(line, "# fact-registry %d", &ver) == 1) {
                if (ver != 1) { std::fclose(f); return FACT_ERR_UNSUPPORTED; }
                header = true;
            }
            continue;
        }
        if (!header) { std::fclose(f); return FACT_ERR_UNSUPPORTED; }      // entries before the format line
        char rule[32], dtype[32], arch[32], layout[8], epi[16];
        long long batch, M, N, K;
        int cfg, split, group_m;
        if (std::sscanf(line, "%31s %31s %31s %lld %lld %lld %lld %7s %15s %d %d %d", rule, dtype, arch, &batch, &M, &N, &K,
                        layout, epi, &cfg, &split, &group_m) != 12)
            continue;
        if (std::strcmp(rule, "gemm") || std::strcmp(dtype, "bf16") || std::strcmp(arch, "gfx950")) continue;
        const int trans_b = !std::strcmp(layout, "nk") ? 1 : !std::strcmp(layout, "kn") ? 0 : -1;
        const int gated = !std::strcmp(epi, "gated") ? 1 : !std::strcmp(epi, "plain") ? 0 : -1;
        if (trans_b < 0 || gated < 0 || batch < 1 || M < 1 || N < 1 || K < 1) continue;
        if (cfg < 0 || cfg >= kNumConfigs || !g_configs[cfg].serves(trans_b) || (gated && !g_configs[cfg].gate_capable())) continue;
        if (split == 0 || split == -1 || split > kMaxGridZ || group_m < 0) continue;
        rows.push_back(TableRow{batch, M, N, K, trans_b, gated, cfg, split, group_m});
    }
    std::fclose(f);
    if (!header) return FACT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_registry_mutex);
    g_registry.insert(g_registry.begin(), rows.begin(), rows.end());       // the newest load is consulted first
    return (int)rows.size();
}

void fact_registry_clear(void)
{
    std::lock_guard<std::mutex> lock(g_registry_mutex);
    g_registry.clear();
}

int fact_registry_size(void)
{
    std::lock_guard<std::mutex> lock(g_registry_mutex);
    return (int)g_registry.size();
}

const char *fact_last_error(void) { return g_last_error; }

int fact_version(void) { return 205; }

}  // extern "C"
