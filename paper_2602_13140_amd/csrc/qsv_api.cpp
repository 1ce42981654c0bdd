// C-ABI layer of libqsv.so: argument validation, workspace carving, plan cache, launch order.
// Every numeric step runs in the HIP kernels; nothing here touches amplitudes on the host.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <deque>
#include <string>
#include <vector>

#include "qsv.h"
#include "qsv_kernels.h"
#include "qsv_plan.h"

using namespace qsv;

namespace {

constexpr size_t kAlign = 256;
constexpr size_t kOpsRegion = 4u << 20;  // persistent: uploaded pass programs
// Launches whose rows hold at least this many bytes store their tiles nontemporally: the chip's
// last-level cache is 256 MiB, and measured on a 512 MiB state such stores are 4 % faster, on a
// 256 MiB state 3 % slower.
constexpr uint64_t kNtStoreBytes = 384ull << 20;
constexpr int kChunkBits = 12;
constexpr int kMaxBatch = 1 << 24;
constexpr int64_t kMaxAmplitudes = (int64_t)1 << 36;

std::string g_create_error;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int ceil_log2_i64(int64_t v) {
    int b = 0;
    while (((int64_t)1 << b) < v) ++b;
    return b;
}

// A plan the context has built.  Entries are never destroyed before qsv_destroy and never move (a
// std::deque only grows at its end), so pointers to them, and the host arrays uploads read from,
// stay valid for the life of the context: also for a HIP graph that recorded such an upload.
struct CachedPlan {
    qsv_circuit c;
    int inverse, tile, grad, low;   // tile: the resolved tile size (the default depends on the rows)
    int defer = 0;                  // planned with deferred CNOTs (index maps)
    size_t maps_off = 0;            // uint32[plan.maps.size()]: the index maps of its passes
    Plan plan;
    bool resident = false;          // its arrays are in the ops region right now
    size_t dev_off;     // byte offset of the ops inside the ops region
    size_t order_off;   // int32[n_mats]: execution order -> (layer*n + qubit)
    size_t execof_off;  // int32[n_mats]: (layer*n + qubit) -> execution order
    std::vector<int32_t> exec_of;
};

}  // namespace

struct qsv_ctx {
    int n = 0;
    int64_t batch = 0;
    int device = 0;
    hipStream_t stream = nullptr;
    float2* state = nullptr;
    char* ws = nullptr;
    size_t ws_bytes = 0;
    std::string err;
    int opt_tile = 0;
    int opt_naive = 0;
    int opt_low = 0;
    int opt_planes = 1;
    int opt_grad_layered = 1;
    int opt_nt_store = -1;   // -1: by state size
    int opt_rev = -1;        // every other pass takes its tiles in descending order; -1: by state size
    int probe_count = 0;
    int opt_probe_layout = -1;  // probe pass: register run of the load and the store (-1: the highest)
    int64_t opt_grad_chunk = 0;
    int opt_split = -1;      // state rows of a launch sequence in two halves on two streams; -1: by state size
    int opt_prio = 1;        // raised issue priority around a tile's loads and stores (measured: 2 % off configs 3 and 4)
    int opt_small_apply = 1; // qsv_apply_layers runs states of at most 2^21 amplitudes on at most 10 qubits in one launch
    int opt_small_regs = 0;  // qsv_forward_small: amplitudes per thread = 2^this (2..4); 0: by batch size
    int opt_defer = -1;      // qsv_apply_layers defers CNOTs whose target lies outside a pass's tile; -1: when it can
    hipStream_t side = nullptr;          // second stream for that (default priority, non-blocking)
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    bool forked = false;                 // a caller further up already runs two halves on the two streams
    std::deque<CachedPlan> cache;
    size_t ops_used = 0;
};

namespace {

qsv_status fail(qsv_ctx* ctx, qsv_status st, const std::string& msg) {
    if (ctx) ctx->err = msg;
    return st;
}

qsv_status hip_fail(qsv_ctx* ctx, hipError_t e, const char* where) {
    return fail(ctx, QSV_ERR_HIP, std::string(where) + ": " + hipGetErrorString(e));
}

#define QSV_HIP(ctx, expr, where)                                \
    do {                                                         \
        hipError_t e__ = (expr);                                 \
        if (e__ != hipSuccess) return hip_fail(ctx, e__, where); \
    } while (0)

// Per-call scratch carved from the workspace after the persistent ops region.  Work on one
// stream is ordered, so consecutive calls may reuse the same bytes.
struct Arena {
    char* base;
    size_t off, limit;
    bool fixed;      // the library's fixed scratch array instead of the caller's workspace
    explicit Arena(qsv_ctx* c) : base(c->ws), off(kOpsRegion), limit(c->ws_bytes), fixed(false) {}
    Arena(void* fixed_scratch, size_t bytes) : base((char*)fixed_scratch), off(0), limit(bytes), fixed(true) {}
    void* take(size_t bytes) {
        const size_t a = align_up(bytes ? bytes : 1);
        if (off + a > limit) { need = off + a; return nullptr; }
        void* p = base + off;
        off += a;
        return p;
    }
    size_t remaining() const { return limit > off ? limit - off : 0; }
    size_t need = 0;
};

qsv_status ws_fail(qsv_ctx* ctx, const Arena& ar, const char* what) {
    char buf[200];
    if (ar.fixed)
        snprintf(buf, sizeof buf, "%s needs %zu bytes of scratch, more than the fixed array of %zu bytes: "
                 "use the entry point that works in the caller's workspace", what, ar.need, ar.limit);
    else
        snprintf(buf, sizeof buf, "workspace too small for %s: needs at least %zu bytes, has %zu", what,
                 ar.need, ar.limit);
    return fail(ctx, QSV_ERR_WORKSPACE, buf);
}

CircDev to_dev(const qsv_circuit& c, int n) {
    CircDev d;
    d.n = n;
    d.n_layers = c.n_layers;
    d.reupload = c.reupload;
    d.n_rot = c.n_rot;
    for (int i = 0; i < 3; ++i) d.rot[i] = c.rot[i];
    return d;
}

int chunk_blocks(int bits) { return bits > kChunkBits ? 1 << (bits - kChunkBits) : 1; }

bool same_circuit(const qsv_circuit& a, const qsv_circuit& b) {
    if (a.n_layers != b.n_layers || a.reupload != b.reupload || a.n_rot != b.n_rot ||
        a.entangler != b.entangler)
        return false;
    for (int i = 0; i < a.n_rot; ++i)
        if (a.rot[i] != b.rot[i]) return false;
    return true;
}

// Finds or builds the plan and makes sure its arrays are resident in the ops region.  Uploads are
// asynchronous copies on the context's stream from host arrays that live as long as the context.
// When the region is full, every plan in it is dropped from the region (not from the host) and the
// region is filled again from its start: the copies that overwrite it are ordered, on the stream,
// behind every kernel that read the old contents, so nothing waits on the host.
qsv_status get_plan(qsv_ctx* ctx, const qsv_circuit& c, int64_t rows, int inverse, int grad,
                    const CachedPlan** out, int defer = 0) {
    int tile = ctx->opt_tile > 0 ? ctx->opt_tile : default_tile(ctx->n, rows);
    tile = std::max(kMinTile, std::min(kMaxTile, tile));
    CachedPlan* hit = nullptr;
    for (CachedPlan& cp : ctx->cache)
        if (cp.inverse == inverse && cp.tile == tile && cp.grad == grad && cp.low == ctx->opt_low &&
            cp.defer == defer && same_circuit(cp.c, c)) {
            hit = &cp;
            break;
        }
    if (hit && hit->resident) {
        *out = hit;
        return QSV_OK;
    }
    if (!hit) {
        CachedPlan cp;
        cp.c = c;
        cp.inverse = inverse;
        cp.tile = tile;
        cp.grad = grad;
        cp.low = ctx->opt_low;
        cp.defer = defer;
        cp.plan = build_plan(c, ctx->n, rows, inverse != 0, tile, grad != 0, ctx->opt_low, defer != 0);
        if (!cp.plan.complete) return fail(ctx, QSV_ERR_UNSUPPORTED, "internal: pass planner failed");
        const size_t nm = cp.plan.mat_order.size();
        cp.exec_of.assign(nm, 0);
        for (size_t k = 0; k < nm; ++k) cp.exec_of[cp.plan.mat_order[k]] = (int32_t)k;
        ctx->cache.push_back(std::move(cp));
        hit = &ctx->cache.back();
    }
    CachedPlan& cp = *hit;
    const size_t nm = cp.plan.mat_order.size();
    const size_t ops_bytes = align_up(cp.plan.ops.size() * sizeof(Op) + sizeof(Op));
    const size_t tab_bytes = align_up(nm * sizeof(int32_t) + 4);
    const size_t map_bytes = align_up(cp.plan.maps.size() * sizeof(uint32_t) + 4);
    const size_t bytes = ops_bytes + 2 * tab_bytes + map_bytes;
    if (bytes > kOpsRegion) return fail(ctx, QSV_ERR_UNSUPPORTED, "circuit too long for the plan buffer");
    if (ctx->ops_used + bytes > kOpsRegion) {
        // While a call has work on the second stream, kernels there may still read the region, and
        // this upload would not be ordered behind them.
        if (ctx->forked)
            return fail(ctx, QSV_ERR_UNSUPPORTED, "the plans of this call do not fit the plan buffer together");
        for (CachedPlan& other : ctx->cache) other.resident = false;
        ctx->ops_used = 0;
    }
    cp.dev_off = ctx->ops_used;
    cp.order_off = cp.dev_off + ops_bytes;
    cp.execof_off = cp.order_off + tab_bytes;
    cp.maps_off = cp.execof_off + tab_bytes;
    if (!cp.plan.maps.empty())
        QSV_HIP(ctx, hipMemcpyAsync(ctx->ws + cp.maps_off, cp.plan.maps.data(), cp.plan.maps.size() * sizeof(uint32_t),
                                    hipMemcpyHostToDevice, ctx->stream),
                "upload index maps");
    if (!cp.plan.ops.empty())
        QSV_HIP(ctx, hipMemcpyAsync(ctx->ws + cp.dev_off, cp.plan.ops.data(),
                                    cp.plan.ops.size() * sizeof(Op), hipMemcpyHostToDevice, ctx->stream),
                "upload plan");
    if (nm) {
        QSV_HIP(ctx, hipMemcpyAsync(ctx->ws + cp.order_off, cp.plan.mat_order.data(), nm * sizeof(int32_t),
                                    hipMemcpyHostToDevice, ctx->stream),
                "upload matrix order");
        QSV_HIP(ctx, hipMemcpyAsync(ctx->ws + cp.execof_off, cp.exec_of.data(), nm * sizeof(int32_t),
                                    hipMemcpyHostToDevice, ctx->stream),
                "upload matrix order");
    }
    ctx->ops_used += bytes;
    cp.resident = true;
    *out = &cp;
    return QSV_OK;
}

RowMap plain_rows(int n) {
    RowMap rm;
    rm.grad = 0; rm.two_p = 0; rm.per = 1; rm.row0 = 0; rm.slots_n = 1; rm.n = n;
    return rm;
}

// What a circuit needs before it can run: the pass plan (fused path) and the fused matrices, which
// are laid out in the plan's execution order (natural order on the one-gate-per-launch path).
struct Prepared {
    const CachedPlan* cp = nullptr;  // null: one-gate-per-launch path
    float* mats = nullptr;
    int mat_stride = 0;              // matrices per sample in a per-sample table; 0: those of the circuit run
};

size_t mats_table_bytes(const qsv_circuit& c, int n, int64_t samples) {
    // one extra entry: the interpreter prefetches the matrix after the one it is using
    return align_up(((size_t)(c.reupload ? samples : 1) * c.n_layers * n + 1) * 32);
}

// the matrix table followed by the builder's side buffer
size_t mats_bytes(const qsv_circuit& c, int n, int64_t samples) {
    return mats_table_bytes(c, n, samples) + align_up(build_mats_side_bytes(to_dev(c, n), samples));
}

qsv_status prepare_circuit(qsv_ctx* ctx, const qsv_circuit& c, int64_t rows, int inverse, int grad,
                           const float* params, const float* feats, int64_t samples, float* mats,
                           Prepared* out, int defer = 0) {
    const int n = ctx->n;
    const bool has_u = (c.reupload + c.n_rot) > 0 && c.n_layers > 0;
    out->mats = mats;
    out->cp = nullptr;
    const int* order = nullptr;
    const int* exec_of = nullptr;
    if (!(ctx->opt_naive || n < kRegBits)) {
        qsv_status st = get_plan(ctx, c, rows, inverse, grad, &out->cp, defer);
        if (st != QSV_OK) return st;
        order = reinterpret_cast<const int*>(ctx->ws + out->cp->order_off);
        exec_of = reinterpret_cast<const int*>(ctx->ws + out->cp->execof_off);
    }
    if (has_u) {
        double* side = reinterpret_cast<double*>(reinterpret_cast<char*>(mats) + mats_table_bytes(c, n, samples));
        QSV_HIP(ctx, launch_build_mats(to_dev(c, n), params, feats, samples, inverse, order, exec_of, mats, side,
                                       ctx->stream),
                "build matrices");
    }
    return QSV_OK;
}

// The same for the layers of c run one by one as one-layer circuits (`one` = c with n_layers = 1):
// the plan is the one-layer circuit's, and the matrices of all layers are built by one launch, every
// layer's in that plan's order; layer l then runs with layer_of(prepared, l).
qsv_status prepare_layers(qsv_ctx* ctx, const qsv_circuit& c, const qsv_circuit& one, int64_t rows, int inverse,
                          const float* params, const float* feats, int64_t samples, float* mats, Prepared* out) {
    const int n = ctx->n;
    const bool has_u = (c.reupload + c.n_rot) > 0 && c.n_layers > 0;
    out->mats = mats;
    out->cp = nullptr;
    out->mat_stride = c.n_layers * n;
    const int* order = nullptr;
    const int* exec_of = nullptr;
    if (!(ctx->opt_naive || n < kRegBits)) {
        qsv_status st = get_plan(ctx, one, rows, inverse, 0, &out->cp);
        if (st != QSV_OK) return st;
        order = reinterpret_cast<const int*>(ctx->ws + out->cp->order_off);
        exec_of = reinterpret_cast<const int*>(ctx->ws + out->cp->execof_off);
    }
    if (has_u) {
        double* side = reinterpret_cast<double*>(reinterpret_cast<char*>(mats) + mats_table_bytes(c, n, samples));
        QSV_HIP(ctx, launch_build_mats(to_dev(c, n), params, feats, samples, inverse, order, exec_of, mats, side,
                                       ctx->stream, order ? n : 0),
                "build matrices");
    }
    return QSV_OK;
}

inline Prepared layer_of(const Prepared& all, int l, int n) {
    Prepared pr = all;
    pr.mats = all.mats + (size_t)l * n * 8;
    return pr;
}

// Runs the prepared circuit on `rows` state rows starting at `state`.
// src (optional): per-sample start states [samples][2^n]; the rows then start from the state of
// their sample.  The fused path reads them in its first pass when a tile never spans two rows,
// otherwise a copy pass fills the rows first.
// zs (optional): what the gradient wants of the final states, <Z_q> per row scattered into out.
// The fused path computes it in its last pass (which then stores nothing) when a tile never spans
// two rows; otherwise the reduction kernels read the final states.  zpart: room for partials.
struct ZSpec { int q; double* out; Scatter sc; double* zpart; };

// pong (needed when the plan defers CNOTs): a second buffer of the state's shape.  A pass with an
// index map reads one buffer and writes the other; the result always ends up in `state`.
qsv_status run_circuit(qsv_ctx* ctx, const qsv_circuit& c, const Prepared& pr, float2* state, int64_t rows,
                       int inverse, const float* ovr, const RowMap& rm, const float2* src = nullptr,
                       const ZSpec* zs = nullptr, float2* pong = nullptr) {
    const int n = ctx->n;
    const bool has_u = (c.reupload + c.n_rot) > 0;
    const int n_mats = has_u ? (pr.mat_stride > 0 ? pr.mat_stride : c.n_layers * n) : 0;
    const float* mats = pr.mats;
    const bool src_in_pass = src && pr.cp && n >= pr.cp->plan.tile && !pr.cp->plan.passes.empty();
    if (src && !src_in_pass)
        QSV_HIP(ctx, launch_gather_rows(src, n, rows, rm, state, ctx->stream), "gather rows");
    auto z_after = [&]() -> qsv_status {
        if (!zs) return QSV_OK;
        QSV_HIP(ctx, launch_expz_block(state, rows, n, zs->zpart, ctx->stream), "expz block");
        QSV_HIP(ctx, launch_expz_finish_scatter(zs->zpart, rows, n, zs->q, zs->out, zs->sc, ctx->stream),
                "expz finish");
        return QSV_OK;
    };
    if (!pr.cp) {
        auto layer_u = [&](int l) -> hipError_t {
            if (!has_u) return hipSuccess;
            for (int q = 0; q < n; ++q) {
                hipError_t e = launch_naive_u(state, rows, n, q, mats, ovr, l * n + q, n_mats,
                                              c.reupload, rm, ctx->stream);
                if (e != hipSuccess) return e;
            }
            return hipSuccess;
        };
        for (int li = 0; li < c.n_layers; ++li) {
            const int l = inverse ? c.n_layers - 1 - li : li;
            if (!inverse) QSV_HIP(ctx, layer_u(l), "naive rotation");
            if (c.entangler == QSV_ENT_CNOT_RING && n >= 2) {
                for (int i = 0; i < n; ++i) {
                    const int q = inverse ? n - 1 - i : i;
                    QSV_HIP(ctx, launch_naive_cnot(state, rows, n, q, (q + 1) % n, ctx->stream),
                            "naive cnot");
                }
            }
            if (c.entangler == QSV_ENT_CZ_LADDER && n >= 2)
                QSV_HIP(ctx, launch_naive_cz_ladder(state, rows, n, ctx->stream), "naive cz");
            if (inverse) QSV_HIP(ctx, layer_u(l), "naive rotation");
        }
        return z_after();
    }
    const CachedPlan* cp = pr.cp;
    if (!cp->resident) return fail(ctx, QSV_ERR_UNSUPPORTED, "internal: the plan was dropped from the plan buffer before use");
    const Plan& pl = cp->plan;
    const int ext = n + ceil_log2_i64(rows);
    const uint64_t n_tiles = ext > pl.tile ? (1ull << (ext - pl.tile)) : 1ull;
    const Op* dev_ops = reinterpret_cast<const Op*>(ctx->ws + cp->dev_off);
    const bool z_in_pass = zs && n >= pl.tile && !pl.passes.empty();
    // Two rows or more: the rows go through the passes as two halves on two streams.  The halves
    // never meet (a tile lies inside one row when n > tile, and the geometry of the passes does not
    // depend on the number of rows), and each one's launch gaps and tails are covered by the
    // other's kernels: measured 7-13 % off the whole sequence from 16 to 256 MiB, 3.5 % at 384 and
    // 512 MiB, 1.2 % at 1 GiB.
    const uint64_t state_bytes = ((uint64_t)rows << n) * 8;
    const bool split = rows >= 2 && n > pl.tile && pl.passes.size() >= 2 &&
                       ctx->opt_split != 0 && !ctx->forked;
    const int64_t rows_a = split ? rows / 2 : rows, rows_b = rows - rows_a;
    struct Join {      // the second stream always rejoins the caller's, also when a launch fails
        qsv_ctx* c; bool on;
        ~Join() {
            if (!on) return;
            if (hipEventRecord(c->ev_join, c->side) == hipSuccess) (void)hipStreamWaitEvent(c->stream, c->ev_join, 0);
        }
    } join{ctx, false};
    if (split) {
        QSV_HIP(ctx, hipEventRecord(ctx->ev_fork, ctx->stream), "fork");
        QSV_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0), "fork");
        join.on = true;
    }
    auto tiles_of = [&](int64_t r) -> uint64_t {
        const int e = n + ceil_log2_i64(r);
        return e > pl.tile ? (1ull << (e - pl.tile)) : 1ull;
    };
    const int waves_per_group = std::max(1, (1 << (pl.tile - kRegBits)) / 64);
    // Which passes change buffers: those with an index map must; when their number is odd, one pass
    // without a map changes too (any pass may), so that the last one writes into `state`.  A plan in
    // which every pass has a map and their number is odd ends with a copy.
    size_t n_mapped = 0, extra_switch = pl.passes.size();
    for (const Pass& ps : pl.passes) n_mapped += ps.map_begin >= 0;
    if (n_mapped && (!pong || src || zs || n > 28))
        return fail(ctx, QSV_ERR_UNSUPPORTED, "internal: a plan with deferred CNOTs needs a second buffer");
    if (n_mapped & 1)
        for (size_t pi = 0; pi < pl.passes.size(); ++pi)
            if (pl.passes[pi].map_begin < 0) { extra_switch = pi; break; }
    float2* cur = state;
    bool first = true;
    for (size_t pi = 0; pi < pl.passes.size(); ++pi) {
        const Pass& ps = pl.passes[pi];
        PassArgs a;
        const bool switches = ps.map_begin >= 0 || pi == extra_switch;
        float2* const dst = switches ? (cur == state ? pong : state) : cur;
        a.state = dst;
        a.in = cur;
        a.imap = ps.map_begin >= 0 ? reinterpret_cast<const unsigned*>(ctx->ws + cp->maps_off) + ps.map_begin : nullptr;
        cur = dst;
        a.src = (first && src_in_pass) ? src : nullptr;
        first = false;
        const bool last = pi + 1 == pl.passes.size();
        a.zout = (last && z_in_pass) ? zs->zpart : nullptr;
        a.zq = zs ? zs->q : 0;
        a.nostore = a.zout ? 1 : 0;
        a.ops = dev_ops + ps.op_begin;
        a.mats = mats;
        a.exec_of = reinterpret_cast<const int*>(ctx->ws + cp->execof_off);
        a.ovr = ovr;
        a.total = (uint64_t)rows_a << n;
        a.nt_store = ctx->opt_nt_store >= 0 ? ctx->opt_nt_store : (state_bytes >= kNtStoreBytes ? 1 : 0);
        // Every other pass walks the tiles downwards, so that it starts with what the pass before
        // wrote last and may still find in the memory-side cache (256 MiB).
        a.rev = (ctx->opt_rev >= 0 ? ctx->opt_rev : (state_bytes >= kNtStoreBytes ? 1 : 0)) ? (int)(pi & 1) : 0;
        a.prio = ctx->opt_prio;
        a.n = n; a.c = ps.c; a.w = ps.w;
        a.n_mats = n_mats;
        a.rowdep = c.reupload;
        a.rm = rm;
        QSV_HIP(ctx, launch_pass(pl.tile, ctx->opt_planes, a, split ? tiles_of(rows_a) : n_tiles, ctx->stream), "fused pass");
        if (!split) continue;
        // second half: rows rows_a .. rows - 1.  With a gradient row map the kernel works with global
        // row numbers (row0 moves); otherwise a row's matrices and start state are found relative to
        // the launch, so those pointers move with the state.
        PassArgs b = a;
        b.state = a.state + ((uint64_t)rows_a << n);
        b.in = a.in + ((uint64_t)rows_a << n);
        b.total = (uint64_t)rows_b << n;
        if (rm.grad) {
            b.rm.row0 = rm.row0 + rows_a;
        } else {
            if (b.src) b.src = b.src + ((uint64_t)rows_a << n);
            if (c.reupload && b.mats) b.mats = b.mats + (uint64_t)rows_a * (uint64_t)n_mats * 8;
        }
        if (b.zout) b.zout = b.zout + (uint64_t)rows_a * ((uint64_t)1 << (n - pl.tile)) * (uint64_t)waves_per_group;
        QSV_HIP(ctx, launch_pass(pl.tile, ctx->opt_planes, b, tiles_of(rows_b), ctx->side), "fused pass");
    }
    if (split) {       // what follows on the caller's stream sees both halves
        join.on = false;
        QSV_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->side), "join");
        QSV_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0), "join");
    }
    if (cur != state)
        QSV_HIP(ctx, hipMemcpyAsync(state, cur, state_bytes, hipMemcpyDeviceToDevice, ctx->stream), "copy back");
    if (z_in_pass) {
        // partials per row: tiles of the row x wavefronts of a workgroup
        const int64_t per_row = ((int64_t)1 << (n - pl.tile)) * (((int64_t)1 << (pl.tile - kRegBits)) / 64 > 0
                                                                    ? ((int64_t)1 << (pl.tile - kRegBits)) / 64 : 1);
        QSV_HIP(ctx, launch_zsum_finish(zs->zpart, rows, per_row, zs->out, zs->sc, ctx->stream), "z finish");
        return QSV_OK;
    }
    return z_after();
}

qsv_status bind_device(qsv_ctx* ctx) {
    QSV_HIP(ctx, hipSetDevice(ctx->device), "hipSetDevice");
    return QSV_OK;
}

}  // namespace

// ================================================================================================
extern "C" {

int64_t qsv_num_params(const qsv_circuit* c, int n_qubits) {
    if (!check_circuit(c, n_qubits, nullptr)) return -1;
    return (int64_t)c->n_layers * (c->reupload + c->n_rot) * n_qubits;
}

size_t qsv_workspace_bytes(int n_qubits, int batch) {
    if (n_qubits < 1 || n_qubits > 30 || batch < 1) return 0;
    const size_t n = (size_t)n_qubits, B = (size_t)batch;
    const size_t row_bytes = ((size_t)8) << n;
    size_t total = kOpsRegion;
    total += align_up(B * 64 * n * 32 + 32) + align_up(B * 64 * (n * 16 + 64));  // per-sample matrices + builder's side buffer, 64 layers
    total += align_up(B * 2 * (16 * 4 * n) * 32);             // shifted matrices, 16 layers x 4 slots
    total += align_up(B * (2 * 64 * 4 * n + 1) * 8);          // gradient values f[B][2P+1]
    total += align_up(B * (size_t)chunk_blocks(n_qubits) * 13 * 8 * 2);  // reduction partials
    total += align_up(B * 16) * 4;                            // norms, scales
    const size_t grad_states = row_bytes * 4 > ((size_t)256 << 20) ? row_bytes * 4 : ((size_t)256 << 20);
    total += grad_states + (8u << 20);
    // the second state buffer of qsv_apply_layers with deferred CNOTs (it shares the bytes above with the
    // gradient's circuit states; this makes sure a copy of the whole state fits whatever the batch)
    if (n_qubits <= 28 && B * row_bytes > grad_states) total += align_up(B * row_bytes - grad_states);
    return total;
}

size_t qsv_grad_workspace_bytes(int n_qubits, int batch, const qsv_circuit* c) {
    const size_t base = qsv_workspace_bytes(n_qubits, batch);
    if (base == 0 || !check_circuit(c, n_qubits, nullptr)) return 0;
    const size_t state_bytes = (size_t)8 << n_qubits;
    return base + align_up((size_t)batch * (size_t)(c->n_layers + 1) * state_bytes) + 4 * kAlign;
}

qsv_status qsv_create(qsv_ctx** out, int n_qubits, int batch, int device, void* hip_stream,
                      void* state_dev, void* ws_dev, size_t ws_bytes) {
    if (!out) { g_create_error = "out is NULL"; return QSV_ERR_INVALID_ARG; }
    *out = nullptr;
    if (n_qubits < 1 || n_qubits > 30) { g_create_error = "n_qubits must be in 1..30"; return QSV_ERR_INVALID_ARG; }
    if (batch < 1 || batch > kMaxBatch || ((int64_t)batch << n_qubits) > kMaxAmplitudes) {
        g_create_error = "batch must be in 1..2^24 with batch * 2^n_qubits <= 2^36";
        return QSV_ERR_INVALID_ARG;
    }
    if (device < 0) { g_create_error = "device must be >= 0"; return QSV_ERR_INVALID_ARG; }
    if (!state_dev || !ws_dev) { g_create_error = "state_dev and ws_dev must not be NULL"; return QSV_ERR_INVALID_ARG; }
    if (((uintptr_t)state_dev & 15) || ((uintptr_t)ws_dev & 255)) {
        g_create_error = "state_dev must be 16-byte aligned and ws_dev 256-byte aligned";
        return QSV_ERR_INVALID_ARG;
    }
    if (ws_bytes < qsv_workspace_bytes(n_qubits, batch)) {
        g_create_error = "workspace smaller than qsv_workspace_bytes(n_qubits, batch)";
        return QSV_ERR_WORKSPACE;
    }
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = set_pass_attributes();
    if (e != hipSuccess) {
        g_create_error = std::string("HIP initialisation failed: ") + hipGetErrorString(e);
        return QSV_ERR_HIP;
    }
    qsv_ctx* ctx = new qsv_ctx();
    ctx->n = n_qubits;
    ctx->batch = batch;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->state = static_cast<float2*>(state_dev);
    ctx->ws = static_cast<char*>(ws_dev);
    ctx->ws_bytes = ws_bytes;
    e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
    if (e != hipSuccess) {
        g_create_error = std::string("creating the second stream failed: ") + hipGetErrorString(e);
        qsv_destroy(ctx);
        return QSV_ERR_HIP;
    }
    *out = ctx;
    return QSV_OK;
}

void qsv_destroy(qsv_ctx* ctx) {
    if (!ctx) return;
    if (hipSetDevice(ctx->device) == hipSuccess) {
        if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
        if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
        if (ctx->side) (void)hipStreamDestroy(ctx->side);
    }
    delete ctx;
}

const char* qsv_last_error(const qsv_ctx* ctx) {
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

qsv_status qsv_set_option(qsv_ctx* ctx, const char* name, int64_t value) {
    if (!ctx || !name) return QSV_ERR_INVALID_ARG;
    if (!strcmp(name, "tile_log2")) {
        if (value != 0 && (value < kMinTile || value > kMaxTile))
            return fail(ctx, QSV_ERR_INVALID_ARG, "tile_log2 must be 0 or in 10..14");
        ctx->opt_tile = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "low_bits")) {
        if (value != 0 && (value < 3 || value > kMinTile))
            return fail(ctx, QSV_ERR_INVALID_ARG, "low_bits must be 0 or in 3..10");
        ctx->opt_low = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "lds_planes")) {
        if (value != 1 && value != 2)
            return fail(ctx, QSV_ERR_INVALID_ARG, "lds_planes must be 1 or 2");
        ctx->opt_planes = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "grad_chunk_rows")) {
        if (value < 0 || value > 32768) return fail(ctx, QSV_ERR_INVALID_ARG, "grad_chunk_rows must be in 0..32768");
        ctx->opt_grad_chunk = value;
        return QSV_OK;
    }
    if (!strcmp(name, "reverse_passes")) {
        if (value < -1 || value > 1) return fail(ctx, QSV_ERR_INVALID_ARG, "reverse_passes must be -1, 0 or 1");
        ctx->opt_rev = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "split_streams")) {
        if (value < -1 || value > 1) return fail(ctx, QSV_ERR_INVALID_ARG, "split_streams must be -1, 0 or 1");
        ctx->opt_split = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "load_store_priority")) {
        if (value < 0 || value > 1) return fail(ctx, QSV_ERR_INVALID_ARG, "load_store_priority must be 0 or 1");
        ctx->opt_prio = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "small_apply")) {
        if (value < 0 || value > 1) return fail(ctx, QSV_ERR_INVALID_ARG, "small_apply must be 0 or 1");
        ctx->opt_small_apply = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "small_regs")) {
        if (value != 0 && (value < 2 || value > 4)) return fail(ctx, QSV_ERR_INVALID_ARG, "small_regs must be 0, 2, 3 or 4");
        ctx->opt_small_regs = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "defer_cnots")) {
        if (value < -1 || value > 1) return fail(ctx, QSV_ERR_INVALID_ARG, "defer_cnots must be -1, 0 or 1");
        ctx->opt_defer = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "probe_layout")) {
        if (value < -1 || value > kMaxTile - kRegBits)
            return fail(ctx, QSV_ERR_INVALID_ARG, "probe_layout must be -1 or in 0..10");
        ctx->opt_probe_layout = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "nt_store")) {
        if (value < -1 || value > 1) return fail(ctx, QSV_ERR_INVALID_ARG, "nt_store must be -1, 0 or 1");
        ctx->opt_nt_store = (int)value;
        return QSV_OK;
    }
    if (!strcmp(name, "grad_layered")) {
        ctx->opt_grad_layered = value != 0;
        return QSV_OK;
    }
    if (!strcmp(name, "naive")) {
        ctx->opt_naive = value != 0;
        return QSV_OK;
    }
    return fail(ctx, QSV_ERR_INVALID_ARG, std::string("unknown option ") + name);
}

qsv_status qsv_amp_encode(qsv_ctx* ctx, const float* x_dev, int64_t dim, float* norm_out_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    if (!x_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "x_dev is NULL");
    if (dim < 1 || dim > ((int64_t)1 << ctx->n)) return fail(ctx, QSV_ERR_INVALID_ARG, "dim must be in 1..2^n");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    Arena ar(ctx);
    int nblk = (int)((dim + 4095) / 4096);
    if (nblk > 1024) nblk = 1024;
    double* partial = (double*)ar.take((size_t)ctx->batch * nblk * 8);
    double* inv = (double*)ar.take((size_t)ctx->batch * 8);
    if (!partial || !inv) return ws_fail(ctx, ar, "qsv_amp_encode");
    if (dim <= 4096 && ctx->n <= 12) {     // a block covers a sample: one launch
        QSV_HIP(ctx, launch_encode_small(x_dev, ctx->batch, dim, ctx->n, inv, norm_out_dev, ctx->state, ctx->stream),
                "encode");
        return QSV_OK;
    }
    QSV_HIP(ctx, launch_norms(x_dev, ctx->batch, dim, partial, nblk, inv, norm_out_dev, ctx->stream), "norms");
    QSV_HIP(ctx, launch_encode_write(x_dev, dim, ctx->n, ctx->batch, inv, plain_rows(ctx->n), ctx->state,
                                     ctx->stream),
            "encode");
    return QSV_OK;
}

qsv_status qsv_apply_layers(qsv_ctx* ctx, const qsv_circuit* c, const float* params_dev,
                            const float* feats_dev, int inverse) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    std::string why;
    if (!check_circuit(c, ctx->n, &why)) return fail(ctx, QSV_ERR_INVALID_ARG, why);
    if (inverse != 0 && inverse != 1) return fail(ctx, QSV_ERR_INVALID_ARG, "inverse must be 0 or 1");
    const int64_t P = qsv_num_params(c, ctx->n);
    if (P > 0 && !params_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "params_dev is NULL");
    if (c->reupload && !feats_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "reupload = 1 needs feats_dev");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    // States small enough that launches cost more than arithmetic: the whole call in one launch, gates in
    // registers and lane exchanges (the kernel of qsv_forward_small, started from the state).
    if (ctx->opt_small_apply != 0 && ctx->n <= kSmallMaxQubits && ctx->opt_tile == 0 && !ctx->opt_naive &&
        ((int64_t)ctx->batch << ctx->n) <= kSmallApplyAmplitudes) {
        const CircDev cd = to_dev(*c, ctx->n);
        const int regs = ctx->opt_small_regs ? ctx->opt_small_regs : small_choose_regs(cd, ctx->batch);
        if (regs != 0 && ctx->n - regs <= 8 && small_mats_per_group(cd, regs) <= kSmallMats) {
            QSV_HIP(ctx, launch_forward_small(regs, nullptr, 0, ctx->batch, cd, c->entangler, params_dev, feats_dev, inverse,
                                              inverse, 0, ctx->state, nullptr, nullptr, ctx->stream),
                    "apply_small");
            return QSV_OK;
        }
    }
    Arena ar(ctx);
    float* mats = (float*)ar.take(mats_bytes(*c, ctx->n, ctx->batch));
    if (!mats) return ws_fail(ctx, ar, "qsv_apply_layers");
    // CNOTs whose target lies outside a pass's tile can be carried by the pass's index map (fewer
    // passes over the state); such passes write a second buffer, taken from the workspace.
    const size_t state_bytes = ((size_t)ctx->batch << ctx->n) * 8;
    float2* pong = nullptr;
    int defer = 0;
    if (ctx->opt_defer != 0 && c->entangler == QSV_ENT_CNOT_RING && ctx->n <= 28 && !ctx->opt_naive &&
        ar.remaining() >= align_up(state_bytes)) {
        int tile = ctx->opt_tile > 0 ? ctx->opt_tile : default_tile(ctx->n, ctx->batch);
        if (ctx->n > tile) {
            pong = (float2*)ar.take(state_bytes);
            defer = pong ? 1 : 0;
        }
    }
    Prepared pr;
    st = prepare_circuit(ctx, *c, ctx->batch, inverse, 0, params_dev, feats_dev, ctx->batch, mats, &pr, defer);
    if (st != QSV_OK) return st;
    return run_circuit(ctx, *c, pr, ctx->state, ctx->batch, inverse, nullptr, plain_rows(ctx->n), nullptr, nullptr, pong);
}

// Every measurement kind; ar is where the kernels' partial results go (the caller's workspace, or the
// library's fixed scratch array).  The partials are written in full before they are read, so the
// bytes need no clearing between calls.
static qsv_status measure_impl(qsv_ctx* ctx, const qsv_measure_req* req, Arena& ar) {
    if (!req) return fail(ctx, QSV_ERR_INVALID_ARG, "req is NULL");
    if (!req->out_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "out_dev is NULL");
    if (req->reserved != 0) return fail(ctx, QSV_ERR_INVALID_ARG, "reserved must be 0");
    const int n = ctx->n;
    const int64_t B = ctx->batch;
    const uint64_t full = (n >= 64) ? ~0ull : ((1ull << n) - 1);
    qsv_status st;
    switch (req->kind) {
        case QSV_M_PROBS: {
            if ((st = bind_device(ctx)) != QSV_OK) return st;
            QSV_HIP(ctx, launch_probs(ctx->state, (uint64_t)B << n, (float*)req->out_dev, ctx->stream),
                    "probs");
            return QSV_OK;
        }
        case QSV_M_EXPZ_ALL:
        case QSV_M_EXPZ_ONE: {
            const int q = req->kind == QSV_M_EXPZ_ONE ? req->qubit : -1;
            if (req->kind == QSV_M_EXPZ_ONE && (q < 0 || q >= n))
                return fail(ctx, QSV_ERR_INVALID_ARG, "qubit out of range");
            if ((st = bind_device(ctx)) != QSV_OK) return st;
            if (chunk_blocks(n) == 1) {           // a row is one chunk: no partial sums to combine
                QSV_HIP(ctx, launch_expz_small(ctx->state, B, n, q, (float*)req->out_dev, ctx->stream), "expz");
                return QSV_OK;
            }
            double* partial = (double*)ar.take((size_t)B * chunk_blocks(n) * 13 * 8);
            if (!partial) return ws_fail(ctx, ar, "qsv_measure(EXPZ)");
            QSV_HIP(ctx, launch_expz_block(ctx->state, B, n, partial, ctx->stream), "expz block");
            QSV_HIP(ctx, launch_expz_finish(partial, B, n, q, (float*)req->out_dev, nullptr, ctx->stream),
                    "expz finish");
            return QSV_OK;
        }
        case QSV_M_MARGINAL:
        case QSV_M_PROJECT_ZERO: {
            if (req->mask == 0 || (req->mask & ~full)) return fail(ctx, QSV_ERR_INVALID_ARG, "mask must be a non-empty subset of the qubits");
            const int m = __builtin_popcountll(req->mask);
            const bool proj = req->kind == QSV_M_PROJECT_ZERO;
            if (!proj && m > 20) return fail(ctx, QSV_ERR_UNSUPPORTED, "marginal over more than 20 qubits");
            if (proj && req->renormalise != 0 && req->renormalise != 1)
                return fail(ctx, QSV_ERR_INVALID_ARG, "renormalise must be 0 or 1");
            const int64_t n_v = proj ? 1 : ((int64_t)1 << m);
            const int64_t nblk = chunk_blocks(n - m);
            if ((uint64_t)B * (uint64_t)n_v * (uint64_t)nblk > 0x7fffffffull)
                return fail(ctx, QSV_ERR_UNSUPPORTED, "marginal too large for one launch");
            if ((st = bind_device(ctx)) != QSV_OK) return st;
            double* partial = (double*)ar.take((size_t)B * n_v * nblk * 8);
            double* scale = (double*)ar.take((size_t)B * 8);
            if (!partial || !scale) return ws_fail(ctx, ar, "qsv_measure(MARGINAL/PROJECT)");
            QSV_HIP(ctx, launch_marginal_block(ctx->state, B, n, req->mask, n_v, partial, ctx->stream),
                    "marginal block");
            QSV_HIP(ctx, launch_marginal_finish(partial, B * n_v, nblk, (float*)req->out_dev,
                                                proj ? (req->renormalise ? 2 : 1) : 0, scale, ctx->stream),
                    "marginal finish");
            if (proj)
                QSV_HIP(ctx, launch_project(ctx->state, B, n, req->mask, scale, ctx->stream), "project");
            return QSV_OK;
        }
        case QSV_M_FIDELITY: {
            if (!req->x_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "x_dev is NULL");
            if (req->dim < 1 || req->dim > ((int64_t)1 << n)) return fail(ctx, QSV_ERR_INVALID_ARG, "dim must be in 1..2^n");
            if ((st = bind_device(ctx)) != QSV_OK) return st;
            int nblk = (int)((req->dim + 4095) / 4096);
            if (nblk > 1024) nblk = 1024;
            double* partial = (double*)ar.take((size_t)B * nblk * 3 * 8);
            if (!partial) return ws_fail(ctx, ar, "qsv_measure(FIDELITY)");
            QSV_HIP(ctx, launch_fidelity_block(ctx->state, B, n, req->x_dev, req->dim, partial, nblk, plain_rows(n), ctx->stream),
                    "fidelity block");
            QSV_HIP(ctx, launch_fidelity_finish(partial, nblk, B, (float*)req->out_dev, nullptr, ctx->stream),
                    "fidelity finish");
            return QSV_OK;
        }
        case QSV_M_SAMPLE: {
            if (req->shots < 0) return fail(ctx, QSV_ERR_INVALID_ARG, "shots must be >= 0");
            if (req->shots > 0 && !req->uniforms_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "uniforms_dev is NULL");
            if ((st = bind_device(ctx)) != QSV_OK) return st;
            unsigned long long* cum = (unsigned long long*)ar.take((size_t)B * chunk_blocks(n) * 8);
            if (!cum) return ws_fail(ctx, ar, "qsv_measure(SAMPLE)");
            QSV_HIP(ctx, launch_sample(ctx->state, B, n, req->uniforms_dev, req->shots, cum,
                                       (long long*)req->out_dev, ctx->stream),
                    "sample");
            return QSV_OK;
        }
        default:
            return fail(ctx, QSV_ERR_INVALID_ARG, "unknown measurement kind");
    }
}

qsv_status qsv_forward_small(qsv_ctx* ctx, const float* x_dev, int64_t dim, const qsv_circuit* c,
                             const float* params_dev, const float* feats_dev, int decode, int kind, void* out_dev,
                             float* norm_out_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    if (!x_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "x_dev is NULL");
    if (dim < 1 || dim > ((int64_t)1 << ctx->n)) return fail(ctx, QSV_ERR_INVALID_ARG, "dim must be in 1..2^n");
    std::string why;
    if (!check_circuit(c, ctx->n, &why)) return fail(ctx, QSV_ERR_INVALID_ARG, why);
    if (decode != 0 && decode != 1) return fail(ctx, QSV_ERR_INVALID_ARG, "decode must be 0 or 1");
    if (kind != QSV_M_PROBS && kind != QSV_M_EXPZ_ALL)
        return fail(ctx, QSV_ERR_INVALID_ARG, "kind must be QSV_M_PROBS or QSV_M_EXPZ_ALL");
    if (!out_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "out_dev is NULL");
    const int64_t P = qsv_num_params(c, ctx->n);
    if (P > 0 && !params_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "params_dev is NULL");
    if (c->reupload && !feats_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "reupload = 1 needs feats_dev");
    if (ctx->n > kSmallMaxQubits)
        return fail(ctx, QSV_ERR_UNSUPPORTED, "qsv_forward_small takes at most 10 qubits: use the separate calls");
    const CircDev cd = to_dev(*c, ctx->n);
    int regs = ctx->opt_small_regs;
    if (regs == 0) regs = small_choose_regs(cd, ctx->batch);
    if (regs == 0 || ctx->n - regs > 8 || small_mats_per_group(cd, regs) > kSmallMats)
        return fail(ctx, QSV_ERR_UNSUPPORTED,
                    "qsv_forward_small keeps at most 512 matrices per workgroup (layers * qubits, times the samples "
                    "that share a wavefront when the circuit re-uploads data): use the separate calls");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    QSV_HIP(ctx, launch_forward_small(regs, x_dev, dim, ctx->batch, cd, c->entangler, params_dev, feats_dev, 0, decode, kind,
                                      ctx->state, (float*)out_dev, norm_out_dev, ctx->stream),
            "forward_small");
    return QSV_OK;
}

qsv_status qsv_measure(qsv_ctx* ctx, const qsv_measure_req* req) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    Arena ar(ctx);
    return measure_impl(ctx, req, ar);
}

qsv_status qsv_measure_static(qsv_ctx* ctx, const qsv_measure_req* req) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    void* fixed = nullptr;     // this device's copy of the fixed array (address looked up once per device)
    QSV_HIP(ctx, static_scratch(ctx->device, &fixed), "address of the fixed scratch array");
    Arena ar(fixed, kStaticScratchBytes);
    return measure_impl(ctx, req, ar);
}

qsv_status qsv_pauli_expect(qsv_ctx* ctx, uint64_t xmask, uint64_t ymask, uint64_t zmask, float* out_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    const int n = ctx->n;
    if (!out_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "out_dev is NULL");
    if ((xmask & ymask) || (xmask & zmask) || (ymask & zmask))
        return fail(ctx, QSV_ERR_INVALID_ARG, "xmask, ymask and zmask must not overlap");
    if ((xmask | ymask | zmask) >> n) return fail(ctx, QSV_ERR_INVALID_ARG, "mask names a qubit >= n_qubits");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    Arena ar(ctx);
    double* partial = (double*)ar.take((size_t)ctx->batch * chunk_blocks(n) * 2 * 8);
    if (!partial) return ws_fail(ctx, ar, "qsv_pauli_expect");
    QSV_HIP(ctx, launch_pauli(ctx->state, ctx->batch, n, xmask, ymask, zmask, partial, out_dev, ctx->stream),
            "pauli expectation");
    return QSV_OK;
}

qsv_status qsv_reset_fidelity(qsv_ctx* ctx, const qsv_circuit* c, const float* params_dev,
                              const float* feats_dev, uint64_t mask, const float* x_dev, int64_t dim,
                              float* out_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    std::string why;
    if (!check_circuit(c, ctx->n, &why)) return fail(ctx, QSV_ERR_INVALID_ARG, why);
    const int n = ctx->n;
    const int64_t B = ctx->batch;
    const int64_t P = qsv_num_params(c, n);
    if (P > 0 && !params_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "params_dev is NULL");
    if (c->reupload && !feats_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "reupload = 1 needs feats_dev");
    if (!x_dev || !out_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "x_dev or out_dev is NULL");
    if (dim < 1 || dim > ((int64_t)1 << n)) return fail(ctx, QSV_ERR_INVALID_ARG, "dim must be in 1..2^n");
    if (mask == 0 || (mask >> n) != 0) return fail(ctx, QSV_ERR_INVALID_ARG, "mask must be a non-empty subset of the qubits");
    const int m = __builtin_popcountll(mask);
    if (m > 10) return fail(ctx, QSV_ERR_UNSUPPORTED, "reset of more than 10 qubits");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    const int64_t per = (int64_t)1 << m;
    const int64_t rows_all = B * per;
    Arena ar(ctx);
    const size_t state_bytes = (size_t)8 << n;
    float* mats = (float*)ar.take(mats_bytes(*c, n, B));
    double* Frow = (double*)ar.take((size_t)rows_all * 8);
    if (!mats || !Frow) return ws_fail(ctx, ar, "qsv_reset_fidelity");
    int nblk = (int)((dim + 4095) / 4096);
    if (nblk > 1024) nblk = 1024;
    const size_t row_bytes = state_bytes + (size_t)nblk * 3 * 8 + 2 * kAlign;
    int64_t chunk = (int64_t)(ar.remaining() / row_bytes);
    if (chunk < 1) { ar.need = ar.off + row_bytes; return ws_fail(ctx, ar, "qsv_reset_fidelity"); }
    if (chunk > rows_all) chunk = rows_all;
    if (chunk > 32768) chunk = 32768;
    if (ctx->opt_grad_chunk > 0 && chunk > ctx->opt_grad_chunk) chunk = ctx->opt_grad_chunk;
    if (chunk < rows_all) { int64_t p2 = 1; while (p2 * 2 <= chunk) p2 *= 2; chunk = p2; }
    float2* work = (float2*)ar.take((size_t)chunk * state_bytes);
    double* partial = (double*)ar.take((size_t)chunk * nblk * 3 * 8);
    if (!work || !partial) return ws_fail(ctx, ar, "qsv_reset_fidelity");
    Prepared pr;
    st = prepare_circuit(ctx, *c, chunk, 1, 0, params_dev, feats_dev, B, mats, &pr);
    if (st != QSV_OK) return st;
    for (int64_t row0 = 0; row0 < rows_all; row0 += chunk) {
        const int64_t rows = (rows_all - row0) < chunk ? (rows_all - row0) : chunk;
        RowMap rm;
        rm.grad = 1; rm.two_p = 0; rm.per = (int)per; rm.row0 = row0;
        rm.slots_n = 1; rm.n = n;
        QSV_HIP(ctx, launch_reset_rows(ctx->state, n, mask, rows, rm, work, ctx->stream), "reset rows");
        st = run_circuit(ctx, *c, pr, work, rows, 1, nullptr, rm);
        if (st != QSV_OK) return st;
        QSV_HIP(ctx, launch_fidelity_block(work, rows, n, x_dev, dim, partial, nblk, rm, ctx->stream),
                "fidelity block");
        QSV_HIP(ctx, launch_fidelity_finish(partial, nblk, rows, nullptr, Frow + row0, ctx->stream),
                "fidelity finish");
    }
    QSV_HIP(ctx, launch_reset_sum(Frow, per, B, out_dev, ctx->stream), "reset sum");
    return QSV_OK;
}

qsv_status qsv_shot_expz(qsv_ctx* ctx, const long long* samples_dev, int64_t shots, float* out_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    if (!samples_dev || !out_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "samples_dev or out_dev is NULL");
    if (shots < 0) return fail(ctx, QSV_ERR_INVALID_ARG, "shots must be >= 0");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    QSV_HIP(ctx, launch_shot_expz(samples_dev, shots, ctx->batch, ctx->n, out_dev, ctx->stream), "shot expz");
    return QSV_OK;
}

qsv_status qsv_param_shift_grad(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                                const float* params_dev, const float* feats_dev, int32_t obs_qubit,
                                float* loss_dev, float* grad_dev, float* mean_loss_dev,
                                float* mean_grad_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    std::string why;
    if (!check_circuit(c, ctx->n, &why)) return fail(ctx, QSV_ERR_INVALID_ARG, why);
    const int n = ctx->n;
    const int64_t B = ctx->batch;
    if (!x_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "x_dev is NULL");
    if (dim < 1 || dim > ((int64_t)1 << n)) return fail(ctx, QSV_ERR_INVALID_ARG, "dim must be in 1..2^n");
    if (obs_qubit < 0 || obs_qubit >= n) return fail(ctx, QSV_ERR_INVALID_ARG, "obs_qubit out of range");
    const int64_t P = qsv_num_params(c, n);
    if (P > 0 && !params_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "params_dev is NULL");
    if (c->reupload && !feats_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "reupload = 1 needs feats_dev");
    if (!loss_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "loss_dev is NULL");
    if (P > 0 && !grad_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "grad_dev is NULL");
    if (2 * P + 1 > 0x3fffffff) return fail(ctx, QSV_ERR_UNSUPPORTED, "too many parameters");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;

    Arena ar(ctx);
    const CircDev cd = to_dev(*c, n);
    const int64_t per = 2 * P + 1;
    const int64_t circuits = B * per;
    const size_t msamples = (size_t)(c->reupload ? B : 1);
    const size_t state_bytes = (size_t)8 << n;
    int nblk = (int)((dim + 4095) / 4096);
    if (nblk > 1024) nblk = 1024;
    double* npart = (double*)ar.take((size_t)B * nblk * 8);
    double* inv = (double*)ar.take((size_t)B * 8);
    float* mats = (float*)ar.take(mats_bytes(*c, n, B));
    float* ovr = (float*)ar.take(msamples * (size_t)(2 * P) * 32);
    double* f = (double*)ar.take((size_t)circuits * 8);
    if (!npart || !inv || !mats || !ovr || !f) return ws_fail(ctx, ar, "qsv_param_shift_grad");
    QSV_HIP(ctx, launch_norms(x_dev, B, dim, npart, nblk, inv, nullptr, ctx->stream), "norms");

    // a chunk of circuit states plus their reduction partials, sized to what is left of the workspace
    const size_t row_bytes = state_bytes + (size_t)chunk_blocks(n) * 13 * 8 + 2 * kAlign;
    auto chunk_rows = [&](int64_t want) -> int64_t {
        int64_t chunk = (int64_t)(ar.remaining() / row_bytes);
        if (chunk > want) chunk = want;
        if (chunk > 32768) chunk = 32768;  // rows index a grid dimension
        if (ctx->opt_grad_chunk > 0 && chunk > ctx->opt_grad_chunk) chunk = ctx->opt_grad_chunk;
        // keep the row count a power of two when several rows share a tile (extended-index tiling)
        if (chunk >= 1 && chunk < want) { int64_t p2 = 1; while (p2 * 2 <= chunk) p2 *= 2; chunk = p2; }
        return chunk;
    };

    // ---- layer by layer: the circuits that shift a parameter of layer l share layers 0..l-1 with
    // the unshifted circuit, so its state before layer l is kept per sample and each shifted
    // circuit runs layers l..L-1 only.  Needs room for (L+1) states per sample; otherwise every
    // shifted circuit is run whole (below).
    const int L = c->n_layers;
    const int slots_n = (c->reupload + c->n_rot) * n;
    const size_t ckpt_bytes = (size_t)B * (size_t)(L + 1) * state_bytes;
    if (ctx->opt_grad_layered && P > 0 && ar.remaining() >= align_up(ckpt_bytes) + row_bytes + 2 * kAlign) {
        float2* ckpt = (float2*)ar.take(ckpt_bytes);
        const int64_t per_l = 2 * (int64_t)slots_n;          // shifted circuits per sample and layer
        const int64_t want = B * per_l > B ? B * per_l : B;
        const int64_t chunk = chunk_rows(want);
        float2* states = (float2*)ar.take((size_t)chunk * state_bytes);
        double* zpart = (double*)ar.take((size_t)(chunk > B ? chunk : B) * chunk_blocks(n) * 13 * 8);
        if (!ckpt || chunk < 1 || !states || !zpart) return ws_fail(ctx, ar, "qsv_param_shift_grad");
        const size_t sample_stride = (size_t)1 << n;          // amplitudes per state
        auto ck = [&](int l) { return ckpt + (size_t)l * (size_t)B * sample_stride; };
        qsv_circuit one = *c;
        one.n_layers = 1;
        // unshifted circuit, one layer at a time: ck(l) = state of every sample before layer l
        QSV_HIP(ctx, launch_encode_write(x_dev, dim, n, B, inv, plain_rows(n), ck(0), ctx->stream), "encode");
        RowMap rm_fwd;    // rows are the samples: the first pass of layer l reads state l and writes state l + 1
        rm_fwd.grad = 1; rm_fwd.two_p = 0; rm_fwd.per = 1; rm_fwd.row0 = 0;
        rm_fwd.slots_n = slots_n < 1 ? 1 : slots_n; rm_fwd.n = n;
        for (int l = 0; l < L; ++l) {
            Prepared pr;
            st = prepare_circuit(ctx, one, B, 0, 0, params_dev + (size_t)l * slots_n, feats_dev, B, mats, &pr);
            if (st != QSV_OK) return st;
            st = run_circuit(ctx, one, pr, ck(l + 1), B, 0, nullptr, rm_fwd, ck(l));
            if (st != QSV_OK) return st;
        }
        QSV_HIP(ctx, launch_expz_block(ck(L), B, n, zpart, ctx->stream), "expz block");
        QSV_HIP(ctx, launch_expz_finish_scatter(zpart, B, n, obs_qubit, f, Scatter{0, 1, per, 2 * P}, ctx->stream),
                "expz finish");
        // shifted circuits of layer l: start from ck(l), run layers l..L-1 with one matrix replaced
        const CircDev cd1 = to_dev(one, n);
        for (int l = 0; l < L; ++l) {
            qsv_circuit tail = *c;
            tail.n_layers = L - l;
            const float* p_l = params_dev + (size_t)l * slots_n;
            Prepared pr;
            st = prepare_circuit(ctx, tail, chunk, 0, 1, p_l, feats_dev, B, mats, &pr);
            if (st != QSV_OK) return st;
            QSV_HIP(ctx, launch_build_shifted(cd1, p_l, feats_dev, B, ovr, ctx->stream), "build shifted");
            const int64_t circuits_l = B * per_l;
            for (int64_t row0 = 0; row0 < circuits_l; row0 += chunk) {
                const int64_t rows = (circuits_l - row0) < chunk ? (circuits_l - row0) : chunk;
                RowMap rm;
                rm.grad = 1;
                rm.two_p = (int)per_l;
                rm.per = (int)per_l;
                rm.row0 = row0;
                rm.slots_n = slots_n;
                rm.n = n;
                const ZSpec zs{obs_qubit, f, Scatter{row0, per_l, per, (int64_t)l * per_l}, zpart};
                st = run_circuit(ctx, tail, pr, states, rows, 0, ovr, rm, ck(l), &zs);
                if (st != QSV_OK) return st;
            }
        }
        QSV_HIP(ctx, launch_grad_finish(f, B, P, cd, feats_dev, loss_dev, grad_dev, mean_loss_dev,
                                        mean_grad_dev, ctx->stream),
                "grad finish");
        return QSV_OK;
    }

    // ---- every shifted circuit whole
    const int64_t chunk = chunk_rows(circuits);
    if (chunk < 1) { ar.need = ar.off + row_bytes; return ws_fail(ctx, ar, "qsv_param_shift_grad"); }
    float2* states = (float2*)ar.take((size_t)chunk * state_bytes);
    double* zpart = (double*)ar.take((size_t)chunk * chunk_blocks(n) * 13 * 8);
    if (!states || !zpart) return ws_fail(ctx, ar, "qsv_param_shift_grad");
    Prepared pr;
    st = prepare_circuit(ctx, *c, chunk, 0, 1, params_dev, feats_dev, B, mats, &pr);
    if (st != QSV_OK) return st;
    if (P > 0)
        QSV_HIP(ctx, launch_build_shifted(cd, params_dev, feats_dev, B, ovr, ctx->stream), "build shifted");
    for (int64_t row0 = 0; row0 < circuits; row0 += chunk) {
        const int64_t rows = (circuits - row0) < chunk ? (circuits - row0) : chunk;
        RowMap rm;
        rm.grad = 1;
        rm.two_p = (int)(2 * P);
        rm.per = (int)per;
        rm.row0 = row0;
        rm.slots_n = slots_n < 1 ? 1 : slots_n;
        rm.n = n;
        QSV_HIP(ctx, launch_encode_write(x_dev, dim, n, rows, inv, rm, states, ctx->stream), "encode rows");
        const ZSpec zs{obs_qubit, f, Scatter{row0, 1, 1, 0}, zpart};
        st = run_circuit(ctx, *c, pr, states, rows, 0, ovr, rm, nullptr, &zs);
        if (st != QSV_OK) return st;
    }
    QSV_HIP(ctx, launch_grad_finish(f, B, P, cd, feats_dev, loss_dev, grad_dev, mean_loss_dev,
                                    mean_grad_dev, ctx->stream),
            "grad finish");
    return QSV_OK;
}

// Reverse-mode loss and gradient for a diagonal observable: kind 0 <Z_q>; 1 the loss 1 - P0(mask);
// 2 the mean squared error of <Z_q> against targets [batch][n].
static qsv_status adjoint_impl(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                               const float* params_dev, const float* feats_dev, int kind, int32_t obs_qubit,
                               uint64_t mask, const float* targets_dev, float* loss_dev, float* grad_dev,
                               float* mean_loss_dev, float* mean_grad_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    std::string why;
    if (!check_circuit(c, ctx->n, &why)) return fail(ctx, QSV_ERR_INVALID_ARG, why);
    const int n = ctx->n;
    const int64_t B = ctx->batch;
    if (!x_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "x_dev is NULL");
    if (dim < 1 || dim > ((int64_t)1 << n)) return fail(ctx, QSV_ERR_INVALID_ARG, "dim must be in 1..2^n");
    if (kind == 0 && (obs_qubit < 0 || obs_qubit >= n)) return fail(ctx, QSV_ERR_INVALID_ARG, "obs_qubit out of range");
    if (kind == 1 && (mask == 0 || (mask >> n) != 0))
        return fail(ctx, QSV_ERR_INVALID_ARG, "mask must name at least one qubit and none beyond n_qubits");
    if (kind == 2 && !targets_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "targets_dev is NULL");
    const int64_t P = qsv_num_params(c, n);
    if (P > 0 && !params_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "params_dev is NULL");
    if (c->reupload && !feats_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "reupload = 1 needs feats_dev");
    if (!loss_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "loss_dev is NULL");
    if (P > 0 && !grad_dev) return fail(ctx, QSV_ERR_INVALID_ARG, "grad_dev is NULL");
    if (2 * P + 1 > 0x3fffffff) return fail(ctx, QSV_ERR_UNSUPPORTED, "too many parameters");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;

    Arena ar(ctx);
    const CircDev cd = to_dev(*c, n);
    const int64_t per = 2 * P + 1;
    const size_t state_bytes = (size_t)8 << n;
    int nblk = (int)((dim + 4095) / 4096);
    if (nblk > 1024) nblk = 1024;
    double* npart = (double*)ar.take((size_t)B * nblk * 8);
    double* inv = (double*)ar.take((size_t)B * 8);
    double* f = (double*)ar.take((size_t)B * per * 8);
    if (!npart || !inv || !f) return ws_fail(ctx, ar, "qsv_adjoint_grad");
    QSV_HIP(ctx, launch_norms(x_dev, B, dim, npart, nblk, inv, nullptr, ctx->stream), "norms");

    // Two ways to have psi at the start of every layer on the way back.  With room for L + 1 states per
    // sample the forward run keeps them (layer l reads state l and writes state l + 1, no copies) and
    // only lambda is taken back: 2 L layers of gates per sample.  Otherwise psi is taken back together
    // with lambda (rows 2r, 2r+1 of one buffer): 3 L layers, 3 states per sample of a chunk.
    const int L = c->n_layers;
    const size_t tpart = (size_t)n * (adj_trans_blocks(n) + 1) * 8 * 8;
    const size_t zbytes = (size_t)chunk_blocks(n) * 13 * 8;
    const size_t small_bytes = tpart + zbytes + 2 * (size_t)n * 8 + 6 * kAlign;
    const size_t ckpt_bytes = (size_t)B * (size_t)(L + 1) * state_bytes;
    const size_t tables = mats_bytes(*c, n, B);
    const bool keep = ctx->opt_grad_layered && P > 0 &&
                      ar.remaining() >= align_up(ckpt_bytes) + state_bytes + small_bytes + 2 * tables + 2 * kAlign;
    float2* ckpt = keep ? (float2*)ar.take(ckpt_bytes) : nullptr;
    if (keep && !ckpt) return ws_fail(ctx, ar, "qsv_adjoint_grad");
    // The samples go through the sweep in chunks; with two samples or more the chunks alternate
    // between the caller's stream and the context's second one, each with scratch of its own, so that
    // the launch gaps and tails of one chunk's kernels are covered by the other's.
    const size_t sample_bytes = (keep ? 1 : 3) * state_bytes + small_bytes;
    const bool two = B >= 2 && ctx->opt_split != 0 && !ctx->forked &&
                     ar.remaining() >= 2 * (sample_bytes + tables + kAlign);
    const int sets = two ? 2 : 1;
    const size_t fixed = (size_t)sets * (tables + kAlign);
    int64_t chunk = ar.remaining() > fixed ? (int64_t)((ar.remaining() - fixed) / (sets * sample_bytes)) : 0;
    if (chunk < 1) {
        ar.need = ar.off + fixed + sets * sample_bytes;
        return ws_fail(ctx, ar, "qsv_adjoint_grad");
    }
    if (two && chunk > (B + 1) / 2) chunk = (B + 1) / 2;
    if (chunk > B) chunk = B;
    if (chunk > 16384) chunk = 16384;   // rows of a chunk index a grid dimension
    if (ctx->opt_grad_chunk > 0 && chunk > ctx->opt_grad_chunk) chunk = ctx->opt_grad_chunk;
    // keep row counts a power of two when several rows share a tile (extended-index tiling)
    if (chunk < B) { int64_t p2 = 1; while (p2 * 2 <= chunk) p2 *= 2; chunk = p2; }
    struct Scratch { float* mats; float2 *Abuf, *S; double *tp, *zpart, *zall, *coef; } scr[2];
    for (int i = 0; i < sets; ++i) {
        Scratch& sc = scr[i];
        sc.mats = (float*)ar.take(tables);
        sc.Abuf = keep ? nullptr : (float2*)ar.take((size_t)chunk * state_bytes);
        sc.S = (float2*)ar.take((size_t)(keep ? 1 : 2) * chunk * state_bytes);
        sc.tp = (double*)ar.take((size_t)chunk * tpart);
        sc.zpart = (double*)ar.take((size_t)chunk * zbytes);
        sc.zall = (double*)ar.take((size_t)chunk * n * 8);
        sc.coef = (double*)ar.take((size_t)chunk * n * 8);
        if (!sc.mats || (!keep && !sc.Abuf) || !sc.S || !sc.tp || !sc.zpart || !sc.zall || !sc.coef)
            return ws_fail(ctx, ar, "qsv_adjoint_grad");
    }

    const int slots_n = (c->reupload + c->n_rot) * n;
    const size_t amps = (size_t)1 << n;
    auto ck = [&](int l, int64_t b0) { return ckpt + ((size_t)l * (size_t)B + (size_t)b0) * amps; };
    qsv_circuit one = *c;
    one.n_layers = 1;
    // one chunk of samples b0 .. b0 + bc - 1 on ctx->stream, with the scratch set sc
    auto run_chunk = [&](int64_t b0, int64_t bc, const Scratch& sc) -> qsv_status {
        // forward: rows are samples b0..b0+bc-1
        RowMap rm1;
        rm1.grad = 1; rm1.two_p = 0; rm1.per = 1; rm1.row0 = b0; rm1.slots_n = slots_n < 1 ? 1 : slots_n; rm1.n = n;
        float2* A = keep ? ck(L, b0) : sc.Abuf;                 // the final states of the chunk
        if (keep) {
            QSV_HIP(ctx, launch_encode_write(x_dev, dim, n, bc, inv, rm1, ck(0, b0), ctx->stream), "encode rows");
            Prepared all;
            st = prepare_layers(ctx, *c, one, bc, 0, params_dev, feats_dev, B, sc.mats, &all);
            if (st != QSV_OK) return st;
            for (int l = 0; l < L; ++l) {
                // the start states are addressed by sample (ck(l, 0)), the rows written are the chunk's
                st = run_circuit(ctx, one, layer_of(all, l, n), ck(l + 1, b0), bc, 0, nullptr, rm1, ck(l, 0));
                if (st != QSV_OK) return st;
            }
        } else {
            QSV_HIP(ctx, launch_encode_write(x_dev, dim, n, bc, inv, rm1, A, ctx->stream), "encode rows");
            Prepared pr;
            st = prepare_circuit(ctx, *c, bc, 0, 0, params_dev, feats_dev, B, sc.mats, &pr);
            if (st != QSV_OK) return st;
            st = run_circuit(ctx, *c, pr, A, bc, 0, nullptr, rm1);
            if (st != QSV_OK) return st;
        }
        // the loss of every sample of the chunk into f[sample][2P]
        if (kind == 0) {
            QSV_HIP(ctx, launch_expz_block(A, bc, n, sc.zpart, ctx->stream), "expz block");
            QSV_HIP(ctx, launch_expz_finish_scatter(sc.zpart, bc, n, obs_qubit, f, Scatter{b0, 1, per, 2 * P},
                                                    ctx->stream),
                    "expz finish");
        } else if (kind == 1) {
            QSV_HIP(ctx, launch_trash_loss(A, n, mask, bc, b0, P, sc.zpart, f, ctx->stream), "trash loss");
        } else {
            QSV_HIP(ctx, launch_expz_block(A, bc, n, sc.zpart, ctx->stream), "expz block");
            QSV_HIP(ctx, launch_expz_finish(sc.zpart, bc, n, -1, nullptr, sc.zall, ctx->stream), "expz finish");
            QSV_HIP(ctx, launch_mse_coef(sc.zall, targets_dev, n, bc, b0, P, sc.coef, f, ctx->stream), "mse loss");
        }
        if (P == 0) return QSV_OK;
        // backward: lambda = O psi (and psi beside it unless its states were kept), taken back layer by layer
        QSV_HIP(ctx, launch_adj_init(A, n, kind, obs_qubit, mask, sc.coef, bc, sc.S, keep ? 0 : 1, ctx->stream),
                "adjoint init");
        RowMap rm2 = rm1;
        if (!keep) {
            rm2.per = 2;
            rm2.row0 = 2 * b0;
        }
        const int64_t back_rows = keep ? bc : 2 * bc;
        Prepared back;      // all layers' inverse matrices by one launch
        st = prepare_layers(ctx, *c, one, back_rows, 1, params_dev, feats_dev, B, sc.mats, &back);
        if (st != QSV_OK) return st;
        for (int l = L - 1; l >= 0; --l) {
            st = run_circuit(ctx, one, layer_of(back, l, n), sc.S, back_rows, 1, nullptr, rm2);
            if (st != QSV_OK) return st;
            const float2* psi0 = keep ? ck(l, b0) : sc.S;
            const float2* lam0 = keep ? sc.S : sc.S + amps;
            QSV_HIP(ctx, launch_adj_layer(psi0, lam0, keep ? 1 : 2, n, bc, sc.tp, cd, l, params_dev, feats_dev, b0, P, f,
                                          ctx->stream),
                    "adjoint layer");
        }
        return QSV_OK;
    };
    // chunk i runs on stream i % 2 with scratch set i % 2 (stream order guards the reuse of a set)
    struct Fork {
        qsv_ctx* c; hipStream_t main; bool on;
        ~Fork() {
            c->stream = main;
            if (!on) return;
            c->forked = false;
            if (hipEventRecord(c->ev_join, c->side) == hipSuccess) (void)hipStreamWaitEvent(main, c->ev_join, 0);
        }
    } fork{ctx, ctx->stream, false};
    if (two && chunk < B) {
        // Plans are uploaded on the stream that first asks for them: have the ones the chunks will use
        // in place before the second stream branches off (three calls: should the second one recycle
        // the plan buffer, the third brings the first plan back).
        if (!(ctx->opt_naive || n < kRegBits)) {
            const CachedPlan* warm = nullptr;
            for (int k = 0; k < 3; ++k) {
                const bool inv_plan = (k == 1);
                if (inv_plan && P == 0) continue;
                st = get_plan(ctx, (inv_plan || keep) ? one : *c, chunk, inv_plan ? 1 : 0, 0, &warm);
                if (st != QSV_OK) return st;
            }
        }
        QSV_HIP(ctx, hipEventRecord(ctx->ev_fork, ctx->stream), "fork");
        QSV_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0), "fork");
        fork.on = true;
        ctx->forked = true;
    }
    int64_t ci = 0;
    for (int64_t b0 = 0; b0 < B; b0 += chunk, ++ci) {
        const int64_t bc = (B - b0) < chunk ? (B - b0) : chunk;
        const int set = fork.on ? (int)(ci & 1) : 0;
        ctx->stream = set ? ctx->side : fork.main;
        st = run_chunk(b0, bc, scr[set]);
        if (st != QSV_OK) return st;
    }
    ctx->stream = fork.main;
    if (fork.on) {        // the finishing kernel sees both streams' work
        fork.on = false;
        ctx->forked = false;
        QSV_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->side), "join");
        QSV_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0), "join");
    }
    QSV_HIP(ctx, launch_grad_finish(f, B, P, cd, feats_dev, loss_dev, grad_dev, mean_loss_dev,
                                    mean_grad_dev, ctx->stream),
            "grad finish");
    return QSV_OK;
}

qsv_status qsv_adjoint_grad(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                            const float* params_dev, const float* feats_dev, int32_t obs_qubit,
                            float* loss_dev, float* grad_dev, float* mean_loss_dev, float* mean_grad_dev) {
    return adjoint_impl(ctx, c, x_dev, dim, params_dev, feats_dev, 0, obs_qubit, 0, nullptr, loss_dev,
                        grad_dev, mean_loss_dev, mean_grad_dev);
}

qsv_status qsv_loss_grad(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                         const float* params_dev, const float* feats_dev, const qsv_loss* loss,
                         float* loss_dev, float* grad_dev, float* mean_loss_dev, float* mean_grad_dev) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    if (!loss) return fail(ctx, QSV_ERR_INVALID_ARG, "loss is NULL");
    if (loss->kind != QSV_LOSS_TRASH && loss->kind != QSV_LOSS_MSE_Z)
        return fail(ctx, QSV_ERR_INVALID_ARG, "unknown loss kind");
    return adjoint_impl(ctx, c, x_dev, dim, params_dev, feats_dev, loss->kind == QSV_LOSS_TRASH ? 1 : 2, 0,
                        loss->mask, loss->targets_dev, loss_dev, grad_dev, mean_loss_dev, mean_grad_dev);
}

qsv_status qsv_sgd_step(qsv_ctx* ctx, float* params_dev, const float* grad_dev, int64_t count, double lr) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    if (count < 0 || (count > 0 && (!params_dev || !grad_dev)))
        return fail(ctx, QSV_ERR_INVALID_ARG, "qsv_sgd_step: bad arguments");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    QSV_HIP(ctx, launch_sgd(params_dev, grad_dev, count, lr, ctx->stream), "sgd step");
    return QSV_OK;
}

qsv_status qsv_adam_step(qsv_ctx* ctx, float* params_dev, const float* grad_dev, float* m_dev, float* v_dev,
                         int64_t count, int64_t t, double lr, double beta1, double beta2, double eps) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    if (count < 0 || t < 1 || (count > 0 && (!params_dev || !grad_dev || !m_dev || !v_dev)) ||
        !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) || !(eps > 0.0))
        return fail(ctx, QSV_ERR_INVALID_ARG, "qsv_adam_step: bad arguments");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    QSV_HIP(ctx, launch_adam(params_dev, grad_dev, m_dev, v_dev, count, t, lr, beta1, beta2, eps, ctx->stream),
            "adam step");
    return QSV_OK;
}

qsv_status qsv_probe_pass(qsv_ctx* ctx, int low_bits, int window_start, int transposes) {
    if (!ctx) return QSV_ERR_INVALID_ARG;
    const int n = ctx->n;
    if (n < kRegBits) return fail(ctx, QSV_ERR_UNSUPPORTED, "probe needs n_qubits >= 4");
    const int tile = ctx->opt_tile ? ctx->opt_tile : default_tile(n, ctx->batch);
    const int ext = n + ceil_log2_i64(ctx->batch);
    if (low_bits < kLowBits || low_bits > tile || window_start < low_bits ||
        (ext > tile && window_start + (tile - low_bits) > ext) || (ext <= tile && window_start != low_bits))
        return fail(ctx, QSV_ERR_INVALID_ARG, "probe geometry does not fit the state");
    if (transposes < 0 || transposes > 16) return fail(ctx, QSV_ERR_INVALID_ARG, "transposes must be in 0..16");
    qsv_status st = bind_device(ctx);
    if (st != QSV_OK) return st;
    Arena ar(ctx);
    Op* dev = (Op*)ar.take(32 * sizeof(Op));
    if (!dev) return ws_fail(ctx, ar, "qsv_probe_pass");
    std::vector<Op> ops;
    const int smax = tile - kRegBits;
    const int sio = ctx->opt_probe_layout >= 0 ? std::min(ctx->opt_probe_layout, smax) : smax;
    ops.push_back({OP_LOAD, (uint8_t)sio, 0, 0, 0});
    for (int i = 0; i < transposes; ++i)
        ops.push_back({OP_XPOSE, (uint8_t)((i & 1) ? sio : (sio ? 0 : smax)), 0, 0, 0});
    ops.push_back({OP_END, 0, 0, 0, 0});
    set_transpose_barriers(ops);
    // a small synchronous upload: this is a measurement aid, not part of the hot path
    QSV_HIP(ctx, hipMemcpyAsync(dev, ops.data(), ops.size() * sizeof(Op), hipMemcpyHostToDevice, ctx->stream),
            "upload probe");
    QSV_HIP(ctx, hipStreamSynchronize(ctx->stream), "upload probe");
    PassArgs a;
    a.state = ctx->state;
    a.in = ctx->state;
    a.imap = nullptr;
    a.src = nullptr;
    a.zout = nullptr; a.zq = 0; a.nostore = 0;
    a.nt_store = ctx->opt_nt_store >= 0 ? ctx->opt_nt_store : ((((uint64_t)ctx->batch << n) * 8) >= kNtStoreBytes ? 1 : 0);
    a.rev = (ctx->opt_rev >= 0 ? ctx->opt_rev : ((((uint64_t)ctx->batch << n) * 8) >= kNtStoreBytes ? 1 : 0))
                ? (ctx->probe_count++ & 1) : 0;
    a.ops = dev;
    a.mats = nullptr;
    a.exec_of = nullptr;
    a.ovr = nullptr;
    a.total = (uint64_t)ctx->batch << n;
    a.prio = ctx->opt_prio;
    a.n = n; a.c = low_bits; a.w = window_start;
    a.n_mats = 0;
    a.rowdep = 0;
    a.rm = plain_rows(n);
    const uint64_t n_tiles = ext > tile ? (1ull << (ext - tile)) : 1ull;
    QSV_HIP(ctx, launch_pass(tile, ctx->opt_planes, a, n_tiles, ctx->stream), "probe pass");
    return QSV_OK;
}

}  // extern "C"
