// Pass planner (host only, no HIP).  See qsv_plan.h for the execution model.
//
// The circuit is first lowered to "fused-level" gates: per layer one 2x2 unitary U(l,q) per qubit
// (the product of that qubit's re-upload and rotation-slot matrices, which commute with the other
// qubits' rotations), followed by the entangler's CNOTs or CZ rungs in program order.  A greedy
// list scheduler then packs those gates into passes and, inside a pass, into register rounds.
// A gate may be moved ahead of earlier, not-yet-executed gates only if it shares no qubit with
// them (disjoint gates commute); diagonal CZ rungs may additionally pass each other.
#include "qsv_plan.h"

#include <algorithm>
#include <cstdio>
#include <cstring>

namespace qsv {

namespace {

enum GateKind : uint8_t { G_U = 0, G_CNOT = 1, G_CZ = 2 };

struct Gate {
    uint8_t kind;
    int8_t q0;   // U: qubit; CNOT: target; CZ: lower qubit of the rung
    int8_t q1;   // CNOT: control; CZ: q0 + 1
    int32_t mat; // U: matrix id l*n + q
};

struct Geom {
    int t, c, w;
    bool local(int q) const { return q < c || (q >= w && q < w + t - c); }
    int pos(int q) const { return q < c ? q : q - w + c; }
};

// CNOTs form the sequential chain that decides how many passes a ring circuit needs, so chain
// progress outweighs rotations that merely run early.
// With deferred CNOTs the chain is cheap to advance and the unitaries of a window's qubits are what a
// pass is short of, so the weights are level there.
struct Weights { int u, cx, cz; };
constexpr Weights kClassicWeights{2, 16, 1}, kDeferWeights{8, 8, 1};
// The geometry of a pass is chosen by what it and the best pass after it complete together; the
// second level is only tried for the kLookTop best first passes.
constexpr int kLookTop = 6;
constexpr size_t kScanLimit = 8192;
constexpr int kMinRoundGates = 2;

std::vector<Gate> lower(const qsv_circuit& c, int n, bool inverse) {
    std::vector<Gate> g;
    const bool has_u = (c.reupload + c.n_rot) > 0;
    auto layer_u = [&](int l) {
        if (!has_u) return;
        for (int q = 0; q < n; ++q) g.push_back({G_U, (int8_t)q, (int8_t)-1, l * n + q});
    };
    if (!inverse) {
        for (int l = 0; l < c.n_layers; ++l) {
            layer_u(l);
            if (c.entangler == QSV_ENT_CNOT_RING && n >= 2)
                for (int q = 0; q < n; ++q)
                    g.push_back({G_CNOT, (int8_t)((q + 1) % n), (int8_t)q, -1});
            if (c.entangler == QSV_ENT_CZ_LADDER)
                for (int q = 0; q + 1 < n; ++q) g.push_back({G_CZ, (int8_t)q, (int8_t)(q + 1), -1});
        }
    } else {
        for (int l = c.n_layers - 1; l >= 0; --l) {
            if (c.entangler == QSV_ENT_CNOT_RING && n >= 2)
                for (int q = n - 1; q >= 0; --q)
                    g.push_back({G_CNOT, (int8_t)((q + 1) % n), (int8_t)q, -1});
            if (c.entangler == QSV_ENT_CZ_LADDER)
                for (int q = n - 2; q >= 0; --q) g.push_back({G_CZ, (int8_t)q, (int8_t)(q + 1), -1});
            layer_u(l);  // the matrix table holds U(l,q)^dagger in inverse mode
        }
    }
    return g;
}

// Deferred CNOTs.  A CNOT is a permutation of basis states, so one whose target qubit is not local to
// the pass need not be a register operation: the pass can instead write every amplitude to the index
// the CNOT sends it to (another tile: such passes read one buffer and write another).  While a pass
// runs, v[q] is the set of index bits whose parity gives the logical value of qubit q for the
// amplitude at a given position (position = the tile's fixed index bits and the amplitude's current
// place inside the tile); v[q] = {q} until a deferred CNOT with target q folds its control's set in.
// Consequences, all enforced below: a unitary on a local qubit needs that qubit in no other set
// (its two amplitudes must agree in every other logical bit); a CNOT with a local target whose
// control has a set of several bits becomes a swap under the parity of those bits, none of which may
// sit in the register run; a register CNOT on a bit that other sets contain folds the control's set
// into them (the amplitude moves, its logical bits do not); and no set of a non-local qubit may hold
// one of the three lowest index bits, so that runs of 64 bytes are still written as a whole.
struct VState {
    uint32_t v[32];
    uint32_t taint = 0;   // bits that occur in the set of another qubit
    bool any = false;     // some set differs from {q}
    void reset(int n) {
        for (int q = 0; q < 32; ++q) v[q] = q < n ? (1u << q) : 0u;
        taint = 0;
        any = false;
    }
    void retaint(int n) {
        taint = 0;
        any = false;
        for (int q = 0; q < n; ++q) {
            taint |= v[q] & ~(1u << q);
            any = any || v[q] != (1u << q);
        }
    }
};

enum ExecForm : uint8_t { F_PLAIN = 0, F_PARITY = 1, F_DEFER = 2, F_LANE = 3 };
struct Exec {
    int gate;
    uint8_t form;
    uint32_t mask;   // F_PARITY, F_DEFER: the control's set when the gate ran
};

// Index bits that never enter the set of a non-local qubit: the three lowest, so that a deferred CNOT
// moves runs of 8 amplitudes (64 bytes, what one request to the memory side carries) and never less.
// Measured on the 26-qubit configuration: with whole 128-byte lines (four bits) 54 passes, 13.07 ms;
// with 64-byte runs 50 passes, 12.65 ms; fewer bits give no fewer passes.
constexpr uint32_t kLowMask = (1u << 3) - 1u;

// One register round: which pending gates can run with the run at tile position s.
// Appends them to exec (program order) and returns the score; *n_real receives the number of gates
// that need the tile in this layout (everything but deferred CNOTs).  vs is updated as gates run.
// Does not modify done.
int scan_round(const Geom& gm, int s, int n, const std::vector<Gate>& G,
               const std::vector<uint8_t>& done, size_t first, bool defer, VState& vs,
               std::vector<Exec>* exec, int* n_real) {
    uint64_t blk_any = 0, blk_diag = 0;
    const uint64_t all = n >= 64 ? ~0ull : ((1ull << n) - 1);
    int score = 0, real = 0;
    const size_t end = std::min(G.size(), first + kScanLimit);
    auto in_run = [&](int q) {
        if (!gm.local(q)) return false;
        const int p = gm.pos(q);
        return p >= s && p < s + kRegBits;
    };
    uint32_t run_mask = 0;    // the qubits behind the register run
    for (int q = 0; q < n; ++q)
        if (in_run(q)) run_mask |= 1u << q;
    for (size_t i = first; i < end; ++i) {
        if (done[i]) continue;
        const Gate& g = G[i];
        uint64_t m = 1ull << g.q0;
        if (g.kind != G_U) m |= 1ull << g.q1;
        bool can;
        Exec ex{(int)i, F_PLAIN, 0};
        if (g.kind == G_CZ) {
            can = !(blk_any & m);
        } else if (g.kind == G_U) {
            can = !((blk_any | blk_diag) & m) && in_run(g.q0) && !((vs.taint >> g.q0) & 1u);
        } else {
            const int t = g.q0, c = g.q1;
            const uint32_t cm = vs.v[c];
            can = !((blk_any | blk_diag) & m) && !((cm >> t) & 1u);
            // control in the register run, target one of the lane's own index bits: the amplitudes with
            // the control set trade places with those of the partner lane (a cross-lane exchange, no
            // transpose); lane_bit >= 0 is the bit of the lane number behind the target
            int lane_bit = -1;
            if (can && gm.local(t) && !in_run(t) && in_run(c) && cm == (1u << c)) {
                const int pp = gm.pos(t);
                const int b = pp < s ? pp : pp - kRegBits;     // bit of the thread index
                if (b < 6) lane_bit = b;
            }
            if (lane_bit >= 0) {
                const bool others_hold_t = (vs.taint >> t) & 1u;
                if (others_hold_t && (cm & kLowMask)) can = false;
                if (can && others_hold_t) {
                    for (int q = 0; q < n; ++q)
                        if (q != t && ((vs.v[q] >> t) & 1u)) vs.v[q] ^= cm;
                    vs.retaint(n);
                }
                ex.form = F_LANE;
                ex.mask = (uint32_t)lane_bit;
            } else if (can && gm.local(t)) {
                can = in_run(t);
                if (can && cm != (1u << c)) {
                    can = !(cm & run_mask);
                    ex.form = F_PARITY;
                    ex.mask = cm;
                }
                const bool others_hold_t = (vs.taint >> t) & 1u;
                if (can && others_hold_t && (cm & kLowMask)) can = false;
                if (can && others_hold_t) {
                    for (int q = 0; q < n; ++q)
                        if (q != t && ((vs.v[q] >> t) & 1u)) vs.v[q] ^= cm;
                    vs.retaint(n);
                }
            } else if (can) {
                can = defer && !(cm & kLowMask);
                if (can) {
                    ex.form = F_DEFER;
                    ex.mask = cm;
                    vs.v[t] ^= cm;
                    vs.retaint(n);
                }
            }
        }
        if (can) {
            if (exec) exec->push_back(ex);
            const Weights& wt = defer ? kDeferWeights : kClassicWeights;
            score += g.kind == G_U ? wt.u : g.kind == G_CNOT ? wt.cx : wt.cz;
            if (ex.form != F_DEFER) ++real;
        } else {
            if (g.kind == G_CZ) blk_diag |= m; else blk_any |= m;
            if (blk_any == all) break;
        }
    }
    if (n_real) *n_real = real;
    return score;
}

void mark_transposes(std::vector<Op>& ops, size_t begin);

void emit_round(const Geom& gm, int s, const std::vector<Gate>& G, const std::vector<Exec>& exec,
                bool rowdep, std::vector<Op>* ops, std::vector<int32_t>* mat_order, std::vector<Op>* defers) {
    bool last_lane = false;
    auto in_run = [&](int q) {
        if (!gm.local(q)) return false;
        const int p = gm.pos(q);
        return p >= s && p < s + kRegBits;
    };
    for (const Exec& ex : exec) {
        const Gate& g = G[ex.gate];
        if (g.kind == G_CZ) {
            // rungs commute, so each goes to the cheapest form for where its two qubits sit
            const bool r0 = in_run(g.q0), r1 = in_run(g.q1);
            if (r0 && r1) {
                const int ja = gm.pos(g.q0) - s, jb = gm.pos(g.q1) - s;
                ops->push_back({OP_CZ_REG, (uint8_t)std::min(ja, jb), (uint8_t)std::max(ja, jb), 0, 0});
                last_lane = false;
            } else if (r0 || r1) {
                const int qr = r0 ? g.q0 : g.q1, qo = r0 ? g.q1 : g.q0;
                ops->push_back({OP_CZ_MIX, (uint8_t)(gm.pos(qr) - s), (uint8_t)qo, 0, 0});
                last_lane = false;
            } else if (last_lane) {
                ops->back().arg |= (int32_t)(1u << g.q0);
            } else {
                ops->push_back({OP_CZ_LANE, 0, 0, 0, (int32_t)(1u << g.q0)});
                last_lane = true;
            }
            continue;
        }
        last_lane = false;
        if (ex.form == F_DEFER) {
            // nothing happens in registers: the pass's index map carries it.  Kept beside the operation
            // list (a = target, b = control qubit, arg = the control's set) for the plan's description.
            if (defers) defers->push_back({OP_CX_DEFER, (uint8_t)g.q0, (uint8_t)g.q1, 0, (int32_t)ex.mask});
            continue;
        }
        if (ex.form == F_LANE) {
            ops->push_back({OP_CX_LANE, (uint8_t)(gm.pos(g.q1) - s), (uint8_t)ex.mask, (uint8_t)g.q0, 0});
            continue;
        }
        const int jt = gm.pos(g.q0) - s;
        if (g.kind == G_U) {
            ops->push_back({OP_U, (uint8_t)jt, (uint8_t)(rowdep ? 1 : 0), 0, (int32_t)mat_order->size()});
            mat_order->push_back(g.mat);
            continue;
        }
        if (ex.form == F_PARITY) {
            ops->push_back({OP_CX_PAR, (uint8_t)jt, (uint8_t)g.q1, 0, (int32_t)ex.mask});
            continue;
        }
        const int qc = g.q1;
        if (gm.local(qc)) {
            const int pc = gm.pos(qc);
            if (pc >= s && pc < s + kRegBits) {
                ops->push_back({OP_CX_REG, (uint8_t)jt, (uint8_t)(pc - s), 0, 0});
            } else {
                const int tbit = pc < s ? pc : pc - kRegBits;  // bit of the thread index
                ops->push_back({OP_CX_DYN, (uint8_t)jt, (uint8_t)qc, (uint8_t)(tbit >= 6 ? 1 : 0), 0});
            }
        } else {
            ops->push_back({OP_CX_DYN, (uint8_t)jt, (uint8_t)qc, 1, 0});
        }
    }
}

// Greedy rounds of one pass.  Marks executed gates in done; emits ops when ops != nullptr.
// Returns the pass score; *n_exec receives the number of gates executed; *vs_out the qubit sets at the
// end of the pass (from which the caller derives the pass's index map).
int run_pass(const Geom& gm, int n, const std::vector<Gate>& G, std::vector<uint8_t>& done,
             size_t first, bool rowdep, bool defer, std::vector<Op>* ops, std::vector<int32_t>* mat_order,
             std::vector<Op>* defers, int* n_exec, VState* vs_out) {
    const int smax = gm.t - kRegBits;
    const int smin_io = std::min(kLowBits, smax);  // layouts with coalesced global access
    // When one tile holds several state rows and matrices differ per row, a lane's 16 amplitudes
    // must share a row: gate rounds keep the run inside the qubit bits.
    const int sgate = (rowdep && n < gm.t) ? std::min(smax, n - kRegBits) : smax;
    int total = 0, cnt = 0;
    VState vs;
    vs.reset(n);
    std::vector<Exec> exec, best_exec;
    auto commit = [&](int s, const std::vector<Exec>& ex) {
        for (const Exec& e : ex) done[e.gate] = 1;
        cnt += (int)ex.size();
        if (ops) emit_round(gm, s, G, ex, rowdep, ops, mat_order, defers);
        while (first < G.size() && done[first]) ++first;
    };
    // first round: loaded straight from global memory
    int s = smax, best = 0;
    VState best_vs = vs;
    best_exec.clear();
    for (int cand = smin_io; cand <= sgate; ++cand) {
        exec.clear();
        VState tv = vs;
        const int sc = scan_round(gm, cand, n, G, done, first, defer, tv, &exec, nullptr);
        if (sc > best) { best = sc; s = cand; best_exec = exec; best_vs = tv; }
    }
    if (ops) ops->push_back({OP_LOAD, (uint8_t)s, 0, 0, 0});
    total += best;
    vs = best_vs;
    commit(s, best_exec);
    for (;;) {
        if (first >= G.size()) break;
        int bs = -1, best_real = 0;
        best = 0;
        for (int cand = 0; cand <= sgate; ++cand) {
            if (cand == s) continue;
            exec.clear();
            VState tv = vs;
            int real = 0;
            const int sc = scan_round(gm, cand, n, G, done, first, defer, tv, &exec, &real);
            // ties go to the later (higher) layout, which also stores coalesced
            if (sc > best || (sc == best && sc > 0 && cand >= smin_io)) {
                best = sc; bs = cand; best_exec = exec; best_vs = tv; best_real = real;
            }
        }
        if (bs < 0 || best == 0) break;
        if (best_real == 0) {
            // only deferred CNOTs: they need no layout, so no transpose either
            total += best;
            vs = best_vs;
            commit(s, best_exec);
            continue;
        }
        const bool critical = !best_exec.empty() && (size_t)best_exec.front().gate == first;
        if (!critical && best_real < kMinRoundGates) {
            // A transpose for one stray gate is not worth it, unless going on like this finishes
            // the whole circuit inside this pass (then it saves a pass over the state).
            std::vector<uint8_t> tmp(done);
            size_t f2 = first;
            int s2 = s;
            VState v2 = vs;
            for (;;) {
                int b2 = 0, bs2 = -1;
                std::vector<Exec> ex2, bex2;
                VState bv2 = v2;
                for (int cand = 0; cand <= sgate; ++cand) {
                    if (cand == s2) continue;
                    ex2.clear();
                    VState tv = v2;
                    const int sc = scan_round(gm, cand, n, G, tmp, f2, defer, tv, &ex2, nullptr);
                    if (sc > b2) { b2 = sc; bs2 = cand; bex2 = ex2; bv2 = tv; }
                }
                if (bs2 < 0) break;
                for (const Exec& e : bex2) tmp[e.gate] = 1;
                while (f2 < G.size() && tmp[f2]) ++f2;
                s2 = bs2;
                v2 = bv2;
            }
            if (f2 < G.size()) break;
        }
        s = bs;
        if (ops) ops->push_back({OP_XPOSE, (uint8_t)s, 0, 0, 0});
        total += best;
        vs = best_vs;
        commit(s, best_exec);
    }
    if (s < smin_io) {
        s = smin_io;  // lowest layout that stores coalesced; it also keeps the exchange inside wavefronts
        if (ops) ops->push_back({OP_XPOSE, (uint8_t)s, 0, 0, 0});
    }
    if (ops) ops->push_back({OP_END, 0, 0, 0, 0});
    if (n_exec) *n_exec = cnt;
    if (vs_out) *vs_out = vs;
    return total;
}

// Lanes hold the six lowest tile bits outside the register run, so while the run stays below tile
// bit 10 every wavefront keeps the same upper tile bits and exchanges only inside its own part of
// LDS: such a transpose needs no workgroup barrier.
void mark_transposes(std::vector<Op>& ops, size_t begin) {
    int s = -1;
    bool any_before = false, prev_cross = false;
    for (size_t i = begin; i < ops.size(); ++i) {
        Op& o = ops[i];
        if (o.kind == OP_LOAD) { s = o.a; continue; }
        if (o.kind != OP_XPOSE) continue;
        const bool cross = (s + kRegBits > 10) || (o.a + kRegBits > 10);
        o.b = cross ? 1 : 0;
        o.c = (any_before && (cross || prev_cross)) ? 1 : 0;
        any_before = true;
        prev_cross = cross;
        s = o.a;
    }
}

// Two or three consecutive CNOTs between neighbouring register bits (what a CNOT ring leaves inside
// a run) become one OP_CX_CHAIN: one operation to fetch and dispatch instead of three, and one
// permutation of the registers instead of three rounds of swaps.
void merge_cx_chains(std::vector<Op>& ops, size_t begin) {
    std::vector<Op> out(ops.begin(), ops.begin() + (long)begin);
    size_t i = begin;
    auto neighbour = [](const Op& o) { return o.kind == OP_CX_REG && o.a == o.b + 1; };
    while (i < ops.size()) {
        if (!neighbour(ops[i])) { out.push_back(ops[i++]); continue; }
        // longest run going up (next control = this target) or down (next target = this control)
        size_t up = 1, down = 1;
        while (up < 3 && i + up < ops.size() && neighbour(ops[i + up]) && ops[i + up].b == ops[i + up - 1].a) ++up;
        while (down < 3 && i + down < ops.size() && neighbour(ops[i + down]) && ops[i + down].a == ops[i + down - 1].b) ++down;
        const size_t len = up >= down ? up : down;
        if (len < 2) { out.push_back(ops[i++]); continue; }
        // arg numbers the six possible chains in the order the interpreter tests them
        const int dir = up >= down ? 0 : 1, a0 = ops[i].b;
        static const int combo[6][3] = {{0, 0, 3}, {1, 2, 3}, {0, 0, 2}, {0, 1, 2}, {1, 2, 2}, {1, 1, 2}};
        int id = -1;
        for (int k = 0; k < 6; ++k)
            if (combo[k][0] == dir && combo[k][1] == a0 && combo[k][2] == (int)len) id = k;
        if (id < 0) { out.push_back(ops[i++]); continue; }   // cannot happen with four register bits
        out.push_back({OP_CX_CHAIN, (uint8_t)a0, (uint8_t)len, (uint8_t)dir, id});
        i += len;
    }
    ops.swap(out);
}

int ceil_log2(int64_t v) {
    int b = 0;
    while (((int64_t)1 << b) < v) ++b;
    return b;
}

}  // namespace

void set_transpose_barriers(std::vector<Op>& ops) { mark_transposes(ops, 0); }

bool check_circuit(const qsv_circuit* c, int n, std::string* why) {
    auto fail = [&](const char* m) { if (why) *why = m; return false; };
    if (!c) return fail("circuit descriptor is NULL");
    if (n < 1 || n > 30) return fail("n_qubits must be in 1..30");
    if (c->n_layers < 0 || c->n_layers > 4096) return fail("n_layers must be in 0..4096");
    if (c->reupload != 0 && c->reupload != 1) return fail("reupload must be 0 or 1");
    if (c->n_rot < 0 || c->n_rot > 3) return fail("n_rot must be in 0..3");
    for (int r = 0; r < c->n_rot; ++r)
        if (c->rot[r] < QSV_RX || c->rot[r] > QSV_RZ) return fail("rotation axis must be 1..3");
    if (c->entangler < QSV_ENT_NONE || c->entangler > QSV_ENT_CZ_LADDER)
        return fail("entangler must be 0..2");
    return true;
}

int default_tile(int n, int64_t batch) {
    const int ext = n + ceil_log2(batch);
    // 2^12 amplitudes per tile measured best for large states.  For 10 or 11 qubits a tile is one
    // state row instead: matrices are then uniform per tile (no per-lane matrix path), and a batch
    // gives four times (twice) as many workgroups to spread over the compute units.
    const int t = std::max(kMinTile, std::min(12, ext));
    return (n < t && n >= kMinTile) ? n : t;
}

Plan build_plan(const qsv_circuit& c, int n, int64_t batch, bool inverse, int tile_log2, bool grad,
                int min_low_bits, bool defer) {
    Plan p;
    p.n = n;
    p.ext_bits = n + ceil_log2(batch);
    int t = tile_log2 > 0 ? tile_log2 : default_tile(n, batch);
    t = std::max(kMinTile, std::min(kMaxTile, t));
    p.tile = t;
    const bool has_u = (c.reupload + c.n_rot) > 0;
    p.n_mats = has_u ? c.n_layers * n : 0;
    p.row_dependent = c.reupload != 0;
    const bool rowdep = p.row_dependent || grad;
    // deferring needs qubits outside the tile, and index maps of 32 bits
    defer = defer && n > t && n <= 30;
    p.deferring = defer;

    const std::vector<Gate> G = lower(c, n, inverse);
    std::vector<uint8_t> done(G.size(), 0);
    size_t first = 0;
    // fewest low bits of a tile: kLowBits unless the caller asks for another number (3 = 64-byte runs)
    const int cmin = std::min(min_low_bits > 0 ? std::max(3, min_low_bits) : kLowBits, t);
    // local set = low c bits + window of t-c bits at w; c >= 4 keeps 128-byte runs contiguous
    auto all_geoms = [&](auto&& fn) {
        for (int cl = cmin; cl <= t; ++cl) {
            const int win = t - cl;
            const int wmax = (win > 0 && n > t) ? n - win : cl;
            for (int w = cl; w <= wmax; ++w) {
                if (w == cl && cl != cmin && n > t) continue;  // same set as (cmin, w = cmin)
                fn(Geom{t, cl, w});
            }
            if (n <= t) break;  // the whole state row is local: one geometry
        }
    };
    struct Cand { Geom g; int score; };
    std::vector<Cand> cands;
    while (first < G.size()) {
        cands.clear();
        all_geoms([&](Geom gm) {
            std::vector<uint8_t> tmp(done);
            int ne = 0;
            const int sc = run_pass(gm, n, G, tmp, first, rowdep, defer, nullptr, nullptr, nullptr, &ne, nullptr);
            cands.push_back({gm, sc});
        });
        std::stable_sort(cands.begin(), cands.end(), [](const Cand& a, const Cand& b) { return a.score > b.score; });
        Geom bestg = cands[0].g;
        if (defer && cands.size() > 1) {
            // two passes ahead (deferral makes the one-pass score short-sighted: a pass that defers a
            // long stretch of the chain scores well and leaves little for the next one)
            int best = -1;
            for (size_t ci = 0; ci < cands.size() && (int)ci < kLookTop; ++ci) {
                std::vector<uint8_t> tmp(done);
                int ne = 0;
                run_pass(cands[ci].g, n, G, tmp, first, rowdep, defer, nullptr, nullptr, nullptr, &ne, nullptr);
                size_t f2 = first;
                while (f2 < G.size() && tmp[f2]) ++f2;
                int b2 = 0;
                if (f2 >= G.size()) b2 = 1 << 24;             // finishes the circuit
                else
                    all_geoms([&](Geom g2) {
                        std::vector<uint8_t> tmp2(tmp);
                        int ne2 = 0;
                        const int sc2 = run_pass(g2, n, G, tmp2, f2, rowdep, defer, nullptr, nullptr, nullptr, &ne2, nullptr);
                        if (sc2 > b2) b2 = sc2;
                    });
                if (cands[ci].score + b2 > best) { best = cands[ci].score + b2; bestg = cands[ci].g; }
            }
        }
        Pass ps;
        ps.t = bestg.t; ps.c = bestg.c; ps.w = bestg.w;
        ps.op_begin = (int)p.ops.size();
        int ne = 0;
        VState vs;
        ps.defer_begin = (int)p.defers.size();
        run_pass(bestg, n, G, done, first, rowdep, defer, &p.ops, &p.mat_order, &p.defers, &ne, &vs);
        mark_transposes(p.ops, (size_t)ps.op_begin);
        merge_cx_chains(p.ops, (size_t)ps.op_begin);
        ps.op_count = (int)p.ops.size() - ps.op_begin;
        ps.defer_count = (int)p.defers.size() - ps.defer_begin;
        ps.n_gates = ne;
        if (vs.any) {
            // index map of the pass: map[j] = the index bits that flip in an amplitude's destination
            // when bit j of its position is set = the qubits whose set holds j (always j itself)
            ps.map_begin = (int)p.maps.size();
            for (int j = 0; j < n; ++j) {
                uint32_t mj = 0;
                for (int q = 0; q < n; ++q)
                    if ((vs.v[q] >> j) & 1u) mj |= 1u << q;
                p.maps.push_back(mj);
            }
        }
        p.passes.push_back(ps);
        if (ne == 0) { p.complete = false; break; }  // cannot happen: the first pending gate always fits some window
        while (first < G.size() && done[first]) ++first;
    }
    return p;
}

std::string describe_plan(const Plan& p) {
    std::string s;
    char buf[96];
    snprintf(buf, sizeof buf, "plan n=%d ext=%d tile=%d mats=%d rowdep=%d passes=%d\n", p.n,
             p.ext_bits, p.tile, p.n_mats, p.row_dependent ? 1 : 0, (int)p.passes.size());
    s += buf;
    for (const Pass& ps : p.passes) {
        snprintf(buf, sizeof buf, "P t=%d c=%d w=%d gates=%d :", ps.t, ps.c, ps.w, ps.n_gates);
        s += buf;
        for (int i = ps.op_begin; i < ps.op_begin + ps.op_count; ++i) {
            const Op& o = p.ops[i];
            switch (o.kind) {
                case OP_END: snprintf(buf, sizeof buf, " E"); break;
                case OP_LOAD: snprintf(buf, sizeof buf, " L%d", o.a); break;
                case OP_XPOSE: snprintf(buf, sizeof buf, " T%d:%d", o.a, o.b | (o.c << 1)); break;
                case OP_U: snprintf(buf, sizeof buf, " U%d:%d:%d", o.a, p.mat_order[o.arg], o.b); break;
                case OP_CX_REG: snprintf(buf, sizeof buf, " X%d:%d", o.a, o.b); break;
                case OP_CX_DYN: snprintf(buf, sizeof buf, " D%d:%d:%d", o.a, o.b, o.c); break;
                case OP_CZ_REG: snprintf(buf, sizeof buf, " Zr%d:%d", o.a, o.b); break;
                case OP_CZ_MIX: snprintf(buf, sizeof buf, " Zm%d:%d", o.a, o.b); break;
                case OP_CZ_LANE: snprintf(buf, sizeof buf, " Zl%x", (unsigned)o.arg); break;
                case OP_CX_CHAIN: snprintf(buf, sizeof buf, " C%c%d:%d", o.c ? 'd' : 'u', o.a, o.b); break;
                case OP_CX_PAR: snprintf(buf, sizeof buf, " Q%d:%d:%x", o.a, o.b, (unsigned)o.arg); break;
                case OP_CX_LANE: snprintf(buf, sizeof buf, " N%d:%d:%d", o.a, o.b, o.c); break;
                default: snprintf(buf, sizeof buf, " ?"); break;
            }
            s += buf;
        }
        for (int i = ps.defer_begin; i < ps.defer_begin + ps.defer_count; ++i) {
            const Op& o = p.defers[i];
            snprintf(buf, sizeof buf, " V%d:%d:%x", o.a, o.b, (unsigned)o.arg);
            s += buf;
        }
        if (ps.map_begin >= 0) {
            s += " M";
            for (int j = 0; j < p.n; ++j) {
                snprintf(buf, sizeof buf, "%s%x", j ? "," : "", (unsigned)p.maps[ps.map_begin + j]);
                s += buf;
            }
        }
        s += "\n";
    }
    return s;
}

}  // namespace qsv

// Host-only C entry point (declared in qsv.h): the text of the plan the library would run.
extern "C" int64_t qsv_plan_describe(const qsv_circuit* c, int n_qubits, int batch, int inverse, int tile_log2,
                                     char* buf, int64_t buf_bytes) {
    using namespace qsv;
    if (!check_circuit(c, n_qubits, nullptr) || batch < 1) return -1;
    const bool defer = (tile_log2 & 0x100) != 0;     // flag bit: the plan with deferred CNOTs
    tile_log2 &= 0xff;
    if (tile_log2 != 0 && (tile_log2 < kMinTile || tile_log2 > kMaxTile)) return -1;
    const Plan p = build_plan(*c, n_qubits, batch, inverse != 0, tile_log2, false, 0, defer);
    const std::string s = describe_plan(p);
    if (buf && buf_bytes > 0) {
        const size_t ncopy = s.size() < (size_t)buf_bytes - 1 ? s.size() : (size_t)buf_bytes - 1;
        memcpy(buf, s.data(), ncopy);
        buf[ncopy] = 0;
    }
    return (int64_t)s.size();
}
