// Host-side pass planner: turns a layered circuit into a list of fused passes over the state.
//
// A pass streams the whole state once (read + write).  Each workgroup owns one tile of 2^t
// amplitudes whose "local" index bits are the low c bits plus a window of t-c bits starting at
// bit w; every other index bit is constant inside the tile.  Inside a pass the tile lives in
// registers: each lane holds 2^R amplitudes spanning a run of R consecutive tile-local bit
// positions, applies every gate whose target sits in that run, and the run is moved by a
// transpose through LDS.  The planner emits, per pass, the operation list the kernel interprets.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "qsv.h"

namespace qsv {

constexpr int kRegBits = 4;      // R: amplitudes per lane = 2^R
constexpr int kMinTile = 10;     // 64 lanes x 16 amplitudes
constexpr int kMaxTile = 14;     // 1024 lanes x 16 amplitudes; one XOR-swizzled LDS plane of 2^14 floats = 64 KiB
constexpr int kLowBits = 4;      // c: 2^4 complex64 = one 128-byte line per contiguous run

enum OpKind : uint8_t {
    OP_END = 0,     // store the tile from the current layout
    OP_LOAD = 1,    // a = run start s: load the tile from global memory in layout s
    OP_XPOSE = 2,   // a = new run start: move the register run through LDS.  b = 1 if the exchange
                    // crosses wavefronts (a run above tile bit 9 is involved) and needs a workgroup
                    // barrier between writes and reads; c = 1 if a barrier is needed before the
                    // writes (an earlier exchange of this pass may still be read by other wavefronts)
    OP_U = 3,       // a = register bit j, b = 1 if the matrix depends on the state row,
                    // arg = index of the matrix in execution order (see Plan::mat_order)
    OP_CX_REG = 4,  // a = target register bit, b = control register bit
    OP_CX_DYN = 5,  // a = target register bit, b = control index bit (extended index),
                    // c = 1 if the control bit is the same for a whole wavefront
    OP_CZ_REG = 6,  // CZ between register bits a and b: sign flip of the 4 amplitudes with both set
    OP_CZ_MIX = 7,  // CZ between register bit a and index bit b outside the run (lane-dependent)
    OP_CZ_LANE = 8, // arg = rung mask (bit q -> CZ(q, q+1)), all rungs between index bits outside
                    // the run: one lane-dependent sign for all 16 amplitudes
    OP_CX_CHAIN = 9,// b = 2 or 3 consecutive OP_CX_REG between neighbouring register bits, as a CNOT
                    // ring produces them, done as one permutation of the registers.  a = control of
                    // the first; c = 0: targets go up (a -> a+1, a+1 -> a+2, ...), c = 1: the same
                    // gates in the opposite order, controls going down (a -> a+1, a-1 -> a, ...)
    OP_CX_PAR = 10, // a = target register bit; the control is the parity of the amplitude's position
                    // bits in arg (a mask over the extended index, no bit of it in the register run);
                    // b = the control qubit (for the description only)
    OP_CX_LANE = 12, // CNOT with the control in register bit a and the target behind bit b (0..5) of the
                    // lane number: the eight amplitudes with the control set are exchanged with the
                    // partner lane's (DPP for b < 2, ds_bpermute above); c = the target qubit (for the
                    // description only)
    OP_CX_DEFER = 11 // never part of an operation list: a CNOT that the pass's index map carries (see
                    // Plan::defers); a = target qubit, b = control qubit, arg = the control's bit set
};

struct Op {
    uint8_t kind, a, b, c;
    int32_t arg;
};
static_assert(sizeof(Op) == 8, "Op must be 8 bytes");

struct Pass {
    int t, c, w;        // tile bits, low bits, window start (extended index bit)
    int op_begin;       // first op in Plan::ops
    int op_count;
    int n_gates;        // circuit gates (fused level) executed by this pass
    int map_begin = -1; // >= 0: the pass writes every amplitude to a mapped index (first of its n entries
                        // in Plan::maps) and therefore must not write the buffer it reads
    int defer_begin = 0, defer_count = 0;   // its deferred CNOTs in Plan::defers
};

struct Plan {
    int n = 0;          // qubits
    int ext_bits = 0;   // n + ceil(log2(batch)): bits of the extended index b*2^n + k
    int tile = 0;       // t used by every pass
    int n_mats = 0;     // matrices per state row: n_layers * n (0 if the circuit has no rotations)
    bool row_dependent = false;  // matrices differ per sample (re-upload)
    bool complete = true;        // false only on an internal scheduling failure
    bool deferring = false;      // planned with deferred CNOTs (passes may carry index maps)
    std::vector<Pass> passes;
    std::vector<Op> ops;
    // Unitaries are numbered in the order the passes execute them, so that a tile reads its
    // matrices front to back: mat_order[k] = layer * n + qubit of the k-th executed unitary.
    std::vector<int32_t> mat_order;
    // Index maps of the passes that defer CNOTs: n entries per such pass; entry j = the index bits that
    // flip in an amplitude's destination index when bit j of its position is set (position = tile
    // bits as stored plus the amplitude's place in the tile at the end of the pass).  Bits >= n (the
    // state row) always map to themselves.
    std::vector<uint32_t> maps;
    std::vector<Op> defers;      // the deferred CNOTs, pass by pass (description and tests only)
};

// Validates a circuit descriptor; returns false and fills why on failure.
bool check_circuit(const qsv_circuit* c, int n, std::string* why);

// tile_log2 = 0 picks the default.  grad = true marks every rotation matrix as row-dependent
// (a shifted circuit overrides one matrix per state row).
// defer = true lets CNOTs whose target is outside a pass's tile be carried by the pass's index map
// (fewer passes; such a plan needs a second state buffer, see Pass::map_begin).
Plan build_plan(const qsv_circuit& c, int n, int64_t batch, bool inverse, int tile_log2, bool grad,
                int min_low_bits = 0, bool defer = false);

std::string describe_plan(const Plan& p);

// Fills in the barrier flags of the OP_XPOSE entries of one pass's operation list (starting with its
// OP_LOAD), as build_plan does for the passes it emits.
void set_transpose_barriers(std::vector<Op>& ops);

int default_tile(int n, int64_t batch);

}  // namespace qsv
