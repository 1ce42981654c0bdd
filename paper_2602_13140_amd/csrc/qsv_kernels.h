// Internal launch interface between the C-ABI layer and the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "qsv_plan.h"

namespace qsv {

// Circuit fields the device-side matrix builders need.
struct CircDev {
    int n, n_layers, reupload, n_rot, rot[3];
    int slots() const { return reupload + n_rot; }
};

// How state rows map to samples.  Plain calls: row = sample.  Gradient launches: row r of the
// chunk is circuit gid = row0 + r; sample = gid / per, variant v = gid % per; v < two_p replaces
// the matrix of parameter v/2 of the circuit being run by its +pi/2 (v even) or -pi/2 (v odd)
// shifted version.  Whole-circuit gradients use per = 2P+1 (variant 2P is the unshifted circuit);
// the layer-by-layer gradient runs the circuit's last layers only and shifts parameters of their
// first layer: per = two_p = 2 * slots * n.
struct RowMap {
    int grad;        // 0 plain, 1 gradient
    int two_p;       // variants that replace a matrix: v < two_p (also the row stride of the shifted table)
    int per;         // circuits per sample (two_p + 1 when the unshifted circuit is among them)
    int64_t row0;
    int slots_n;     // (reupload + n_rot) * n
    int n;
};

struct PassArgs {
    float2* state;       // the buffer the tiles are written to
    const float2* in;    // the buffer the tiles are read from: state itself, or (a pass with an index map
                         // must not write what it reads) another buffer of the same shape
    const unsigned* imap;  // not NULL: n entries; an amplitude whose position (tile bits plus its place in
                         // the tile at the end of the pass) has bit j set is written to the index with the
                         // bits imap[j] flipped: deferred CNOTs (needs n > tile and n <= 28)
    const float2* src;   // not NULL: tiles are read from src[sample of the row] instead of in (needs n >= tile)
    const Op* ops;
    double* zout;        // not NULL: the pass also writes <Z_zq> partials [tile][wavefront] (needs n >= tile)
    int zq;
    int nostore;         // with zout: the state is not written back
    int nt_store;        // nontemporal tile stores (states much larger than the last-level cache)
    int rev;             // workgroups take the tiles in descending order (see run_circuit)
    int prio;            // wavefronts raise their issue priority while they compute addresses and issue the
                         // tile's loads, and again for its stores (the gates run at the base priority)
    const float* mats;   // [samples if rowdep][n_mats][8], matrices in execution order
    const int* exec_of;  // [n_mats]: (layer * n + qubit) -> execution-order index
    const float* ovr;    // gradient: [samples if rowdep][2P][8] shifted matrices
    uint64_t total;      // valid extended indices = rows * 2^n
    int n, c, w;
    int n_mats;
    int rowdep;          // matrices differ per sample
    RowMap rm;
};

hipError_t launch_pass(int tile, int planes, const PassArgs& a, uint64_t n_tiles, hipStream_t st);

// Address, on the current device (which must be `device`), of the library's fixed scratch array of
// kStaticScratchBytes bytes (256-byte aligned).  Looked up once per device; allocates nothing.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
hipError_t static_scratch(int device, void** ptr);
hipError_t set_pass_attributes();

// one-gate-per-launch kernels (fallback for n < 4 and cross-check path)
hipError_t launch_naive_u(float2* state, int64_t rows, int n, int q, const float* mats,
                          const float* ovr, int mat_id, int n_mats, int rowdep, const RowMap& rm,
                          hipStream_t st);
hipError_t launch_naive_cnot(float2* state, int64_t rows, int n, int ctrl, int tgt, hipStream_t st);
hipError_t launch_naive_cz_ladder(float2* state, int64_t rows, int n, hipStream_t st);

// fused per-(layer, qubit) matrices; out: [samples if reupload][n_layers*n][8] floats.  order
// (device, [n_layers*n], may be NULL = natural order) gives the (layer*n + qubit) id stored at
// each position of a sample's table, exec_of (device, same length, NULL with order) its inverse.
// period = n: the two tables have n entries, describe a one-layer circuit and repeat for every layer
// (the table of the whole circuit as the tables of its layers, run one by one, back to back).
hipError_t launch_build_mats(const CircDev& c, const float* params, const float* feats,
                             int64_t samples, int inverse, const int* order, const int* exec_of, float* out,
                             double* side, hipStream_t st, int period = 0);
// bytes of the side buffer launch_build_mats needs (phase factors and the last qubit's matrices in double)
inline size_t build_mats_side_bytes(const CircDev& c, int64_t samples) {
    const size_t tables = (size_t)(c.reupload ? samples : 1);
    return tables * (size_t)c.n_layers * ((size_t)c.n * 16 + 64);
}
// shifted matrices for the parameter-shift rule; out: [samples if reupload][2P][8]
hipError_t launch_build_shifted(const CircDev& c, const float* params, const float* feats,
                                int64_t samples, float* out, hipStream_t st);

// encoding
hipError_t launch_norms(const float* x, int64_t samples, int64_t dim, double* partial, int nblk,
                        double* inv_norm, float* norm_out, hipStream_t st);
// norm and state rows of small samples (dim <= 4096, n <= 12) in one launch; inv_norm receives 1/||x_b||
hipError_t launch_encode_small(const float* x, int64_t samples, int64_t dim, int n, double* inv_norm, float* norm_out,
                               float2* state, hipStream_t st);
// A whole small workload in one launch: encoding, circuit (decode = 1: followed by its inverse), final
// state, and the measurement `kind` (QSV_M_PROBS or QSV_M_EXPZ_ALL).  A thread keeps 2^regs amplitudes
// (regs = 2, 3 or 4), the other index bits are bits of the thread number (at most 8: 256 threads); with
// fewer than 6 of them a wavefront holds 2^(6 - bits) samples.  A workgroup keeps the matrices of its
// samples in LDS (at most kSmallMats).
constexpr int kSmallMaxQubits = 10;
constexpr int64_t kSmallApplyAmplitudes = (int64_t)1 << 21;   // batch * 2^n up to which one launch beats the fused passes
constexpr int kSmallMats = 512;   // matrices a workgroup keeps in LDS (16 KiB)
inline int small_rows_per_group(int n, int regs) {
    const int tb = n > regs ? n - regs : 0;
    return tb < 6 ? 64 >> tb : 1;
}
inline int64_t small_mats_per_group(const CircDev& c, int regs) {
    if (c.reupload + c.n_rot == 0) return 0;
    return (int64_t)(c.reupload ? small_rows_per_group(c.n, regs) : 1) * c.n_layers * c.n;
}
// Amplitudes per thread: the most that still gives the chip about four wavefronts per SIMD (4096), else the
// fewest; among those only what fits the matrix limit.  0: nothing fits.
inline int small_choose_regs(const CircDev& c, int64_t batch) {
    int fallback = 0;
    for (int r = 4; r >= 2; --r) {
        if (c.n - r > 8 || small_mats_per_group(c, r) > kSmallMats) continue;
        const int rows_g = small_rows_per_group(c.n, r);
        const int tb = c.n > r ? c.n - r : 0;
        const int64_t waves = ((batch + rows_g - 1) / rows_g) * (tb > 6 ? 1 << (tb - 6) : 1);
        if (waves >= 4096) return r;
        fallback = r;             // the smallest that fits so far
    }
    return fallback;
}
// x = NULL: start from the amplitudes in `state`; passes pass_first..pass_last (0 = the circuit, 1 = its inverse);
// kind = 0: no measurement (the final state is always written)
hipError_t launch_forward_small(int regs, const float* x, int64_t dim, int64_t batch, const CircDev& c, int entangler,
                                const float* params, const float* feats, int pass_first, int pass_last, int kind,
                                float2* state, float* out, float* norm_out, hipStream_t st);
hipError_t launch_encode_write(const float* x, int64_t dim, int n, int64_t rows, const double* inv_norm,
                               const RowMap& rm, float2* state, hipStream_t st);

// measurement
hipError_t launch_probs(const float2* state, uint64_t total, float* out, hipStream_t st);
// partial: [rows][nblk][13] doubles; nblk = max(1, 2^n / 4096)
hipError_t launch_expz_block(const float2* state, int64_t rows, int n, double* partial, hipStream_t st);
// rows of at most 4096 amplitudes: <Z_q> of every qubit (q_only < 0) or of q_only in one launch, same bits as block + finish
hipError_t launch_expz_small(const float2* state, int64_t rows, int n, int q_only, float* out_f, hipStream_t st);
hipError_t launch_expz_finish(const double* partial, int64_t rows, int n, int q_only, float* out_f,
                              double* out_d, hipStream_t st);
// Where one-qubit results of gradient rows go: circuit gid = row0 + r lands at
// out[(gid / per) * stride + offset + gid % per].
struct Scatter { int64_t row0, per, stride, offset; };
hipError_t launch_expz_finish_scatter(const double* partial, int64_t rows, int n, int q, double* out,
                                      const Scatter& sc, hipStream_t st);
// out[scatter(row)] = sum of the row's per_row partials written by a pass with zout
hipError_t launch_zsum_finish(const double* partial, int64_t rows, int64_t per_row, double* out,
                              const Scatter& sc, hipStream_t st);
// states[r] = src[sample of row r] for the rows of a gradient chunk (src: [samples][2^n])
hipError_t launch_gather_rows(const float2* src, int n, int64_t rows, const RowMap& rm, float2* states,
                              hipStream_t st);
// partial: [rows][n_v][nblk] doubles with nblk = max(1, 2^(n-m) / 4096)
hipError_t launch_marginal_block(const float2* state, int64_t rows, int n, uint64_t mask, int64_t n_v,
                                 double* partial, hipStream_t st);
hipError_t launch_marginal_finish(const double* partial, int64_t rows_times_v, int64_t nblk, float* out,
                                  int renorm_mode, double* scale, hipStream_t st);
hipError_t launch_project(float2* state, int64_t rows, int n, uint64_t mask, const double* scale,
                          hipStream_t st);
hipError_t launch_fidelity_block(const float2* state, int64_t rows, int n, const float* x, int64_t dim,
                                 double* partial, int nblk, const RowMap& rm, hipStream_t st);
hipError_t launch_fidelity_finish(const double* partial, int nblk, int64_t rows, float* out, double* out_d,
                                  hipStream_t st);
// trash reset: rows (sample, outcome) of a chunk from the state; sum of the rows' fidelities per sample
hipError_t launch_reset_rows(const float2* state, int n, uint64_t mask, int64_t rows, const RowMap& rm,
                             float2* work, hipStream_t st);
hipError_t launch_reset_sum(const double* Frow, int64_t per, int64_t B, float* out, hipStream_t st);
// finite-shot <Z_q> from samples [rows][shots] -> out [rows][n]
hipError_t launch_shot_expz(const long long* samples, int64_t shots, int64_t rows, int n, float* out,
                            hipStream_t st);
// sampling: bsum/cum are uint64 [rows][nblk], nblk = max(1, 2^n / 4096)
hipError_t launch_sample(const float2* state, int64_t rows, int n, const double* uniforms, int64_t shots,
                         unsigned long long* cum, long long* out, hipStream_t st);

// <P> of a Pauli string (X on xmask, Y on ymask, Z on zmask) per row; partial: rows * blocks * 2 doubles
hipError_t launch_pauli(const float2* state, int64_t rows, int n, uint64_t xmask, uint64_t ymask,
                        uint64_t zmask, double* partial, float* out, hipStream_t st);

// Reverse-mode gradient.  launch_adj_init: S[2r] = A[r], S[2r+1] = O A[r] (rows of A) for the
// diagonal observable O: kind 0 Z_q; kind 1 -P0(mask); kind 2 sum_q coef[r][q] Z_q.
// launch_trash_loss: f[sample0+r][2P] = 1 - P0(mask) of row r (partial: rows * blocks doubles, blocks
// as for the <Z> reductions).  launch_mse_coef: from z[rows][n] and targets y[samples][n], the loss
// 1/n sum (z-y)^2 into f[.][2P] and coef = 2/n (z-y).
// launch_adj_init: lambda = O psi for the rows of A; paired = 1 writes (psi, lambda) into rows 2r, 2r+1
// of S, paired = 0 writes lambda alone into row r.
// launch_adj_layer: for row pairs (psi0 + rstride r 2^n, lam0 + rstride r 2^n), both taken back to the
// start of `layer`, the derivatives with respect to that layer's angles, written into f[sample][2p],
// f[sample][2p+1] as (g, -g).  partial: row_pairs * n * (adj_trans_blocks(n) + 1) * 8 doubles.
hipError_t launch_adj_init(const float2* A, int n, int kind, int q, uint64_t mask, const double* coef,
                           int64_t rows, float2* S, int paired, hipStream_t st);
hipError_t launch_trash_loss(const float2* A, int n, uint64_t mask, int64_t rows, int64_t sample0, int64_t P,
                             double* partial, double* f, hipStream_t st);
hipError_t launch_mse_coef(const double* z, const float* y, int n, int64_t rows, int64_t sample0, int64_t P,
                           double* coef, double* f, hipStream_t st);
// optimiser steps in double on float storage; t is the 1-based step count of Adam
hipError_t launch_sgd(float* p, const float* g, int64_t count, double lr, hipStream_t st);
hipError_t launch_adam(float* p, const float* g, float* m, float* v, int64_t count, int64_t t, double lr,
                       double b1, double b2, double eps, hipStream_t st);
int adj_trans_blocks(int n);
hipError_t launch_adj_layer(const float2* psi0, const float2* lam0, int rstride, int n, int64_t row_pairs,
                            double* partial, const CircDev& c,
                            int layer, const float* params, const float* feats, int64_t sample0, int64_t P,
                            double* f, hipStream_t st);

// gradient assembly from f[B][2P+1] (double)
hipError_t launch_grad_finish(const double* f, int64_t B, int64_t P, const CircDev& c, const float* feats,
                              float* loss, float* grad, float* mean_loss, float* mean_grad,
                              hipStream_t st);

}  // namespace qsv
