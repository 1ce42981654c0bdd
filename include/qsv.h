/* qsv — batched complex64 state-vector simulation of layered parameterised circuits on one
 * AMD MI355X (gfx950).  C ABI of libqsv.so.
 *
 * What the calls compute is fixed by the task statement (its "north star" paragraph and the five
 * workload configs); the source paper itself contains no circuit material, so the conventions
 * below are the stated readings that the CPU oracle pins with closed forms.
 *
 * Conventions
 *   - qubit q is bit q of the amplitude index k (qubit 0 = least-significant bit = stride 1).
 *   - state: DEVICE memory, complex64 [batch][2^n], interleaved (re, im) float32, sample-major.
 *   - RX(t) = [[c,-is],[-is,c]], RY(t) = [[c,-s],[s,c]], RZ(t) = diag(e^{-it/2}, e^{+it/2}),
 *     c = cos(t/2), s = sin(t/2).
 *   - one layer = [re-upload RX(w[l][q] * feats[b][q]) on q = 0..n-1, if reupload]
 *                 -> rotation slot 0 on q = 0..n-1 -> slot 1 ... -> entangler.
 *   - CNOT ring: CNOT(control q, target (q+1) mod n) for q = 0,1,...,n-1 in that order (none for
 *     n = 1).  CZ ladder: CZ(q, q+1) for q = 0..n-2.
 *   - parameters: float32 [P] shared by the whole batch, P = n_layers*(reupload+n_rot)*n, flat
 *     index p = (l*(reupload+n_rot) + slot)*n + q; slot 0 holds w when reupload = 1.
 *
 * Ownership and execution
 *   - The caller owns every device buffer (state, inputs, outputs, workspace); the context owns
 *     only host-side plans.  No call allocates or frees device memory.
 *   - All work is enqueued on the HIP stream given to qsv_create and is asynchronous with respect
 *     to the host; no call synchronises the stream (one exception, a measurement aid and no part of
 *     the path: qsv_probe_pass).  The pass plans of the circuits a context has run are kept in host
 *     memory until qsv_destroy and uploaded by asynchronous copies on the stream; when the plan
 *     region of the workspace is full it is refilled from its start, in stream order.
 *     Part of a call's kernels may run on a second
 *     stream that the context owns (default priority); it waits for the caller's stream at the
 *     start of that work and the caller's stream waits for it before the call's remaining work, so
 *     to the caller everything is ordered as if it ran on the one stream (also under stream
 *     capture, where the second stream joins the capture and leaves it within the call).  Host
 *     structs (qsv_circuit, qsv_measure_req) are read during the call and may be reused afterwards.
 *   - Pointers named *_dev are device pointers; everything else is host memory.
 *   - Argument errors are detected on the host before anything is launched and reported through
 *     the return code; qsv_last_error gives the text.  No exceptions, no abort.
 *   - One context per stream; a context is not thread-safe.
 */
#ifndef QSV_H
#define QSV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct qsv_ctx qsv_ctx;

typedef enum {
    QSV_OK = 0,
    QSV_ERR_INVALID_ARG = 1,
    QSV_ERR_UNSUPPORTED = 2,
    QSV_ERR_ZERO_NORM = 3,   /* reserved, never returned: calls are asynchronous, so a zero vector
                                is reported in band (norm 0 and an all-zero state from
                                qsv_amp_encode, -1 for every shot from QSV_M_SAMPLE) */
    QSV_ERR_WORKSPACE = 4,
    QSV_ERR_HIP = 5
} qsv_status;

typedef enum { QSV_RX = 1, QSV_RY = 2, QSV_RZ = 3 } qsv_axis;
typedef enum { QSV_ENT_NONE = 0, QSV_ENT_CNOT_RING = 1, QSV_ENT_CZ_LADDER = 2 } qsv_ent;

/* Layered circuit (task statement: "encoder/decoder variational layers", "data re-uploading
 * blocks"; workload configs 0-4 give the rotation lists and entanglers). */
typedef struct {
    int32_t n_layers;  /* >= 0 */
    int32_t reupload;  /* 1: every layer starts with RX(w[l][q] * feats[b][q]) on each qubit */
    int32_t n_rot;     /* 0..3 rotation slots per layer */
    int32_t rot[3];    /* qsv_axis of each slot, in application order */
    int32_t entangler; /* qsv_ent */
} qsv_circuit;

/* Number of parameters P of a circuit on n qubits; -1 on a bad descriptor. */
int64_t qsv_num_params(const qsv_circuit* c, int n_qubits);

/* Workspace size in bytes that is enough for every call below at (n_qubits, batch) with up to
 * 64 layers, a copy of the state for qsv_apply_layers with deferred CNOTs included (up to 28
 * qubits).  Returns 0 for n_qubits outside 1..30 or batch < 1.  A larger workspace lets
 * qsv_param_shift_grad run more circuits per launch. */
size_t qsv_workspace_bytes(int n_qubits, int batch);

/* Workspace size in bytes with which qsv_param_shift_grad can work layer by layer on circuit c:
 * qsv_workspace_bytes plus room for n_layers + 1 states per sample.  Returns 0 on bad arguments.
 * With less, qsv_param_shift_grad still works and runs every shifted circuit whole. */
size_t qsv_grad_workspace_bytes(int n_qubits, int batch, const qsv_circuit* c);

/* Create a context bound to (n_qubits, batch), a device ordinal, a HIP stream (hipStream_t cast
 * to void*, NULL = default stream), the caller's state buffer complex64 [batch][2^n] and the
 * caller's workspace (256-byte aligned device memory of at least qsv_workspace_bytes bytes).
 * batch must be in 1..2^24 with batch * 2^n_qubits <= 2^36.  Nothing is launched. */
qsv_status qsv_create(qsv_ctx** out, int n_qubits, int batch, int device, void* hip_stream,
                      void* state_dev, void* ws_dev, size_t ws_bytes);
void qsv_destroy(qsv_ctx* ctx);

/* Text of the last error on this context (or of the last failed qsv_create when ctx is NULL).
 * The string is owned by the library and stays valid until the next call on the context. */
const char* qsv_last_error(const qsv_ctx* ctx);

/* Amplitude encoding (task statement: "amplitude encoding of classical vectors"; every config):
 * state[b][k] = x[b][k] / ||x[b]||_2 for k < dim, 0 for dim <= k < 2^n, imaginary part 0.
 * x_dev: float32 [batch][dim], 1 <= dim <= 2^n.  norm_out_dev: float32 [batch] or NULL, receives
 * ||x[b]||_2.  A zero vector gives an all-zero state and norm 0 (no NaN). */
qsv_status qsv_amp_encode(qsv_ctx* ctx, const float* x_dev, int64_t dim, float* norm_out_dev);

/* Apply the layered circuit to every sample of the state, in place (task statement: "encoder/
 * decoder variational layers, data re-uploading blocks").  params_dev: float32 [P].  feats_dev:
 * float32 [batch][n], required when c->reupload = 1, ignored otherwise.  inverse = 1 applies the
 * exact inverse: layers last..first, inside a layer the entangler gates in reverse order, then
 * the rotation slots in reverse order with negated angles, then the re-upload RX negated. */
qsv_status qsv_apply_layers(qsv_ctx* ctx, const qsv_circuit* c, const float* params_dev,
                            const float* feats_dev, int inverse);

/* Measurement kinds (task statement: "measurement probabilities/expectations", "trash-qubit
 * probability", "fidelity with the input state", "seeded measurement samples"). */
typedef enum {
    QSV_M_PROBS = 1,        /* out float32 [batch][2^n]: p[k] = |a[k]|^2 */
    QSV_M_EXPZ_ALL = 2,     /* out float32 [batch][n]: <Z_q> = sum_k (1-2 bit_q(k)) p[k] */
    QSV_M_EXPZ_ONE = 3,     /* out float32 [batch]: <Z_qubit> */
    QSV_M_MARGINAL = 4,     /* out float32 [batch][2^m], m = popcount(mask) <= 20: probability of
                               each reading v of the mask qubits (lowest mask qubit = bit 0 of v) */
    QSV_M_PROJECT_ZERO = 5, /* out float32 [batch]: P0 = P(all mask qubits read 0); the state is
                               then projected onto that subspace (other amplitudes set to 0) and,
                               when renormalise = 1, divided by sqrt(P0); P0 = 0 leaves zeros */
    QSV_M_FIDELITY = 6,     /* out float32 [batch]: |<a_in|a>|^2 with a_in = x/||x||, x_dev float32
                               [batch][dim] zero-padded to 2^n */
    QSV_M_SAMPLE = 7        /* out int64 [batch][shots]: basis-state indices drawn by the integer
                               inverse-CDF rule below from the caller's uniforms */
} qsv_mkind;

/* Sampling rule (bit-exact by construction): with p32[k] = float32(|a[k]|^2) exactly as
 * QSV_M_PROBS writes it, w[k] = floor(double(p32[k]) * 2^60) as uint64, W[k] = w[0]+...+w[k],
 * r = floor(u * 2^53), t = floor(r * W[last] / 2^53) (128-bit product); the sample is the smallest
 * k with W[k] > t.  Shots keep the order of the uniforms.  W[last] = 0 writes -1 for every shot. */
typedef struct {
    int32_t kind;               /* qsv_mkind */
    int32_t qubit;              /* EXPZ_ONE */
    uint64_t mask;              /* MARGINAL, PROJECT_ZERO: non-empty subset of qubits 0..n-1 */
    int32_t renormalise;        /* PROJECT_ZERO */
    int32_t reserved;           /* must be 0 */
    const float* x_dev;         /* FIDELITY */
    int64_t dim;                /* FIDELITY: 1..2^n */
    const double* uniforms_dev; /* SAMPLE: float64 [batch][shots], values in [0,1) */
    int64_t shots;              /* SAMPLE: >= 0 */
    void* out_dev;              /* result, type and shape fixed by kind */
} qsv_measure_req;

qsv_status qsv_measure(qsv_ctx* ctx, const qsv_measure_req* req);

/* A whole small workload in ONE kernel launch (task statement: "batch-parallel launches across
 * samples"; workload configs 0 and 1, whose separate calls cost more in launches than in arithmetic):
 * qsv_amp_encode(x), qsv_apply_layers(c, inverse = 0), with decode = 1 then qsv_apply_layers(c,
 * inverse = 1) (encoder followed by its decoder), the final state written to the context's state
 * buffer, and one measurement of it, kind = QSV_M_PROBS (out_dev float32 [batch][2^n]) or
 * QSV_M_EXPZ_ALL (out_dev float32 [batch][n]).  Arguments as in those calls; norm_out_dev may be
 * NULL.  Same definitions and tolerances as the separate calls (the probabilities are the same
 * float32 function of the stored state; sums may differ in their last bits from the separate
 * calls', which add in another order).  A thread keeps 4, 8 or 16 amplitudes in registers and a
 * workgroup of at most 256 threads holds a sample, so this serves n_qubits <= 10, and circuits with
 * at most 512 matrices per workgroup: n_layers * n_qubits, times the samples that share a
 * wavefront when reupload = 1 (2^(8 - n_qubits) of them up to 8 qubits, one above).  Anything else
 * returns QSV_ERR_UNSUPPORTED before a launch, and the separate calls serve it.  Needs no
 * workspace.  It pays while the launches of the separate calls cost more than their arithmetic:
 * up to about 2^21 amplitudes in the whole batch (measured: 10 qubits x 1024 samples 35 against
 * 72 us); per gate it is about three times slower than the fused passes of qsv_apply_layers, so
 * larger batches are better served by the separate calls. */
qsv_status qsv_forward_small(qsv_ctx* ctx, const float* x_dev, int64_t dim, const qsv_circuit* c,
                             const float* params_dev, const float* feats_dev, int decode, int kind,
                             void* out_dev, float* norm_out_dev);

/* qsv_measure for callers that cannot allocate device memory and have no workspace to spare for it:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same request,
 * same kernels, same results bit for bit; only the kernels' partial results (block sums, cumulative
 * weights) go to a fixed array of 4 MiB inside the library's code object instead of the caller's
 * workspace.  The call allocates and frees nothing, on the device or through any library.  Every GPU
 * the library runs on holds one copy of the array until the process ends.  A request whose partial
 * results need more than 4 MiB (enough for all five workload configs; the need grows with
 * batch * 2^n_qubits / 4096) is rejected with QSV_ERR_WORKSPACE before anything is launched.  All
 * calls on one GPU share that GPU's array, whatever their context or stream: calls that overlap in
 * time on one GPU race, so keep them on one stream or order them with events.  Nothing in the array
 * needs to start at zero: every byte that is read has been written earlier in the same call. */
qsv_status qsv_measure_static(qsv_ctx* ctx, const qsv_measure_req* req);

/* Fidelity of an autoencoder with a true reset of its trash qubits (task statement, workload
 * config 3; the projection of QSV_M_PROJECT_ZERO is the post-selected stand-in for it).  The
 * context's state is taken as the encoder output.  For every outcome t of measuring the qubits of
 * mask (at most 10), the unnormalised conditional state with the trash qubits set to 0 is run
 * through circuit c in inverse mode (the decoder) and
 *   out[b] = sum_t | <x_b / ||x_b||  |  D (psi_t (x) |0>) > |^2        (float [batch]).
 * Works in the workspace, 2^m decoder runs per sample in chunks; the state is left as it was. */
qsv_status qsv_reset_fidelity(qsv_ctx* ctx, const qsv_circuit* c, const float* params_dev,
                              const float* feats_dev, uint64_t mask, const float* x_dev, int64_t dim,
                              float* out_dev);

/* Finite-shot estimate of <Z_q> for every qubit from basis-state samples as QSV_M_SAMPLE writes
 * them: samples_dev int64 [batch][shots]; out_dev float [batch][n_qubits] = mean over the shots of
 * (1 - 2 bit_q); entries < 0 (no valid outcome) are skipped, a row without valid shots gives 0. */
qsv_status qsv_shot_expz(qsv_ctx* ctx, const long long* samples_dev, int64_t shots, float* out_dev);

/* Expectation value of a Pauli string on the current state (task statement: "measurement
 * (... <Z> ...)", widened to X and Y): P = product over qubits of X (bit set in xmask), Y (ymask)
 * or Z (zmask), identity elsewhere; the masks must not overlap and name qubits < n_qubits.
 * out_dev: float [batch].  Computed directly as sum_k conj(a[k ^ f]) i^nY (-1)^popcount(k & s) a[k]
 * with f = xmask | ymask, s = ymask | zmask: one read pass, the state is not modified. */
qsv_status qsv_pauli_expect(qsv_ctx* ctx, uint64_t xmask, uint64_t ymask, uint64_t zmask, float* out_dev);

/* Parameter-shift gradient of f_b = <Z_obs> after encode + circuit (task statement: "parameter-
 * shift gradients over the batch"; config 2: "2 circuits per param per sample"):
 *   grad[b][p] = 1/2 [ f_b(angle_p + pi/2) - f_b(angle_p - pi/2) ]
 * (times feats[b][q] when p is a re-upload weight, whose angle is w*feat).  x_dev float32
 * [batch][dim]; loss_dev float32 [batch] receives the unshifted f_b; grad_dev float32 [batch][P];
 * mean_loss_dev [1] and mean_grad_dev [P] receive the batch means when not NULL.  Uses the
 * workspace for the shifted circuits' states; the context's state buffer is left untouched.
 * When the workspace has room for n_layers + 1 states per sample (qsv_grad_workspace_bytes), the
 * unshifted circuit's state before every layer is kept and a circuit that shifts a parameter of
 * layer l runs layers l..L-1 only, from that state: the same values with about half the gate
 * applications (option grad_layered = 0 switches this off). */
qsv_status qsv_param_shift_grad(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                                const float* params_dev, const float* feats_dev, int32_t obs_qubit,
                                float* loss_dev, float* grad_dev, float* mean_loss_dev,
                                float* mean_grad_dev);

/* The same loss and gradient as qsv_param_shift_grad (same arguments, same outputs, equal up to
 * rounding), evaluated in reverse mode (task statement: "gradients over the batch"; listed there
 * as the cross-check of the shift rule).  Per sample one forward run gives psi and the loss; psi
 * and lambda = Z_obs psi are then taken back through the layers together, and at the start of
 * each layer the derivative with respect to an angle of slot s on qubit q is
 * 2 Re <lambda| W^dagger (-i/2 P_s) W |psi> on that qubit, W = the layer's earlier slots on it,
 * read off the 2x2 sums  M_q[a][b] = sum_rest conj(lambda[a, rest]) psi[b, rest].
 * Work: about 3 L layers and L n reductions per sample instead of 2 P circuits.  Uses the workspace
 * (three states per sample of a chunk); the context's state buffer is left untouched. */
qsv_status qsv_adjoint_grad(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                            const float* params_dev, const float* feats_dev, int32_t obs_qubit,
                            float* loss_dev, float* grad_dev, float* mean_loss_dev,
                            float* mean_grad_dev);

/* Training losses built from the measured quantities (task statement: the autoencoder of workload
 * config 3 empties its trash qubits; the re-uploading model of config 1 regresses <Z_q>).
 *   QSV_LOSS_TRASH: loss_b = 1 - P0_b, P0 = probability that every qubit of mask reads 0.
 *   QSV_LOSS_MSE_Z: loss_b = 1/n sum_q (<Z_q>_b - targets[b][q])^2, targets_dev float [batch][n]. */
typedef enum { QSV_LOSS_TRASH = 1, QSV_LOSS_MSE_Z = 2 } qsv_loss_kind;
typedef struct {
    int32_t kind;             /* qsv_loss_kind */
    int32_t reserved;         /* 0 */
    uint64_t mask;            /* QSV_LOSS_TRASH: trash qubits, bit q = qubit q; at least one, all < n_qubits */
    const float* targets_dev; /* QSV_LOSS_MSE_Z: [batch][n_qubits]; else ignored */
} qsv_loss;

/* Per-sample loss [batch] and gradient [batch][P] of a training loss, and optionally their batch
 * means, evaluated in reverse mode as in qsv_adjoint_grad (lambda = O psi with O = -P0 projector,
 * or sum_q 2/n (<Z_q> - y) Z_q); the values are those of the shift rule.  Arguments as
 * qsv_param_shift_grad; loss is a host struct read during the call. */
qsv_status qsv_loss_grad(qsv_ctx* ctx, const qsv_circuit* c, const float* x_dev, int64_t dim,
                         const float* params_dev, const float* feats_dev, const qsv_loss* loss,
                         float* loss_dev, float* grad_dev, float* mean_loss_dev, float* mean_grad_dev);

/* Optimiser steps on the device, asynchronous on the context's stream; arithmetic in double, storage
 * float.  qsv_sgd_step: params -= lr * grad.  qsv_adam_step (Kingma and Ba, Algorithm 1): m, v are
 * the caller's moment buffers [count] (zero before the first step), t >= 1 the step count.
 * count = 0 is a no-op; bad arguments return QSV_ERR_INVALID_ARG. */
qsv_status qsv_sgd_step(qsv_ctx* ctx, float* params_dev, const float* grad_dev, int64_t count, double lr);
qsv_status qsv_adam_step(qsv_ctx* ctx, float* params_dev, const float* grad_dev, float* m_dev, float* v_dev,
                         int64_t count, int64_t t, double lr, double beta1, double beta2, double eps);

/* Host-only introspection of the pass plan the library would run for a circuit (no GPU needed):
 * writes a text description (one line per pass, one token per operation) into buf and returns the
 * number of bytes needed (excluding the terminator), or -1 on a bad descriptor.  tile_log2 = 0
 * picks the library's default tile size.  Used by the host-logic tests. */
int64_t qsv_plan_describe(const qsv_circuit* c, int n_qubits, int batch, int inverse,
                          int tile_log2, char* buf, int64_t buf_bytes);

/* Measurement aid: one pass of the fused-pass kernel that only loads every tile (low_bits low index
 * bits plus a window starting at bit window_start, as the planner would choose), moves the
 * register run through LDS `transposes` times and stores the tile back unchanged.  It gives the
 * streaming ceiling of the pass kernel's access pattern, with no gate arithmetic.  The state is
 * left as it was.  Unlike every other call it synchronises the stream once (after uploading its
 * operation list) and must not be called while the stream is being captured. */
qsv_status qsv_probe_pass(qsv_ctx* ctx, int low_bits, int window_start, int transposes);

/* Testing/tuning knobs: tile_log2 in 10..14 (0 = default) forces the tile size of the fused pass
 * kernel (14 exists with one LDS plane only); defer_cnots = 1 / 0 lets qsv_apply_layers carry the
 * CNOTs whose target qubit lies outside a pass's tile by the index the pass writes each amplitude to
 * (fewer passes over the state; such passes write a second buffer taken from the workspace), or keeps
 * every CNOT a register operation (-1, the default, defers whenever the circuit has a CNOT ring, more
 * qubits than the tile has index bits, at most 28 of them, and the workspace has room for a copy of
 * the state; the result is the same up to rounding order); load_store_priority = 1 (default) / 0 makes
 * the pass kernel's wavefronts raise their issue priority while they issue a tile's loads and stores;
 * small_apply = 1 (default) / 0 lets qsv_apply_layers run states of at most 10 qubits and 2^21 amplitudes in
 * all in one launch with the gates in registers and lane exchanges (the kernel of qsv_forward_small, started
 * from the state; measured 1.6 to 4 times faster there than the fused passes, whose launches cost more than
 * their arithmetic on such states), or always takes the fused passes;
 * small_regs = 2, 3 or 4 fixes the amplitudes per thread of qsv_forward_small at 4, 8 or 16 (0, the
 * default, takes the most that still gives the chip about four wavefronts per SIMD); low_bits in 4..10 (0 = default) forces the planner's minimum number of low index bits
 * per tile; lds_planes = 1 (default) moves real and imaginary parts through one LDS plane one
 * after the other, 2 through two planes at once; naive = 1 routes qsv_apply_layers through the
 * one-gate-per-launch kernels; grad_layered = 0 makes qsv_param_shift_grad run every shifted
 * circuit whole; nt_store = 1 / 0 forces nontemporal / ordinary tile stores in the fused pass (-1,
 * the default, chooses by the size of the state); reverse_passes = 1 / 0 makes every other fused
 * pass take its tiles from the last to the first, so that it starts with what the pass before it
 * wrote last, or not (-1, the default, chooses by the size of the state; the result does not
 * depend on it); split_streams = 1 / 0 sends the state rows through a sequence of fused passes as
 * two halves, the second on a stream of the library's own that forks from and rejoins the caller's
 * stream inside the call, or not (-1, the default, is 1; it takes at least two rows and more qubits
 * than the tile has index bits; the result does not depend on it);
 * probe_layout in 0..9 (-1 = the highest) sets the register run qsv_probe_pass loads
 * and stores the tile in; grad_chunk_rows in 1..32768 (0 = as many as fit) caps the circuits per
 * launch of qsv_param_shift_grad.  Unknown names and values out of range return
 * QSV_ERR_INVALID_ARG. */
qsv_status qsv_set_option(qsv_ctx* ctx, const char* name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* QSV_H */
