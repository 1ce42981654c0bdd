// CPU oracle for the batched state-vector path.  TEST INFRASTRUCTURE ONLY.
//
// This file is the plain definition of what the path computes, written out one gate at a time
// in complex128.  It shares no code, headers, tables or helpers with the HIP library and must
// never be called from it: only the tests, the smoke check and the benchmark's CPU-baseline leg
// load it.  There is no fusion, tiling or reordering here; every function can be checked against
// the task statement (the "north star" text and the five workload configs) by eye.
//
// Conventions (the source paper contains no circuit material, so every one of these is a stated
// reading; each is pinned by a closed form or by a dense 2^n x 2^n brute force in the CPU tests):
//   * qubit q is bit q of the amplitude index k; qubit 0 is the least-significant bit.
//   * state layout: complex128 state[B][2^n], sample-major.
//   * RX(t) = [[c,-is],[-is,c]], RY(t) = [[c,-s],[s,c]], RZ(t) = diag(e^{-it/2}, e^{+it/2}),
//     c = cos(t/2), s = sin(t/2)   (i.e. exp(-i t P / 2)).
//   * a layer = [re-upload RX(w[l][q]*feat[b][q]) on q = 0..n-1] -> each rotation slot in listed
//     order on q = 0..n-1 -> entangler.
//   * CNOT ring: for q = 0..n-1 in that order CNOT(control q, target (q+1) mod n); no gate for
//     n = 1.   CZ ladder: CZ(q, q+1) for q = 0..n-2.
//   * inverse: layers last..first; inside a layer the entangler gates in reverse order, then the
//     rotation slots in reverse order with negated angles, then the re-upload RX negated.
//   * parameters: flat index p = (l*(reupload+n_rot)+slot)*n + q; slot 0 is w when reupload = 1.
//
// Every function below is pinned by tests/test_oracle_pins.py (closed forms, truth tables,
// dense brute force for n <= 6, finite differences); none is "parity unpinned".
//
// Build: g++ -O2 -fopenmp -shared -fPIC qsv_oracle.cpp -o liboracle.so

#include <cmath>
#include <complex>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef std::complex<double> cplx;

extern "C" {

typedef struct {
    int32_t n_layers;
    int32_t reupload;
    int32_t n_rot;
    int32_t rot[3];     // 1 = RX, 2 = RY, 3 = RZ, in application order
    int32_t entangler;  // 0 none, 1 CNOT ring, 2 CZ ladder
} oracle_circuit;

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

int64_t oracle_num_params(const oracle_circuit* c, int n) {
    return (int64_t)c->n_layers * (c->reupload + c->n_rot) * n;
}

// ---------------------------------------------------------------- single gates
// One body per gate.  par != 0 splits the gate's loop over index pairs across threads (used for
// large states, one sample at a time); par == 0 runs it on the calling thread (used under a loop
// that is parallel over samples).  The pairs of one gate are disjoint and nothing is summed, so
// the numbers do not depend on par or on the thread count.
// Rotation exp(-i theta P/2) on qubit q.  axis: 1 X, 2 Y, 3 Z.
static void rot_one(cplx* a, int n, int axis, int q, double theta, int par) {
    const int64_t half = (int64_t)1 << (n - 1);
    const int64_t bit = (int64_t)1 << q;
    const double c = std::cos(0.5 * theta), s = std::sin(0.5 * theta);
    const cplx I(0.0, 1.0);
#pragma omp parallel for schedule(static) if (par)
    for (int64_t i = 0; i < half; ++i) {
        const int64_t k0 = ((i >> q) << (q + 1)) | (i & (bit - 1));
        const int64_t k1 = k0 | bit;
        const cplx v0 = a[k0], v1 = a[k1];
        if (axis == 1) {
            a[k0] = c * v0 - I * s * v1;
            a[k1] = -I * s * v0 + c * v1;
        } else if (axis == 2) {
            a[k0] = c * v0 - s * v1;
            a[k1] = s * v0 + c * v1;
        } else {
            a[k0] = cplx(c, -s) * v0;
            a[k1] = cplx(c, s) * v1;
        }
    }
}

static void cnot_one(cplx* a, int n, int ctrl, int tgt, int par) {
    const int64_t dim = (int64_t)1 << n;
    const int64_t cb = (int64_t)1 << ctrl, tb = (int64_t)1 << tgt;
#pragma omp parallel for schedule(static) if (par)
    for (int64_t k = 0; k < dim; ++k) {
        if ((k & cb) && !(k & tb)) {
            const cplx t = a[k];
            a[k] = a[k | tb];
            a[k | tb] = t;
        }
    }
}

static void cz_one(cplx* a, int n, int q0, int q1, int par) {
    const int64_t dim = (int64_t)1 << n;
    const int64_t m = ((int64_t)1 << q0) | ((int64_t)1 << q1);
#pragma omp parallel for schedule(static) if (par)
    for (int64_t k = 0; k < dim; ++k)
        if ((k & m) == m) a[k] = -a[k];
}

int oracle_gate_rot(cplx* state, int64_t B, int n, int axis, int q, double theta) {
    if (n < 1 || q < 0 || q >= n || axis < 1 || axis > 3) return 1;
    const int64_t dim = (int64_t)1 << n;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) rot_one(state + b * dim, n, axis, q, theta, 0);
    return 0;
}

int oracle_gate_cnot(cplx* state, int64_t B, int n, int ctrl, int tgt) {
    if (n < 2 || ctrl == tgt || ctrl < 0 || tgt < 0 || ctrl >= n || tgt >= n) return 1;
    const int64_t dim = (int64_t)1 << n;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) cnot_one(state + b * dim, n, ctrl, tgt, 0);
    return 0;
}

int oracle_gate_cz(cplx* state, int64_t B, int n, int q0, int q1) {
    if (n < 2 || q0 == q1 || q0 < 0 || q1 < 0 || q0 >= n || q1 >= n) return 1;
    const int64_t dim = (int64_t)1 << n;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) cz_one(state + b * dim, n, q0, q1, 0);
    return 0;
}

// ---------------------------------------------------------------- amplitude encoding
// a[k] = x[k] / ||x||_2 for k < dim, 0 above; zero vector -> all-zero state and norm 0.
int oracle_amp_encode(const float* x, int64_t B, int64_t dim, int n, cplx* state,
                      double* norm_out) {
    if (n < 1 || n > 30 || B < 1) return 1;
    const int64_t N = (int64_t)1 << n;
    if (dim < 1 || dim > N) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const float* xb = x + b * dim;
        double s = 0.0;
        for (int64_t k = 0; k < dim; ++k) s += (double)xb[k] * (double)xb[k];
        const double nrm = std::sqrt(s);
        cplx* ab = state + b * N;
        for (int64_t k = 0; k < N; ++k)
            ab[k] = (k < dim && nrm > 0.0) ? cplx((double)xb[k] / nrm, 0.0) : cplx(0.0, 0.0);
        if (norm_out) norm_out[b] = nrm;
    }
    return 0;
}

// ---------------------------------------------------------------- layered circuit
// One sample's circuit, gates applied one at a time.  par is handed to every gate (see above).
// shift_p >= 0 adds shift to the ANGLE of parameter shift_p (for a re-upload weight the angle is
// w*feat, and the shift is added to that product).
static void run_circuit(cplx* a, int n, const oracle_circuit* c, const double* params,
                        const double* feat_b, int inverse, int64_t shift_p, double shift,
                        int par) {
    const int slots = c->reupload + c->n_rot;
    auto angle = [&](int l, int slot, int q) -> double {
        const int64_t p = ((int64_t)l * slots + slot) * n + q;
        double t = params[p];
        if (c->reupload && slot == 0) t *= feat_b[q];
        if (p == shift_p) t += shift;
        return t;
    };
    auto rot = [&](int axis, int q, double t) { rot_one(a, n, axis, q, t, par); };
    auto cnot = [&](int cq, int tq) { cnot_one(a, n, cq, tq, par); };
    auto cz = [&](int q0, int q1) { cz_one(a, n, q0, q1, par); };
    if (!inverse) {
        for (int l = 0; l < c->n_layers; ++l) {
            if (c->reupload)
                for (int q = 0; q < n; ++q) rot(1, q, angle(l, 0, q));
            for (int r = 0; r < c->n_rot; ++r)
                for (int q = 0; q < n; ++q) rot(c->rot[r], q, angle(l, c->reupload + r, q));
            if (c->entangler == 1 && n >= 2)
                for (int q = 0; q < n; ++q) cnot(q, (q + 1) % n);
            if (c->entangler == 2)
                for (int q = 0; q + 1 < n; ++q) cz(q, q + 1);
        }
    } else {
        for (int l = c->n_layers - 1; l >= 0; --l) {
            if (c->entangler == 1 && n >= 2)
                for (int q = n - 1; q >= 0; --q) cnot(q, (q + 1) % n);
            if (c->entangler == 2)
                for (int q = n - 2; q >= 0; --q) cz(q, q + 1);
            for (int r = c->n_rot - 1; r >= 0; --r)
                for (int q = n - 1; q >= 0; --q) rot(c->rot[r], q, -angle(l, c->reupload + r, q));
            if (c->reupload)
                for (int q = n - 1; q >= 0; --q) rot(1, q, -angle(l, 0, q));
        }
    }
}

static int check_circuit(const oracle_circuit* c, int n) {
    if (!c || n < 1 || n > 30) return 1;
    if (c->n_layers < 0 || c->n_rot < 0 || c->n_rot > 3) return 1;
    if (c->reupload != 0 && c->reupload != 1) return 1;
    if (c->entangler < 0 || c->entangler > 2) return 1;
    for (int r = 0; r < c->n_rot; ++r)
        if (c->rot[r] < 1 || c->rot[r] > 3) return 1;
    return 0;
}

// params: double[P] (shared by the batch); feats: double[B][n] or NULL when reupload = 0.
// mode chooses how the work is spread over threads, never what is computed: 1 = one thread per
// sample, every gate on that thread; 2 = the samples one by one, every gate's pair loop split
// across threads; 0 = mode 2 for n >= 18 (few, large states), else mode 1.
int oracle_apply_layers_mode(cplx* state, int64_t B, int n, const oracle_circuit* c,
                             const double* params, const double* feats, int inverse, int mode) {
    if (check_circuit(c, n) || B < 1) return 1;
    if (c->reupload && !feats) return 1;
    if (mode < 0 || mode > 2) return 1;
    const int64_t N = (int64_t)1 << n;
    const bool pairs = mode == 2 || (mode == 0 && n >= 18);
    if (pairs) {
        for (int64_t b = 0; b < B; ++b)
            run_circuit(state + b * N, n, c, params, feats ? feats + b * n : nullptr, inverse, -1,
                        0.0, 1);
    } else {
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t b = 0; b < B; ++b)
            run_circuit(state + b * N, n, c, params, feats ? feats + b * n : nullptr, inverse, -1,
                        0.0, 0);
    }
    return 0;
}

int oracle_apply_layers(cplx* state, int64_t B, int n, const oracle_circuit* c,
                        const double* params, const double* feats, int inverse) {
    return oracle_apply_layers_mode(state, B, n, c, params, feats, inverse, 0);
}

// ---------------------------------------------------------------- measurement
// p[b][k] = |a[b][k]|^2
void oracle_probs(const cplx* state, int64_t B, int n, double* p) {
    const int64_t tot = B << n;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < tot; ++i) p[i] = std::norm(state[i]);
}

// z[b][q] = sum_k (1 - 2*bit_q(k)) |a[b][k]|^2
void oracle_expz_all(const cplx* state, int64_t B, int n, double* z) {
    const int64_t N = (int64_t)1 << n;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int q = 0; q < n; ++q) {
            double s = 0.0;
            for (int64_t k = 0; k < N; ++k) {
                const double p = std::norm(state[b * N + k]);
                s += ((k >> q) & 1) ? -p : p;
            }
            z[b * n + q] = s;
        }
    }
}

static int64_t extract_bits(int64_t k, uint64_t mask) {  // gather the mask bits of k, LSB first
    int64_t v = 0;
    int j = 0;
    for (int q = 0; q < 64; ++q)
        if ((mask >> q) & 1) {
            v |= ((k >> q) & 1) << j;
            ++j;
        }
    return v;
}

static int popcount64(uint64_t m) {
    int c = 0;
    while (m) { c += (int)(m & 1); m >>= 1; }
    return c;
}

// out[b][v] = P(the mask qubits read v), v built from the mask qubits in ascending order
// (lowest mask qubit = bit 0 of v).
int oracle_marginal(const cplx* state, int64_t B, int n, uint64_t mask, double* out) {
    if (mask == 0 || (n < 64 && (mask >> n) != 0)) return 1;
    const int m = popcount64(mask);
    const int64_t N = (int64_t)1 << n, M = (int64_t)1 << m;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t v = 0; v < M; ++v) out[b * M + v] = 0.0;
        for (int64_t k = 0; k < N; ++k)
            out[b * M + extract_bits(k, mask)] += std::norm(state[b * N + k]);
    }
    return 0;
}

// p0[b] = P(all mask qubits read 0); then a[k] = 0 where k & mask != 0, and, when renormalise is
// set, the kept amplitudes are divided by sqrt(p0).  p0 = 0 with renormalise leaves a zero state.
int oracle_project_zero(cplx* state, int64_t B, int n, uint64_t mask, int renormalise,
                        double* p0) {
    if (mask == 0 || (n < 64 && (mask >> n) != 0)) return 1;
    const int64_t N = (int64_t)1 << n;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        cplx* a = state + b * N;
        double s = 0.0;
        for (int64_t k = 0; k < N; ++k)
            if (((uint64_t)k & mask) == 0) s += std::norm(a[k]);
        const double scale = renormalise ? (s > 0.0 ? 1.0 / std::sqrt(s) : 0.0) : 1.0;
        for (int64_t k = 0; k < N; ++k)
            a[k] = (((uint64_t)k & mask) == 0) ? a[k] * scale : cplx(0.0, 0.0);
        if (p0) p0[b] = s;
    }
    return 0;
}

// F[b] = | sum_k conj(ain[k]) a[k] |^2 with ain = x_b / ||x_b|| (zero-padded, real).
int oracle_fidelity(const cplx* state, int64_t B, int n, const float* x, int64_t dim, double* F) {
    const int64_t N = (int64_t)1 << n;
    if (dim < 1 || dim > N) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        double s = 0.0;
        cplx acc(0.0, 0.0);
        for (int64_t k = 0; k < dim; ++k) {
            const double xv = (double)x[b * dim + k];
            s += xv * xv;
            acc += xv * state[b * N + k];
        }
        F[b] = s > 0.0 ? std::norm(acc) / s : 0.0;
    }
    return 0;
}

// ---------------------------------------------------------------- trash reset
// Fidelity of an autoencoder whose trash qubits are really reset to |0> (task statement, workload
// config 3: "trash-qubit probability ..., decoder, fidelity"; the reset is the physical operation
// the projection onto trash = 0 stands in for).  Measuring the trash qubits gives outcome t with the
// unnormalised conditional state psi_t on the other qubits; after the reset the register holds
// psi_t (x) |0..0>.  With D the circuit c run in inverse mode (the decoder),
//   F[b] = sum_t | <a_in,b| D ( psi_t (x) |0> ) |^2,   a_in = x_b / ||x_b||,
// which is <a_in| D rho D^dagger |a_in> for the reset (mixed) state rho.  state is not modified.
int oracle_reset_fidelity(const cplx* state, int64_t B, int n, const oracle_circuit* c,
                          const double* params, const double* feats, uint64_t mask, const float* x,
                          int64_t dim, double* F) {
    if (check_circuit(c, n) || B < 1) return 1;
    if (c->reupload && !feats) return 1;
    if (mask == 0 || (n < 64 && (mask >> n) != 0)) return 1;
    const int64_t N = (int64_t)1 << n;
    if (dim < 1 || dim > N) return 1;
    int m = 0;
    for (int q = 0; q < n; ++q) m += (int)((mask >> q) & 1);
    if (m > 20) return 1;
    for (int64_t b = 0; b < B; ++b) {
        std::vector<cplx> work((size_t)N);
        const double* fb = feats ? feats + b * n : nullptr;
        double total = 0.0;
        for (int64_t t = 0; t < ((int64_t)1 << m); ++t) {
            // spread the bits of t over the mask positions
            uint64_t tbits = 0;
            int j = 0;
            for (int q = 0; q < n; ++q)
                if ((mask >> q) & 1) { if ((t >> j) & 1) tbits |= (uint64_t)1 << q; ++j; }
            for (int64_t k = 0; k < N; ++k)
                work[k] = (((uint64_t)k & mask) == 0) ? state[b * N + (k | (int64_t)tbits)] : cplx(0.0, 0.0);
            run_circuit(work.data(), n, c, params, fb, 1, -1, 0.0, 0);
            double Ft = 0.0;
            oracle_fidelity(work.data(), 1, n, x + b * dim, dim, &Ft);
            total += Ft;
        }
        F[b] = total;
    }
    return 0;
}

// ---------------------------------------------------------------- Pauli strings
// E[b] = <a_b| P |a_b> for P = product over qubits of X (bit in xmask), Y (ymask) or Z (zmask);
// the masks must not overlap.  Written as the definition: copy the state, apply the one-qubit
// Pauli matrices one qubit at a time (X: swap the pair; Y: (a0, a1) -> (-i a1, i a0); Z: negate a1),
// then take the inner product with the original.  The result of a Hermitian operator is real; the
// imaginary part is returned too so that tests can see it vanish.
int oracle_pauli_expect(const cplx* state, int64_t B, int n, uint64_t xmask, uint64_t ymask,
                        uint64_t zmask, double* re, double* im) {
    if ((xmask & ymask) || (xmask & zmask) || (ymask & zmask)) return 1;
    if (n < 64 && ((xmask | ymask | zmask) >> n)) return 1;
    const int64_t N = (int64_t)1 << n;
    const cplx I(0.0, 1.0);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        std::vector<cplx> w(state + b * N, state + (b + 1) * N);
        for (int q = 0; q < n; ++q) {
            const int64_t bit = (int64_t)1 << q;
            const bool X = (xmask >> q) & 1, Y = (ymask >> q) & 1, Z = (zmask >> q) & 1;
            if (!X && !Y && !Z) continue;
            for (int64_t k0 = 0; k0 < N; ++k0) {
                if (k0 & bit) continue;
                const int64_t k1 = k0 | bit;
                const cplx a0 = w[k0], a1 = w[k1];
                if (X) { w[k0] = a1; w[k1] = a0; }
                else if (Y) { w[k0] = -I * a1; w[k1] = I * a0; }
                else { w[k1] = -a1; }
            }
        }
        cplx acc(0.0, 0.0);
        for (int64_t k = 0; k < N; ++k) acc += std::conj(state[b * N + k]) * w[k];
        re[b] = acc.real();
        if (im) im[b] = acc.imag();
    }
    return 0;
}

// ---------------------------------------------------------------- sampling
// Integer inverse CDF over a float32 probability vector:
//   w_k = floor(double(p32_k) * 2^60)            (exact: a float times a power of two)
//   W_k = w_0 + ... + w_k                        (uint64)
//   r   = floor(u * 2^53)                        (exact for u in [0,1))
//   t   = floor(r * W_last / 2^53)               (128-bit product)
//   sample = smallest k with W_k > t
// W_last = 0 gives -1 for every shot and return code 3.
int oracle_sample(const float* p32, int64_t B, int n, const double* u, int64_t shots,
                  int64_t* out) {
    const int64_t N = (int64_t)1 << n;
    int rc = 0;
    std::vector<uint64_t> W((size_t)N);
    for (int64_t b = 0; b < B; ++b) {
        uint64_t acc = 0;
        for (int64_t k = 0; k < N; ++k) {
            const double pk = (double)p32[b * N + k];
            const uint64_t w = pk > 0.0 ? (uint64_t)std::floor(std::ldexp(pk, 60)) : 0;
            acc += w;
            W[(size_t)k] = acc;
        }
        for (int64_t s = 0; s < shots; ++s) {
            if (acc == 0) { out[b * shots + s] = -1; rc = 3; continue; }
            const uint64_t r = (uint64_t)std::floor(std::ldexp(u[b * shots + s], 53));
            const unsigned __int128 prod = (unsigned __int128)r * (unsigned __int128)acc;
            const uint64_t t = (uint64_t)(prod >> 53);
            int64_t lo = 0, hi = N - 1;  // smallest k with W[k] > t
            while (lo < hi) {
                const int64_t mid = lo + (hi - lo) / 2;
                if (W[(size_t)mid] > t) hi = mid; else lo = mid + 1;
            }
            out[b * shots + s] = lo;
        }
    }
    return rc;
}

// ---------------------------------------------------------------- parameter-shift gradient
// f_b(theta) = <Z_obs> after encode + circuit.  For every listed parameter p:
//   g[b][j] = 1/2 [ f_b(angle_p + pi/2) - f_b(angle_p - pi/2) ]     (x feat_b[q] for a re-upload
//   weight, by the chain rule, since the shifted angle is w*feat).
// subset == NULL means all P parameters (then n_subset is ignored); grad is [B][n_listed].
static double expz_one(const cplx* a, int n, int q) {
    const int64_t N = (int64_t)1 << n;
    double s = 0.0;
    for (int64_t k = 0; k < N; ++k) {
        const double p = std::norm(a[k]);
        s += ((k >> q) & 1) ? -p : p;
    }
    return s;
}

int oracle_param_shift_grad(const float* x, int64_t B, int64_t dim, int n, const oracle_circuit* c,
                            const double* params, const double* feats, int obs_qubit,
                            const int64_t* subset, int64_t n_subset, double* loss, double* grad) {
    if (check_circuit(c, n) || B < 1 || obs_qubit < 0 || obs_qubit >= n) return 1;
    if (c->reupload && !feats) return 1;
    const int64_t N = (int64_t)1 << n;
    if (dim < 1 || dim > N) return 1;
    const int64_t P = oracle_num_params(c, n);
    const int64_t nl = subset ? n_subset : P;
    if (subset)
        for (int64_t j = 0; j < n_subset; ++j)
            if (subset[j] < 0 || subset[j] >= P) return 1;
    const int slots = c->reupload + c->n_rot;
    const double half_pi = 1.57079632679489661923;
    const int64_t jobs = B * (nl + 1);
#pragma omp parallel
    {
        std::vector<cplx> enc((size_t)N), work((size_t)N);
#pragma omp for schedule(dynamic, 1)
        for (int64_t job = 0; job < jobs; ++job) {
            const int64_t b = job / (nl + 1), j = job % (nl + 1);
            double nrm = 0.0;
            oracle_amp_encode(x + b * dim, 1, dim, n, enc.data(), &nrm);
            const double* fb = feats ? feats + b * n : nullptr;
            if (j == nl) {
                work = enc;
                run_circuit(work.data(), n, c, params, fb, 0, -1, 0.0, 0);
                if (loss) loss[b] = expz_one(work.data(), n, obs_qubit);
                continue;
            }
            const int64_t p = subset ? subset[j] : j;
            work = enc;
            run_circuit(work.data(), n, c, params, fb, 0, p, +half_pi, 0);
            const double fp = expz_one(work.data(), n, obs_qubit);
            work = enc;
            run_circuit(work.data(), n, c, params, fb, 0, p, -half_pi, 0);
            const double fm = expz_one(work.data(), n, obs_qubit);
            double g = 0.5 * (fp - fm);
            const int slot = (int)((p / n) % slots);
            if (c->reupload && slot == 0) g *= fb[p % n];
            grad[b * nl + j] = g;
        }
    }
    return 0;
}

// ------------------------------------------------------------------------------------------------
// Training losses and their gradients (task statement: "measurement (... trash-qubit marginal ...)"
// and "parameter-shift gradients over the batch"; the two losses are the ones the workload configs
// describe: an autoencoder that empties its trash qubits, and a regression of <Z_q> on targets).
//   kind 1 (trash):  loss_b = 1 - P0_b,  P0 = probability that every qubit of mask reads 0.
//                    P0 is the expectation of a projector, so the shift rule applies to it:
//                    g = -1/2 [ P0(+) - P0(-) ].
//   kind 2 (mse_z):  loss_b = 1/n sum_q ( <Z_q>_b - y[b][q] )^2.  Chain rule over the shift rule of
//                    each <Z_q>:  g = 2/n sum_q ( <Z_q> - y ) 1/2 [ <Z_q>(+) - <Z_q>(-) ].
// Re-upload weights get the factor feat_b[q] as in oracle_param_shift_grad.  subset as there.
static double prob_mask_zero(const cplx* a, int n, uint64_t mask) {
    const int64_t N = (int64_t)1 << n;
    double s = 0.0;
    for (int64_t k = 0; k < N; ++k)
        if (((uint64_t)k & mask) == 0) s += std::norm(a[k]);
    return s;
}

static void expz_vec(const cplx* a, int n, double* z) {
    for (int q = 0; q < n; ++q) z[q] = expz_one(a, n, q);
}

int oracle_loss_grad(const float* x, int64_t B, int64_t dim, int n, const oracle_circuit* c,
                     const double* params, const double* feats, int kind, uint64_t mask,
                     const double* targets, const int64_t* subset, int64_t n_subset, double* loss,
                     double* grad) {
    if (check_circuit(c, n) || B < 1) return 1;
    if (c->reupload && !feats) return 1;
    if (kind == 1) { if (mask == 0 || (n < 64 && (mask >> n) != 0)) return 1; }
    else if (kind == 2) { if (!targets) return 1; }
    else return 1;
    const int64_t N = (int64_t)1 << n;
    if (dim < 1 || dim > N) return 1;
    const int64_t P = oracle_num_params(c, n);
    const int64_t nl = subset ? n_subset : P;
    if (subset)
        for (int64_t j = 0; j < n_subset; ++j)
            if (subset[j] < 0 || subset[j] >= P) return 1;
    const int slots = c->reupload + c->n_rot;
    const double half_pi = 1.57079632679489661923;
    for (int64_t b = 0; b < B; ++b) {
        std::vector<cplx> enc((size_t)N), work((size_t)N);
        std::vector<double> z0(n), zp(n), zm(n);
        double nrm = 0.0;
        oracle_amp_encode(x + b * dim, 1, dim, n, enc.data(), &nrm);
        const double* fb = feats ? feats + b * n : nullptr;
        const double* yb = targets ? targets + b * n : nullptr;
        work = enc;
        run_circuit(work.data(), n, c, params, fb, 0, -1, 0.0, 0);
        if (kind == 1) {
            if (loss) loss[b] = 1.0 - prob_mask_zero(work.data(), n, mask);
        } else {
            expz_vec(work.data(), n, z0.data());
            double acc = 0.0;
            for (int q = 0; q < n; ++q) acc += (z0[q] - yb[q]) * (z0[q] - yb[q]);
            if (loss) loss[b] = acc / n;
        }
        for (int64_t j = 0; j < nl; ++j) {
            const int64_t p = subset ? subset[j] : j;
            double g;
            if (kind == 1) {
                work = enc;
                run_circuit(work.data(), n, c, params, fb, 0, p, +half_pi, 0);
                const double fp = prob_mask_zero(work.data(), n, mask);
                work = enc;
                run_circuit(work.data(), n, c, params, fb, 0, p, -half_pi, 0);
                const double fm = prob_mask_zero(work.data(), n, mask);
                g = -0.5 * (fp - fm);
            } else {
                work = enc;
                run_circuit(work.data(), n, c, params, fb, 0, p, +half_pi, 0);
                expz_vec(work.data(), n, zp.data());
                work = enc;
                run_circuit(work.data(), n, c, params, fb, 0, p, -half_pi, 0);
                expz_vec(work.data(), n, zm.data());
                g = 0.0;
                for (int q = 0; q < n; ++q) g += (z0[q] - yb[q]) * 0.5 * (zp[q] - zm[q]);
                g *= 2.0 / n;
            }
            const int slot = (int)((p / n) % slots);
            if (c->reupload && slot == 0) g *= fb[p % n];
            grad[b * nl + j] = g;
        }
    }
    return 0;
}

}  // extern "C"
