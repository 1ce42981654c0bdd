// Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no HIP): the pass
// planner of the library and every entry point of the CPU oracle, each driven over a sweep of small
// cases.  tests/test_sanitizers.py compiles this file together with csrc/qsv_plan.cpp and
// oracle/qsv_oracle.cpp (two separate programs share nothing but this driver) and fails on any
// report.  The numbers themselves are checked elsewhere; here only plan invariants are asserted.
#include <complex>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#ifdef SANITIZE_PLANNER
#include "qsv_plan.h"

static int fail(const char* what, int n, int L, int tile) {
    fprintf(stderr, "planner invariant broken: %s (n=%d L=%d tile=%d)\n", what, n, L, tile);
    return 1;
}

int main() {
    using namespace qsv;
    int plans = 0;
    for (int n = 1; n <= 30; n += (n < 16 ? 1 : 3))
        for (int ent = 0; ent <= 2; ++ent)
            for (int reup = 0; reup <= 1; ++reup)
                for (int n_rot = (reup ? 0 : 1); n_rot <= 3; n_rot += 2)
                    for (int L : {0, 1, 3})
                        for (int tile : {0, kMinTile, kMaxTile})
                            for (int inverse = 0; inverse <= 1; ++inverse) {
                                qsv_circuit c{};
                                c.n_layers = L; c.reupload = reup; c.n_rot = n_rot; c.entangler = ent;
                                for (int r = 0; r < n_rot; ++r) c.rot[r] = 1 + (r + n) % 3;
                                std::string why;
                                if (!check_circuit(&c, n, &why)) return fail("check_circuit", n, L, tile);
                                for (int64_t batch : {(int64_t)1, (int64_t)3, (int64_t)64}) {
                                    if (n > 22 && batch > 1) continue;
                                    const Plan p = build_plan(c, n, batch, inverse != 0, tile, batch == 3);
                                    ++plans;
                                    if (n < kRegBits) continue;   // such states take the one-gate-per-launch path
                                    if (!p.complete) return fail("incomplete", n, L, tile);
                                    // every unitary exactly once
                                    const int want = (reup + n_rot) > 0 ? L * n : 0;
                                    if ((int)p.mat_order.size() != want) return fail("matrix count", n, L, tile);
                                    std::vector<int> seen(want ? want : 1, 0);
                                    for (int32_t m : p.mat_order) {
                                        if (m < 0 || m >= want || seen[m]++) return fail("matrix order", n, L, tile);
                                    }
                                    // operation lists: begin with a load, end with the store, stay in range
                                    for (const Pass& ps : p.passes) {
                                        if (ps.op_count < 2 || ps.op_begin < 0 ||
                                            ps.op_begin + ps.op_count > (int)p.ops.size())
                                            return fail("op range", n, L, tile);
                                        if (p.ops[ps.op_begin].kind != OP_LOAD ||
                                            p.ops[ps.op_begin + ps.op_count - 1].kind != OP_END)
                                            return fail("op framing", n, L, tile);
                                        if (ps.c < kLowBits && ps.c != ps.t) return fail("low bits", n, L, tile);
                                        if (p.ext_bits > ps.t && ps.w + (ps.t - ps.c) > p.ext_bits)
                                            return fail("window", n, L, tile);
                                    }
                                    const std::string text = describe_plan(p);
                                    if (text.empty()) return fail("describe", n, L, tile);
                                }
                            }
    // the C entry point, including a buffer that is too short and bad descriptors
    qsv_circuit c{};
    c.n_layers = 2; c.n_rot = 2; c.rot[0] = 2; c.rot[1] = 3; c.entangler = 1;
    char small[16];
    const int64_t need = qsv_plan_describe(&c, 12, 4, 0, 0, small, sizeof small);
    if (need <= 0 || small[sizeof small - 1] != 0) return fail("describe into a short buffer", 12, 2, 0);
    std::vector<char> big((size_t)need + 1);
    if (qsv_plan_describe(&c, 12, 4, 0, 0, big.data(), (int64_t)big.size()) != need) return fail("describe", 12, 2, 0);
    if (qsv_plan_describe(&c, 12, 4, 0, 0, nullptr, 0) != need) return fail("describe without buffer", 12, 2, 0);
    if (qsv_plan_describe(nullptr, 12, 4, 0, 0, nullptr, 0) != -1) return fail("null circuit", 12, 2, 0);
    if (qsv_plan_describe(&c, 12, 4, 0, 99, nullptr, 0) != -1) return fail("bad tile", 12, 2, 0);
    c.rot[1] = 7;
    if (qsv_plan_describe(&c, 12, 4, 0, 0, nullptr, 0) != -1) return fail("bad axis", 12, 2, 0);
    printf("planner: %d plans clean\n", plans);
    return 0;
}
#endif

#ifdef SANITIZE_ORACLE
typedef std::complex<double> cplx;
extern "C" {
typedef struct { int32_t n_layers, reupload, n_rot, rot[3], entangler; } oracle_circuit;
void oracle_set_threads(int t);
int64_t oracle_num_params(const oracle_circuit* c, int n);
int oracle_gate_rot(cplx* state, int64_t B, int n, int axis, int q, double theta);
int oracle_gate_cnot(cplx* state, int64_t B, int n, int ctrl, int tgt);
int oracle_gate_cz(cplx* state, int64_t B, int n, int q0, int q1);
int oracle_amp_encode(const float* x, int64_t B, int64_t dim, int n, cplx* state, double* norm_out);
int oracle_apply_layers_mode(cplx* state, int64_t B, int n, const oracle_circuit* c, const double* params,
                             const double* feats, int inverse, int mode);
void oracle_probs(const cplx* state, int64_t B, int n, double* p);
void oracle_expz_all(const cplx* state, int64_t B, int n, double* z);
int oracle_marginal(const cplx* state, int64_t B, int n, uint64_t mask, double* out);
int oracle_project_zero(cplx* state, int64_t B, int n, uint64_t mask, int renormalise, double* p0);
int oracle_fidelity(const cplx* state, int64_t B, int n, const float* x, int64_t dim, double* F);
int oracle_reset_fidelity(const cplx* state, int64_t B, int n, const oracle_circuit* c, const double* params,
                          const double* feats, uint64_t mask, const float* x, int64_t dim, double* F);
int oracle_pauli_expect(const cplx* state, int64_t B, int n, uint64_t xmask, uint64_t ymask, uint64_t zmask,
                        double* re, double* im);
int oracle_sample(const float* p32, int64_t B, int n, const double* u, int64_t shots, int64_t* out);
int oracle_param_shift_grad(const float* x, int64_t B, int64_t dim, int n, const oracle_circuit* c,
                            const double* params, const double* feats, int obs_qubit, const int64_t* subset,
                            int64_t n_subset, double* loss, double* grad);
int oracle_loss_grad(const float* x, int64_t B, int64_t dim, int n, const oracle_circuit* c, const double* params,
                     const double* feats, int kind, uint64_t mask, const double* targets, const int64_t* subset,
                     int64_t n_subset, double* loss, double* grad);
}

static double lcg(uint64_t& s) {   // inputs only: any numbers will do here
    s = s * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(s >> 11) / 9007199254740992.0;
}

int main() {
    oracle_set_threads(2);
    uint64_t seed = 12345;
    int calls = 0;
    for (int n = 1; n <= 7; ++n)
        for (int ent = 0; ent <= 2; ++ent)
            for (int reup = 0; reup <= 1; ++reup) {
                const int64_t B = 3, N = (int64_t)1 << n, dim = N > 2 ? N - 1 : N;
                oracle_circuit c{};
                c.n_layers = 2; c.reupload = reup; c.n_rot = 2; c.rot[0] = 1 + n % 3; c.rot[1] = 3; c.entangler = ent;
                const int64_t P = oracle_num_params(&c, n);
                std::vector<double> params((size_t)P), feats((size_t)(B * n)), targets((size_t)(B * n));
                for (auto& v : params) v = 6.28 * lcg(seed);
                for (auto& v : feats) v = lcg(seed) - 0.5;
                for (auto& v : targets) v = 2.0 * lcg(seed) - 1.0;
                std::vector<float> x((size_t)(B * dim));
                for (auto& v : x) v = (float)(lcg(seed) - 0.5);
                std::vector<cplx> st((size_t)(B * N));
                std::vector<double> nrm((size_t)B), p((size_t)(B * N)), z((size_t)(B * n)), F((size_t)B), re((size_t)B), im((size_t)B);
                if (oracle_amp_encode(x.data(), B, dim, n, st.data(), nrm.data())) return 1;
                for (int mode = 0; mode <= 2; ++mode) {
                    if (oracle_apply_layers_mode(st.data(), B, n, &c, params.data(), reup ? feats.data() : nullptr, 0, mode)) return 1;
                    if (oracle_apply_layers_mode(st.data(), B, n, &c, params.data(), reup ? feats.data() : nullptr, 1, mode)) return 1;
                }
                if (oracle_apply_layers_mode(st.data(), B, n, &c, params.data(), reup ? feats.data() : nullptr, 0, 0)) return 1;
                oracle_gate_rot(st.data(), B, n, 1 + n % 3, n - 1, 0.3);
                if (n >= 2) { oracle_gate_cnot(st.data(), B, n, 0, n - 1); oracle_gate_cz(st.data(), B, n, n - 1, 0); }
                oracle_probs(st.data(), B, n, p.data());
                oracle_expz_all(st.data(), B, n, z.data());
                const uint64_t mask = n >= 2 ? (((uint64_t)1 << (n - 1)) | 1u) : 1u;
                std::vector<double> marg((size_t)(B * 4));
                if (oracle_marginal(st.data(), B, n, mask, marg.data())) return 1;
                if (oracle_fidelity(st.data(), B, n, x.data(), dim, F.data())) return 1;
                if (oracle_reset_fidelity(st.data(), B, n, &c, params.data(), reup ? feats.data() : nullptr, mask, x.data(), dim, F.data())) return 1;
                const uint64_t xm = 1u, zm = n >= 2 ? 2u : 0u, ym = n >= 3 ? 4u : 0u;
                if (oracle_pauli_expect(st.data(), B, n, xm, ym, zm, re.data(), im.data())) return 1;
                std::vector<float> p32((size_t)(B * N));
                for (size_t i = 0; i < p32.size(); ++i) p32[i] = (float)p[i];
                std::vector<double> u((size_t)(B * 5));
                for (auto& v : u) v = lcg(seed);
                u[0] = 0.0; u[1] = 0x1.fffffffffffffp-1;
                std::vector<int64_t> smp((size_t)(B * 5));
                oracle_sample(p32.data(), B, n, u.data(), 5, smp.data());
                for (int64_t v : smp) if (v < 0 || v >= N) return 1;
                std::vector<cplx> proj(st);
                if (oracle_project_zero(proj.data(), B, n, mask, 1, F.data())) return 1;
                std::vector<double> loss((size_t)B), grad((size_t)(B * (P ? P : 1)));
                if (oracle_param_shift_grad(x.data(), B, dim, n, &c, params.data(), reup ? feats.data() : nullptr, n - 1,
                                            nullptr, 0, loss.data(), grad.data())) return 1;
                const int64_t subset[2] = {0, P - 1};
                if (P >= 1 && oracle_param_shift_grad(x.data(), B, dim, n, &c, params.data(), reup ? feats.data() : nullptr, 0,
                                                      subset, 2, loss.data(), grad.data())) return 1;
                if (oracle_loss_grad(x.data(), B, dim, n, &c, params.data(), reup ? feats.data() : nullptr, 1, mask, nullptr,
                                     nullptr, 0, loss.data(), grad.data())) return 1;
                if (oracle_loss_grad(x.data(), B, dim, n, &c, params.data(), reup ? feats.data() : nullptr, 2, 0, targets.data(),
                                     subset, P >= 1 ? 2 : 0, loss.data(), grad.data())) return 1;
                ++calls;
            }
    // bad arguments come back as return codes
    oracle_circuit c{};
    c.n_rot = 1; c.rot[0] = 9;
    std::vector<cplx> st(4);
    if (!oracle_apply_layers_mode(st.data(), 1, 2, &c, nullptr, nullptr, 0, 0)) return 1;
    if (!oracle_gate_cnot(st.data(), 1, 2, 1, 1)) return 1;
    printf("oracle: %d cases clean\n", calls);
    return 0;
}
#endif
