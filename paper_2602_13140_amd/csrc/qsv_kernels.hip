// HIP kernels for gfx950 (CDNA4): fused gate passes, encoding, measurement, sampling, gradient
// assembly.  64-wide wavefronts throughout.  No code is shared with the CPU oracle.
#include "qsv_kernels.h"
#include "qsv_gate_asm.h"

#include <mutex>

namespace qsv {

namespace {

constexpr int R = kRegBits;
constexpr int NR = 1 << R;
constexpr int CHUNK_BITS = 12;            // reduction kernels: 256 threads x 16 elements
constexpr int CHUNK = 1 << CHUNK_BITS;

typedef unsigned long long u64;

__device__ __forceinline__ float prob32(float2 a) {
    // one fixed rounding sequence so that every kernel that needs p32 gets the same bits: re * re
    // rounded, then one fused multiply-add (written out: a plain sum of two products leaves the
    // compiler free to fuse either product, differently from kernel to kernel)
    return __builtin_fmaf(a.y, a.y, a.x * a.x);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Reduction kernels run one block per (chunk of a row, row): the chunk in grid.x, the row spread over
// grid.y and grid.z (a grid dimension other than x holds at most 65535 blocks).
__device__ __forceinline__ unsigned long long grid_row() {
    return (unsigned long long)blockIdx.z * gridDim.y + blockIdx.y;
}

// Sum over a 256-thread block; result valid in thread 0.  sm: 4 doubles.
__device__ __forceinline__ double block_sum256(double v, double* sm) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[w] = v;
    __syncthreads();
    return sm[0] + sm[1] + sm[2] + sm[3];
}

// ------------------------------------------------------------------------------------------
// Row mapping (plain: row = sample; gradient: row -> (sample, shifted parameter)).
struct RowCtx {
    u64 sample;
    int ovr_id;     // matrix id replaced by the shifted matrix, or -1
    u64 ovr_off;    // float offset of that matrix inside the shifted table (per-sample part added by caller)
};

__device__ __forceinline__ RowCtx row_ctx(const RowMap& rm, u64 row) {
    RowCtx rc;
    rc.sample = row;
    rc.ovr_id = -1;
    rc.ovr_off = 0;
    if (rm.grad) {
        const u64 gid = (u64)rm.row0 + row;
        const u64 per = (u64)rm.per;
        rc.sample = gid / per;
        const int v = (int)(gid % per);
        if (v < rm.two_p) {
            const int p = v >> 1;
            const int l = p / rm.slots_n;
            const int q = p % rm.n;
            rc.ovr_id = l * rm.n + q;
            rc.ovr_off = (u64)v * 8;
        }
    }
    return rc;
}

// ------------------------------------------------------------------------------------------
// Fused pass kernel.
//
// Tile-local index tau (T bits) <-> extended index e: e = tile_base | (tau & (2^c-1)) |
// ((tau >> c) << w).  In layout s a lane holds the 16 amplitudes tau = thr_part | (i << s),
// i = 0..15, where thr_part spreads the thread index over the other T-4 bits.


// One 2x2 complex matrix times one amplitude pair, in place.  (a,b) = (re,im) of the amplitude
// whose target bit is 0, (c,d) of the one whose bit is 1; m = (m00r,m00i,m01r,m01i,m10r,m10i,m11r,
// m11i).  Written as one asm block with tied operands so that the 32 amplitude registers never
// move: four interleaved accumulation chains whose last step overwrites an input that is dead by
// then.  16 VALU instructions per pair, none of them a copy.  Used where the matrix differs per lane;
// matrices shared by a wavefront are applied inside the interpreter.
#define QSV_U_PAIR_BODY                      \
    "v_mul_f32 %4, %8, %0\n\t"               \
    "v_mul_f32 %5, %9, %0\n\t"               \
    "v_mul_f32 %6, %12, %0\n\t"              \
    "v_mul_f32 %7, %13, %0\n\t"              \
    "v_fma_f32 %4, -%9, %1, %4\n\t"          \
    "v_fma_f32 %5, %8, %1, %5\n\t"           \
    "v_fma_f32 %6, -%13, %1, %6\n\t"         \
    "v_fma_f32 %7, %12, %1, %7\n\t"          \
    "v_fma_f32 %4, %10, %2, %4\n\t"          \
    "v_fma_f32 %5, %11, %2, %5\n\t"          \
    "v_fma_f32 %6, %14, %2, %6\n\t"          \
    "v_fma_f32 %7, %15, %2, %7\n\t"          \
    "v_fma_f32 %0, -%11, %3, %4\n\t"         \
    "v_fma_f32 %1, %10, %3, %5\n\t"          \
    "v_fma_f32 %2, -%15, %3, %6\n\t"         \
    "v_fma_f32 %3, %14, %3, %7\n\t"

// matrix in vector registers (differs per lane: several state rows share a tile)
__device__ __forceinline__ void u_pair_v(float& a, float& b, float& c, float& d, const float (&m)[8]) {
    float t0, t1, t2, t3;
    asm volatile(QSV_U_PAIR_BODY
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
                 : "v"(m[0]), "v"(m[1]), "v"(m[2]), "v"(m[3]), "v"(m[4]), "v"(m[5]), "v"(m[6]), "v"(m[7]));
}

template <int J>
__device__ __forceinline__ void apply_u(float (&vr)[NR], float (&vi)[NR], const float (&m)[8]) {
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        if (i & (1 << J)) continue;
        const int i1 = i | (1 << J);
        u_pair_v(vr[i], vi[i], vr[i1], vi[i1], m);
    }
}

__device__ __forceinline__ void apply_u_any(int j, float (&vr)[NR], float (&vi)[NR], const float (&m)[8]) {
    switch (j) {
        case 0: apply_u<0>(vr, vi, m); break;
        case 1: apply_u<1>(vr, vi, m); break;
        case 2: apply_u<2>(vr, vi, m); break;
        default: apply_u<3>(vr, vi, m); break;
    }
}

// constant-address-space views: uniform loads through them become scalar loads
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(4))) u32x2* cuint2_p;
typedef const __attribute__((address_space(4))) f32x4* cfloat4_p;

// A value that is certainly held in a scalar register (an "s" input constraint alone is not
// enough: the compiler may hand a vector register to the asm).
__device__ __forceinline__ unsigned to_sgpr(unsigned v) {
    unsigned r;
    // The compiler cannot see into the asm, so it does not pad the one wait state this chip needs
    // between a vector write of a register and a readfirstlane of it; s_nop covers it.
    asm volatile("s_nop 4\n\tv_readfirstlane_b32 %0, %1\n\ts_nop 1" : "=s"(r) : "v"(v));
    return r;
}

// The 16 amplitudes of a lane live in 32 separately named scalars (vr0..vr15, vi0..vi15): as an
// array the compiler turns them into one 16-wide vector value and copies the whole tuple around
// the asm block.  QSV_16 applies a statement macro to every index.
#define QSV_16(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)
// The same 16 indices in Gray-code order, with the register bit that changes on the way in and the
// direction (+: the bit turns on): X(k, bit, sign).  The address of element k of a tile then follows
// from the previous one by adding or subtracting one of four strides, two scalar instructions
// instead of the nine it takes to build it from k (scalar instructions compete with the vector
// ones for issue slots).  The walk starts from "element 0 minus stride 0".
#define QSV_16G(X) X(0, 0, +) X(1, 0, +) X(3, 1, +) X(2, 0, -) X(6, 2, +) X(7, 0, +) X(5, 1, -) X(4, 0, -) \
                   X(12, 3, +) X(13, 0, +) X(15, 1, +) X(14, 0, -) X(10, 2, -) X(11, 0, +) X(9, 1, -) X(8, 0, -)
#define QSV_DECL(k) float vr##k, vi##k;
#define QSV_RV(k) [r##k] "+v"(vr##k), [i##k] "+v"(vi##k),

// Byte offsets of register elements 1, 2, 4, 8 in layout s inside an LDS plane, as XORed onto the
// lane's own address part: swz(k << s) * 4 with swz(x) = x ^ ((x >> 4) & 31).  swz is linear over
// XOR, so the offset of any element is the XOR of the offsets of its set bits.  One 16-byte row per
// layout.
struct XpOffsets {
    unsigned v[12][4];
    constexpr XpOffsets() : v() {
        for (int s = 0; s < 12; ++s)
            for (int j = 0; j < 4; ++j) {
                const unsigned x = (1u << j) << s;
                v[s][j] = (x ^ ((x >> 4) & 31u)) * 4u;
            }
    }
};
__device__ __attribute__((aligned(64))) const XpOffsets k_xp_tab = XpOffsets();
#define k_xp_off k_xp_tab.v

// PERLANE = true is the variant for tiles that hold several state rows (n < T): it adds the
// per-lane-matrix path; the main variant keeps its operation loop minimal.
//
// Structure of a pass: the first operation loads the tile; the assembly interpreter then runs
// gates, sign flips and LDS transposes in place until it meets an operation it does not handle
// (a per-lane unitary, or the end), which the C++ loop handles before re-entering it.
template <int T, bool PERLANE, int PLANES>
// 96 scalar registers (the interpreter pins 37 of them) allow eight wavefronts per SIMD; the main
// variant needs no scalar spills for that (the per-lane-matrix variant has some, and is limited by
// its vector registers anyway).
__global__ __launch_bounds__(1 << (T - R)) __attribute__((amdgpu_num_sgpr(96)))
void k_pass(const PassArgs a) {
    // PLANES XOR-swizzled planes of 2^T floats each (real and imaginary parts at once, or one
    // after the other through a single plane, which halves the LDS a workgroup holds); see the
    // interpreter's generator.  The segment must start at LDS byte 0 (no static LDS here).
    extern __shared__ float lds[];
    // A workgroup that has just started shares its SIMDs with up to seven older ones in the middle of
    // their gates; the sooner its loads are on their way, the more of their latency those gates hide.
    if (a.prio) __builtin_amdgcn_s_setprio(3);
    constexpr unsigned PLANE = 1u << T;
    static_assert(PLANES == 1 || (PLANE * 4u < 65536u && PLANE / 64u < 256u),
                  "with two planes the second plane is reached through the LDS offset fields");
    const unsigned lds_byte0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)lds;
    const unsigned thr = threadIdx.x;
    const u64 tb = a.rev ? (u64)(gridDim.x - 1u - blockIdx.x) : (u64)blockIdx.x;
    const int c = a.c, w = a.w;
    const unsigned cmask = (1u << c) - 1u;
    const int wc = w - c;
    const u64 tile_base = ((tb & ((1ull << wc) - 1ull)) << c) | ((tb >> wc) << (w + T - c));
    auto expand = [&](unsigned tau) -> u64 {
        return (u64)(tau & cmask) | ((u64)(tau >> c) << w);
    };
    if (tile_base >= a.total) return;  // padding tile (batch not a power of two): nothing to do
    if (lds_byte0 != 0) return;        // cannot happen; the swizzled addressing relies on it
    // every element of the tile in range? (false only for the last tile of a ragged batch)
    const bool full = (tile_base | expand((1u << T) - 1u)) < a.total;
    // tiles never straddle a state row unless T > n, in which case rows are per lane
    const bool rows_uniform = !PERLANE;
    const RowCtx urc = row_ctx(a.rm, tile_base >> a.n);
    // scalar operands of the interpreter
    const u64 mbase = (u64)(uintptr_t)(a.mats + (a.rowdep && rows_uniform ? urc.sample * (u64)a.n_mats * 8 : 0));
    const u64 ovrp = (u64)(uintptr_t)(a.ovr + (a.rowdep && rows_uniform ? urc.sample * (u64)a.rm.two_p * 8 : 0) + urc.ovr_off);
    const unsigned mlo = to_sgpr((unsigned)mbase), mhi = to_sgpr((unsigned)(mbase >> 32));
    const unsigned olo = to_sgpr((unsigned)ovrp), ohi = to_sgpr((unsigned)(ovrp >> 32));
    // unitaries are numbered in execution order; exec_of maps (layer, qubit) ids to that order
    const unsigned ovr_id = to_sgpr((unsigned)((rows_uniform && urc.ovr_id >= 0) ? a.exec_of[urc.ovr_id] : -1));
    const unsigned nonuni = to_sgpr(rows_uniform ? 0u : 1u);
    const unsigned sc_c = to_sgpr((unsigned)c), sc_w = to_sgpr((unsigned)w), sc_cmask = to_sgpr(cmask);
    const unsigned tblo = to_sgpr((unsigned)tile_base), tbhi = to_sgpr((unsigned)(tile_base >> 32));
    const u64 tab = (u64)(uintptr_t)&k_xp_off[0][0];
    const unsigned tablo = to_sgpr((unsigned)tab), tabhi = to_sgpr((unsigned)(tab >> 32));
    unsigned opslo = to_sgpr((unsigned)(uintptr_t)a.ops), opshi = to_sgpr((unsigned)((u64)(uintptr_t)a.ops >> 32));

    QSV_16(QSV_DECL)
    // ---- first operation: load the tile in layout s (register run at tile bits s..s+3)
    const u32x2 first = *(cuint2_p)(uintptr_t)a.ops;
    unsigned scur = to_sgpr((first.x >> 8) & 0xffu);
    const unsigned tau0 = ((thr >> scur) << (scur + R)) | (thr & ((1u << scur) - 1u));
    u64 e0 = tile_base | expand(tau0);
    // A tile's index bits span less than 2^29 elements unless n > 28: then an element's address is
    // a scalar base (tile and register part) plus one 32-bit per-lane byte offset, which costs no
    // vector arithmetic per element.
    const bool off32 = (expand((1u << T) - 1u) >> 29) == 0;
    // Where the tile is read from: the state itself, or (first pass of a gradient chunk, rows
    // uniform per tile) the kept start state of the row's sample, so that no copy pass is needed.
    const float2* ld = a.in;
    if (a.src && rows_uniform) {
        const u64 d = (u64)(((long long)urc.sample - (long long)(tile_base >> a.n)) << a.n);
        const long long ds = (long long)(((u64)to_sgpr((unsigned)(d >> 32)) << 32) | to_sgpr((unsigned)d));
        ld = a.src + ds;
    }
    if (full && off32 && ld == a.in) {
        // the common case, written against the kernel argument itself: the compiler then keeps the
        // per-element base in scalar registers and spends no vector arithmetic on addresses
        const unsigned lane_byte = (unsigned)expand(tau0) * 8u;
        const u64 st0 = expand(1u << scur) * 8u, st1 = expand(2u << scur) * 8u, st2 = expand(4u << scur) * 8u,
                  st3 = expand(8u << scur) * 8u;
        const char* bp = (const char*)(a.in + tile_base) - st0;
#define QSV_LD(k, bit, sign) { bp = bp sign st##bit; \
                    const float2 v = *(const float2*)(bp + lane_byte); vr##k = v.x; vi##k = v.y; }
        QSV_16G(QSV_LD)
#undef QSV_LD
    } else if (full && off32) {
        const unsigned lane_byte = (unsigned)expand(tau0) * 8u;
#define QSV_LD(k) { const char* bp = (const char*)(ld + (tile_base | expand((unsigned)k << scur))); \
                    const float2 v = *(const float2*)(bp + lane_byte); vr##k = v.x; vi##k = v.y; }
        QSV_16(QSV_LD)
#undef QSV_LD
    } else if (full) {
#define QSV_LD(k) { const float2 v = ld[e0 | expand((unsigned)k << scur)]; vr##k = v.x; vi##k = v.y; }
        QSV_16(QSV_LD)
#undef QSV_LD
    } else {
#define QSV_LD(k) { const u64 e = e0 | expand((unsigned)k << scur); const float2 v = ld[e < a.total ? e : tile_base]; \
                    vr##k = e < a.total ? v.x : 0.f; vi##k = e < a.total ? v.y : 0.f; }
        QSV_16(QSV_LD)
#undef QSV_LD
    }
    { const u64 nx = (u64)(uintptr_t)a.ops + 8; opslo = to_sgpr((unsigned)nx); opshi = to_sgpr((unsigned)(nx >> 32)); }
    if (a.prio) __builtin_amdgcn_s_setprio(0);
    unsigned e0lo = (unsigned)e0, e0hi = (unsigned)(e0 >> 32);
    unsigned ldsb = (tau0 ^ ((tau0 >> 4) & 31u)) * 4u;

    for (;;) {
        {
            float t0, t1, t2, t3, tc, m0, m1, m2, m3, m4, m5, m6, m7;
            unsigned ba0, ba1, ba2, ba3, bb0, bb1, bb2, bb3;
#define QSV_LOOP_OUT QSV_16(QSV_RV) [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2),                 \
                     [t3] "=&v"(t3), [tc] "=&v"(tc), [m0] "=&v"(m0), [m1] "=&v"(m1), [m2] "=&v"(m2), \
                     [m3] "=&v"(m3), [m4] "=&v"(m4), [m5] "=&v"(m5), [m6] "=&v"(m6), [m7] "=&v"(m7), \
                     [ba0] "=&v"(ba0), [ba1] "=&v"(ba1), [ba2] "=&v"(ba2), [ba3] "=&v"(ba3),       \
                     [bb0] "=&v"(bb0), [bb1] "=&v"(bb1), [bb2] "=&v"(bb2), [bb3] "=&v"(bb3),       \
                     [opslo] "+s"(opslo), [opshi] "+s"(opshi),                                     \
                     [scur] "+s"(scur), [ldsb] "+v"(ldsb), [e0lo] "+v"(e0lo), [e0hi] "+v"(e0hi)
#define QSV_LOOP_IN [mlo] "s"(mlo), [mhi] "s"(mhi), [olo] "s"(olo), [ohi] "s"(ohi),                 \
                    [ovrid] "s"(ovr_id), [nonuni] "s"(nonuni), [thr] "v"(thr), [c] "s"(sc_c),       \
                    [w] "s"(sc_w), [cmask] "s"(sc_cmask), [tblo] "s"(tblo), [tbhi] "s"(tbhi),       \
                    [tablo] "s"(tablo), [tabhi] "s"(tabhi)
            // four texts: two or one LDS plane, and whether a unitary may have to be left to the C++
            // code below (several state rows per tile with row-dependent matrices)
            if constexpr (PLANES == 2 && PERLANE) {
                asm volatile(QSV_GATE_LOOP_ASM_2P_ROWS
                             : QSV_LOOP_OUT
                             : QSV_LOOP_IN, [plane4] "n"(PLANE * 4u), [pl64] "n"(PLANE / 64u)
                             : QSV_GATE_LOOP_CLOBBERS);
            } else if constexpr (PLANES == 2) {
                asm volatile(QSV_GATE_LOOP_ASM_2P
                             : QSV_LOOP_OUT
                             : QSV_LOOP_IN, [plane4] "n"(PLANE * 4u), [pl64] "n"(PLANE / 64u)
                             : QSV_GATE_LOOP_CLOBBERS);
            } else if constexpr (PERLANE) {
                unsigned ldsn;
                asm volatile(QSV_GATE_LOOP_ASM_1P_ROWS
                             : QSV_LOOP_OUT, [ldsn] "=&v"(ldsn)
                             : QSV_LOOP_IN
                             : QSV_GATE_LOOP_CLOBBERS);
            } else {
                unsigned ldsn;
                asm volatile(QSV_GATE_LOOP_ASM_1P
                             : QSV_LOOP_OUT, [ldsn] "=&v"(ldsn)
                             : QSV_LOOP_IN
                             : QSV_GATE_LOOP_CLOBBERS);
            }
#undef QSV_LOOP_OUT
#undef QSV_LOOP_IN
        }
        // Operations are read as one aligned 64-bit word each and decoded with shifts.
        const u64 opp = ((u64)opshi << 32) | opslo;
        const u32x2 word = *(cuint2_p)(uintptr_t)opp;
        const unsigned kind = word.x & 0xffu;
        const int arg = (int)word.y;
        e0 = ((u64)e0hi << 32) | e0lo;
        if (PERLANE && kind == OP_U) {
            // several rows per tile and row-dependent matrices: per-lane matrix.  The run lies
            // inside the qubit bits (planner rule), so a lane's 16 amplitudes share one row.
            float m[8], xr[NR], xi[NR];
            const u64 ee = e0 < a.total ? e0 : 0;
            const RowCtx rc = row_ctx(a.rm, ee >> a.n);
            const int lane_ovr = rc.ovr_id >= 0 ? a.exec_of[rc.ovr_id] : -1;
            const float* p = (arg == lane_ovr)
                ? a.ovr + (a.rowdep ? rc.sample * (u64)a.rm.two_p * 8 : 0) + rc.ovr_off
                : a.mats + ((a.rowdep ? rc.sample * (u64)a.n_mats : 0) + (u64)arg) * 8;
            const float4 lo = *reinterpret_cast<const float4*>(p);
            const float4 hi = *reinterpret_cast<const float4*>(p + 4);
            m[0] = lo.x; m[1] = lo.y; m[2] = lo.z; m[3] = lo.w;
            m[4] = hi.x; m[5] = hi.y; m[6] = hi.z; m[7] = hi.w;
#define QSV_IN(k) xr[k] = vr##k; xi[k] = vi##k;
            QSV_16(QSV_IN)
#undef QSV_IN
            apply_u_any((int)((word.x >> 8) & 0xffu), xr, xi, m);
#define QSV_OUT(k) vr##k = xr[k]; vi##k = xi[k];
            QSV_16(QSV_OUT)
#undef QSV_OUT
        } else {
            break;  // OP_END (the interpreter never stops on anything else)
        }
        { const u64 nx = opp + 8; opslo = (unsigned)nx; opshi = (unsigned)(nx >> 32); }
    }
    if (a.zout) {
        // Last pass of a gradient row: <Z_q> of the tile instead of (or besides) the stored state.
        // A lane sums its 16 probabilities with the sign of bit q (register part: per element,
        // uniform; the rest: from the lane's index), a wavefront adds its lanes in double, and each
        // wavefront writes one partial: [tile][wavefront], summed per row in a fixed order later.
        const int zq = a.zq;
        float acc = 0.f;
#define QSV_Z(k) { const float p = vr##k * vr##k + vi##k * vi##k; \
                   acc += ((expand((unsigned)k << scur) >> zq) & 1ull) ? -p : p; }
        QSV_16(QSV_Z)
#undef QSV_Z
        if ((e0 >> zq) & 1ull) acc = -acc;
        const double tot = wave_sum((double)acc);
        if ((thr & 63u) == 0) a.zout[tb * (blockDim.x >> 6) + (thr >> 6)] = tot;
        if (a.nostore) return;
    }
    if (a.prio) __builtin_amdgcn_s_setprio(3);
    if (a.imap) {
        // Deferred CNOTs: every amplitude goes to the index its position maps to.  The map is linear
        // over XOR, so the destination is (tile's part) ^ (lane's part) ^ (register element's part);
        // bits at and above n (the state row) stay.  The host only sets imap when every tile is full and
        // byte offsets inside a row fit 32 bits.
        const unsigned nmask = (1u << a.n) - 1u;
        const unsigned* im = a.imap;
        unsigned et = 0;
        for (unsigned rem = to_sgpr((unsigned)tile_base & nmask); rem; rem &= rem - 1u) et ^= im[__builtin_ctz(rem)];
        const unsigned pos_lane = (unsigned)(e0 ^ tile_base);      // the lane's own index bits (register bits zero)
        unsigned el = et;
        for (int b = 0; b < T; ++b) {
            if (b >= (int)scur && b < (int)scur + R) continue;       // register bits follow below
            const int q = b < c ? b : b - c + w;                     // index bit behind tile bit b
            if (q >= a.n) continue;
            el ^= ((pos_lane >> q) & 1u) ? im[q] : 0u;
        }
        auto reg_part = [&](int j) -> unsigned {
            const int b = (int)scur + j;
            const int q = b < c ? b : b - c + w;
            return im[q];
        };
        const unsigned x0 = reg_part(0), x1 = reg_part(1), x2 = reg_part(2), x3 = reg_part(3);
        char* bp = (char*)(a.state + (tile_base & ~(u64)nmask));
        unsigned idx = el ^ x0;                                      // the walk starts from "element 0 minus bit 0"
        if (a.nt_store) {
#define QSV_ST(k, bit, sign) { idx ^= x##bit; \
                    f32x2 v; v.x = vr##k; v.y = vi##k; __builtin_nontemporal_store(v, (f32x2*)(bp + (u64)idx * 8u)); }
            QSV_16G(QSV_ST)
#undef QSV_ST
        } else {
#define QSV_ST(k, bit, sign) { idx ^= x##bit; *(float2*)(bp + (u64)idx * 8u) = make_float2(vr##k, vi##k); }
            QSV_16G(QSV_ST)
#undef QSV_ST
        }
    } else if (full && off32 && a.nt_store) {
        // States much larger than the last-level cache: nontemporal stores, so that the lines written
        // now (read again only a whole pass later) do not displace what the pass still has to read.
        const unsigned lane_byte = (unsigned)(e0 ^ tile_base) * 8u;   // the lane's own index bits
        const u64 st0 = expand(1u << scur) * 8u, st1 = expand(2u << scur) * 8u, st2 = expand(4u << scur) * 8u,
                  st3 = expand(8u << scur) * 8u;
        char* bp = (char*)(a.state + tile_base) - st0;
#define QSV_ST(k, bit, sign) { bp = bp sign st##bit; \
                    f32x2 v; v.x = vr##k; v.y = vi##k; __builtin_nontemporal_store(v, (f32x2*)(bp + lane_byte)); }
        QSV_16G(QSV_ST)
#undef QSV_ST
    } else if (full && off32) {
        const unsigned lane_byte = (unsigned)(e0 ^ tile_base) * 8u;
        const u64 st0 = expand(1u << scur) * 8u, st1 = expand(2u << scur) * 8u, st2 = expand(4u << scur) * 8u,
                  st3 = expand(8u << scur) * 8u;
        char* bp = (char*)(a.state + tile_base) - st0;
#define QSV_ST(k, bit, sign) { bp = bp sign st##bit; *(float2*)(bp + lane_byte) = make_float2(vr##k, vi##k); }
        QSV_16G(QSV_ST)
#undef QSV_ST
    } else if (full) {
#define QSV_ST(k) a.state[e0 | expand((unsigned)k << scur)] = make_float2(vr##k, vi##k);
        QSV_16(QSV_ST)
#undef QSV_ST
    } else {
#define QSV_ST(k) { const u64 e = e0 | expand((unsigned)k << scur); if (e < a.total) a.state[e] = make_float2(vr##k, vi##k); }
        QSV_16(QSV_ST)
#undef QSV_ST
    }
}

// ------------------------------------------------------------------------------------------
// One-gate-per-launch kernels.
__global__ __launch_bounds__(256) void k_naive_u(float2* state, u64 pairs, int n, int q,
                                                 const float* mats, const float* ovr, int mat_id,
                                                 int n_mats, int rowdep, RowMap rm) {
    const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
    if (i >= pairs) return;
    const u64 bit = 1ull << q;
    const u64 k0 = ((i >> q) << (q + 1)) | (i & (bit - 1));  // extended index, bit q clear
    const u64 k1 = k0 | bit;
    const RowCtx rc = row_ctx(rm, k0 >> n);
    const float* m = (mat_id == rc.ovr_id)
        ? ovr + (rowdep ? rc.sample * (u64)rm.two_p * 8 : 0) + rc.ovr_off
        : mats + ((rowdep ? rc.sample * (u64)n_mats : 0) + (u64)mat_id) * 8;
    const float2 x0 = state[k0], x1 = state[k1];
    float2 y0, y1;
    y0.x = m[0] * x0.x - m[1] * x0.y + m[2] * x1.x - m[3] * x1.y;
    y0.y = m[0] * x0.y + m[1] * x0.x + m[2] * x1.y + m[3] * x1.x;
    y1.x = m[4] * x0.x - m[5] * x0.y + m[6] * x1.x - m[7] * x1.y;
    y1.y = m[4] * x0.y + m[5] * x0.x + m[6] * x1.y + m[7] * x1.x;
    state[k0] = y0;
    state[k1] = y1;
}

__global__ __launch_bounds__(256) void k_naive_cnot(float2* state, u64 total, int ctrl, int tgt) {
    const u64 k = (u64)blockIdx.x * 256 + threadIdx.x;
    if (k >= total) return;
    if (((k >> ctrl) & 1) && !((k >> tgt) & 1)) {
        const u64 k1 = k | (1ull << tgt);
        const float2 t = state[k];
        state[k] = state[k1];
        state[k1] = t;
    }
}

__global__ __launch_bounds__(256) void k_naive_cz_ladder(float2* state, u64 total, int n) {
    const u64 e = (u64)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const u64 k = e & ((1ull << n) - 1);
    if (__popcll(k & (k >> 1)) & 1) {
        float2 v = state[e];
        v.x = -v.x; v.y = -v.y;
        state[e] = v;
    }
}

// ------------------------------------------------------------------------------------------
// Fused per-(layer, qubit) matrices, computed in double and rounded once to float.
struct M2 { double r[4], i[4]; };  // row-major 2x2: [0]=m00 [1]=m01 [2]=m10 [3]=m11

__device__ __forceinline__ M2 rot_m(int axis, double t) {
    double s, c;
    sincos(0.5 * t, &s, &c);
    M2 m;
    for (int k = 0; k < 4; ++k) { m.r[k] = 0.0; m.i[k] = 0.0; }
    if (axis == QSV_RX) { m.r[0] = c; m.i[1] = -s; m.i[2] = -s; m.r[3] = c; }
    else if (axis == QSV_RY) { m.r[0] = c; m.r[1] = -s; m.r[2] = s; m.r[3] = c; }
    else { m.r[0] = c; m.i[0] = -s; m.r[3] = c; m.i[3] = s; }
    return m;
}

__device__ __forceinline__ M2 mul_m(const M2& a, const M2& b) {  // a * b
    M2 o;
    for (int r = 0; r < 2; ++r)
        for (int cc = 0; cc < 2; ++cc) {
            double sr = 0.0, si = 0.0;
            for (int k = 0; k < 2; ++k) {
                const double ar = a.r[r * 2 + k], ai = a.i[r * 2 + k];
                const double br = b.r[k * 2 + cc], bi = b.i[k * 2 + cc];
                sr += ar * br - ai * bi;
                si += ar * bi + ai * br;
            }
            o.r[r * 2 + cc] = sr; o.i[r * 2 + cc] = si;
        }
    return o;
}

// U(l,q) for one sample: slots applied in order (re-upload RX first), i.e. U = R_last ... R_first.
// shift_slot >= 0 adds shift to that slot's angle.
__device__ M2 fused_raw(const CircDev& c, const float* params, const float* feats, u64 sample, int l,
                        int q, int shift_slot, double shift, int inverse) {
    M2 u;
    for (int k = 0; k < 4; ++k) { u.r[k] = (k == 0 || k == 3) ? 1.0 : 0.0; u.i[k] = 0.0; }
    const int slots = c.reupload + c.n_rot;
    for (int sl = 0; sl < slots; ++sl) {
        double t = (double)params[((u64)l * slots + sl) * c.n + q];
        int axis;
        if (c.reupload && sl == 0) { t *= (double)feats[sample * c.n + q]; axis = QSV_RX; }
        else axis = c.rot[sl - c.reupload];
        if (sl == shift_slot) t += shift;
        u = mul_m(rot_m(axis, t), u);
    }
    if (inverse) {  // conjugate transpose
        M2 d;
        d.r[0] = u.r[0]; d.i[0] = -u.i[0];
        d.r[1] = u.r[2]; d.i[1] = -u.i[2];
        d.r[2] = u.r[1]; d.i[2] = -u.i[1];
        d.r[3] = u.r[3]; d.i[3] = -u.i[3];
        u = d;
    }
    return u;
}

// Phase bookkeeping.  Within one layer the single-qubit unitaries act on different qubits, so a
// scalar factor may move freely between them.  Every matrix but the one of the last qubit is
// stored as W = conj(p) U with p = m00 / |m00|, which makes m00 real (and, for the common
// rotation sequences, a whole row or column real: the interpreter tests the stored zeros and
// picks a shorter multiply sequence).  The last qubit's matrix takes the product of the removed
// factors, so the layer as a whole, and hence the state, is unchanged.
struct Ph { double r, i; };

__device__ __forceinline__ Ph phase_of(const M2& u) {
    const double mag = hypot(u.r[0], u.i[0]);
    if (mag < 1e-6) return {1.0, 0.0};
    return {u.r[0] / mag, u.i[0] / mag};
}

__device__ __forceinline__ void scale_m(M2& u, double pr, double pi) {  // u *= (pr + i pi)
    for (int k = 0; k < 4; ++k) {
        const double a = u.r[k], b = u.i[k];
        u.r[k] = a * pr - b * pi;
        u.i[k] = a * pi + b * pr;
    }
}

__device__ __forceinline__ void strip_phase(M2& u) {
    const Ph p = phase_of(u);
    if (p.r == 1.0 && p.i == 0.0) return;
    const double mag = hypot(u.r[0], u.i[0]);
    scale_m(u, p.r, -p.i);
    u.r[0] = mag; u.i[0] = 0.0;
}

// Product of the factors removed from qubits 0..n-2 of layer l.
__device__ Ph layer_phase(const CircDev& c, const float* params, const float* feats, u64 sample,
                          int l, int inverse) {
    Ph acc = {1.0, 0.0};
    for (int q = 0; q + 1 < c.n; ++q) {
        const Ph p = phase_of(fused_raw(c, params, feats, sample, l, q, -1, 0.0, inverse));
        const double r = acc.r * p.r - acc.i * p.i;
        acc.i = acc.r * p.i + acc.i * p.r;
        acc.r = r;
    }
    return acc;
}

__device__ __forceinline__ void store_m(M2& u, float* out8) {
    // imaginary parts that vanish by structure come out as rounding noise of a few 1e-17:
    // store them as exact zeros so that the fast paths apply
    for (int k = 0; k < 4; ++k)
        if (fabs(u.i[k]) < 1e-14) u.i[k] = 0.0;
    for (int k = 0; k < 4; ++k) { out8[2 * k] = (float)u.r[k]; out8[2 * k + 1] = (float)u.i[k]; }
}

// Entry pos of an order table.  period > 0: the table has `period` entries and describes one layer;
// it repeats for every layer (entry pos of layer pos / period is that layer's entry pos % period).
__device__ __forceinline__ int ordered(const int* table, int period, int pos) {
    return period > 0 ? (pos / period) * period + table[pos % period] : table[pos];
}

// Two steps, so that every thread does the same amount of work.  Step 1, one thread per matrix:
// build it, and for every qubit but the last store it without its phase factor and note the factor;
// the last qubit's matrix is kept in double.  Step 2, one thread per (sample, layer): multiply the
// last qubit's matrix by the product of the layer's factors and store it.
// side: [tables][L*n] factors (2 doubles each), then [tables][L] matrices (8 doubles each).
__global__ __launch_bounds__(256) void k_build_mats(CircDev c, const float* params, const float* feats,
                                                    u64 count, int inverse, const int* order, int period,
                                                    float* out, double* side) {
    const u64 idx = (u64)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    const u64 per = (u64)c.n_layers * c.n;
    const u64 sample = idx / per;
    const int pos = (int)(idx % per);
    const int lq = order ? ordered(order, period, pos) : pos;
    const int l = lq / c.n, q = lq % c.n;
    M2 u = fused_raw(c, params, feats, sample, l, q, -1, 0.0, inverse);
    if (q + 1 < c.n) {
        const Ph p = phase_of(u);
        double* ps = side + (sample * per + (u64)lq) * 2;
        ps[0] = p.r; ps[1] = p.i;
        strip_phase(u);
        store_m(u, out + idx * 8);
    } else {
        const u64 tables = count / per;
        double* ms = side + tables * per * 2 + (sample * c.n_layers + (u64)l) * 8;
        for (int k = 0; k < 4; ++k) { ms[2 * k] = u.r[k]; ms[2 * k + 1] = u.i[k]; }
    }
}

// One table shared by the whole batch and few qubits: one launch in which the thread of a layer's
// last qubit recomputes that layer's factors itself.
__global__ __launch_bounds__(256) void k_build_mats_shared(CircDev c, const float* params, u64 count,
                                                           int inverse, const int* order, int period, float* out) {
    const u64 idx = (u64)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    const int lq = order ? ordered(order, period, (int)idx) : (int)idx;
    const int l = lq / c.n, q = lq % c.n;
    M2 u = fused_raw(c, params, nullptr, 0, l, q, -1, 0.0, inverse);
    if (q + 1 < c.n) strip_phase(u);
    else { const Ph p = layer_phase(c, params, nullptr, 0, l, inverse); scale_m(u, p.r, p.i); }
    store_m(u, out + idx * 8);
}

__global__ __launch_bounds__(256) void k_build_mats_last(CircDev c, u64 tables, const int* exec_of, int period,
                                                         float* out, const double* side) {
    const u64 idx = (u64)blockIdx.x * 256 + threadIdx.x;
    if (idx >= tables * c.n_layers) return;
    const u64 per = (u64)c.n_layers * c.n;
    const u64 sample = idx / c.n_layers;
    const int l = (int)(idx % c.n_layers);
    Ph acc = {1.0, 0.0};
    for (int q = 0; q + 1 < c.n; ++q) {      // same order of multiplication as layer_phase
        const double* ps = side + (sample * per + (u64)l * c.n + q) * 2;
        const double r = acc.r * ps[0] - acc.i * ps[1];
        acc.i = acc.r * ps[1] + acc.i * ps[0];
        acc.r = r;
    }
    const double* ms = side + tables * per * 2 + idx * 8;
    M2 u;
    for (int k = 0; k < 4; ++k) { u.r[k] = ms[2 * k]; u.i[k] = ms[2 * k + 1]; }
    scale_m(u, acc.r, acc.i);
    const int lq = l * c.n + c.n - 1;
    const u64 pos = exec_of ? (u64)ordered(exec_of, period, lq) : (u64)lq;
    store_m(u, out + (sample * per + pos) * 8);
}

// Matrices with one angle shifted by +-pi/2 (parameter-shift rule), consistent with the phase
// bookkeeping of the unshifted table they are substituted into.
__global__ __launch_bounds__(256) void k_build_shifted(CircDev c, const float* params,
                                                       const float* feats, u64 count, float* out) {
    const u64 idx = (u64)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    const int slots = c.reupload + c.n_rot;
    const u64 two_p = 2ull * c.n_layers * slots * c.n;
    const u64 sample = idx / two_p;
    const int v = (int)(idx % two_p);
    const int p = v >> 1;
    const int q = p % c.n;
    const int sl = (p / c.n) % slots;
    const int l = p / (c.n * slots);
    const double shift = (v & 1) ? -1.57079632679489661923 : 1.57079632679489661923;
    M2 u = fused_raw(c, params, feats, sample, l, q, sl, shift, 0);
    if (q + 1 < c.n) {
        const Ph ph = phase_of(fused_raw(c, params, feats, sample, l, q, -1, 0.0, 0));
        scale_m(u, ph.r, -ph.i);
    } else {
        const Ph ph = layer_phase(c, params, feats, sample, l, 0);
        scale_m(u, ph.r, ph.i);
    }
    store_m(u, out + idx * 8);
}

// ------------------------------------------------------------------------------------------
// Amplitude encoding.
// inv_norm != NULL (only with nblk = 1): the block is the whole sample and finishes the norm itself.
__global__ __launch_bounds__(256) void k_sumsq(const float* x, u64 rows, u64 dim, double* partial, int nblk,
                                               double* inv_norm, float* norm_out) {
    __shared__ double sm[4];
    const u64 b = grid_row();
    if (b >= rows) return;
    const float* xb = x + b * dim;
    double acc = 0.0;
    if ((dim & 3) == 0 && ((uintptr_t)x & 15) == 0) {
        // rows are 16-byte aligned: four floats per load (the one-float form reaches 2 TB/s only)
        const float4* xv = reinterpret_cast<const float4*>(xb);
        const u64 dimv = dim >> 2;
        for (u64 base = (u64)blockIdx.x * (CHUNK / 4); base < dimv; base += (u64)nblk * (CHUNK / 4)) {
            float4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u64 k = base + (u64)i * 256 + threadIdx.x;
                v[i] = k < dimv ? xv[k] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc += (double)v[i].x * v[i].x + (double)v[i].y * v[i].y + (double)v[i].z * v[i].z +
                       (double)v[i].w * v[i].w;
        }
    } else {
        for (u64 base = (u64)blockIdx.x * CHUNK; base < dim; base += (u64)nblk * CHUNK) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const u64 k = base + (u64)i * 256 + threadIdx.x;
                if (k < dim) { const double v = (double)xb[k]; acc += v * v; }
            }
        }
    }
    const double tot = block_sum256(acc, sm);
    if (threadIdx.x == 0) {
        partial[b * nblk + blockIdx.x] = tot;
        if (inv_norm) {
            const double nrm = sqrt(tot);
            inv_norm[b] = nrm > 0.0 ? 1.0 / nrm : 0.0;
            if (norm_out) norm_out[b] = (float)nrm;
        }
    }
}

__global__ __launch_bounds__(256) void k_norm_finish(const double* partial, int nblk, double* inv_norm,
                                                     float* norm_out) {
    __shared__ double sm[4];
    const u64 b = blockIdx.x;
    double acc = 0.0;
    for (int i = threadIdx.x; i < nblk; i += 256) acc += partial[b * nblk + i];
    const double tot = block_sum256(acc, sm);
    if (threadIdx.x == 0) {
        const double nrm = sqrt(tot);
        inv_norm[b] = nrm > 0.0 ? 1.0 / nrm : 0.0;
        if (norm_out) norm_out[b] = (float)nrm;
    }
}

__global__ __launch_bounds__(256) void k_encode_write(const float* x, u64 dim, int n, u64 total,
                                                      const double* inv_norm, RowMap rm,
                                                      float2* state) {
    const u64 e2 = ((u64)blockIdx.x * 256 + threadIdx.x) * 2;
    if (e2 >= total) return;
    const u64 row = e2 >> n;
    const u64 sample = row_ctx(rm, row).sample;
    const double inv = inv_norm[sample];
    const u64 k = e2 & ((1ull << n) - 1);
    const float* xb = x + sample * dim;
    float4 o;
    o.x = k < dim ? (float)((double)xb[k] * inv) : 0.f;
    o.y = 0.f;
    o.z = (k + 1) < dim ? (float)((double)xb[k + 1] * inv) : 0.f;
    o.w = 0.f;
    *reinterpret_cast<float4*>(state + e2) = o;
}

// Small samples (one block covers a sample): norm and state row in one launch.  Same arithmetic as
// k_sumsq + k_encode_write, so the bits are the same.
__global__ __launch_bounds__(256) void k_encode_small(const float* x, u64 rows, u64 dim, int n, double* inv_norm,
                                                      float* norm_out, float2* state) {
    __shared__ double sm[4];
    const u64 b = grid_row();
    if (b >= rows) return;
    const float* xb = x + b * dim;
    double acc = 0.0;
    for (u64 k = threadIdx.x; k < dim; k += 256) { const double v = (double)xb[k]; acc += v * v; }
    const double tot = block_sum256(acc, sm);
    const double nrm = sqrt(tot);
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    if (threadIdx.x == 0) {
        inv_norm[b] = inv;
        if (norm_out) norm_out[b] = (float)nrm;
    }
    float2* row = state + (b << n);
    for (u64 k = threadIdx.x; k < (1ull << n); k += 256)
        row[k] = make_float2(k < dim ? (float)((double)xb[k] * inv) : 0.f, 0.f);
}

// ------------------------------------------------------------------------------------------
// Measurement.
__global__ __launch_bounds__(256) void k_probs(const float2* state, u64 total, float* out) {
    const u64 e2 = ((u64)blockIdx.x * 256 + threadIdx.x) * 2;
    if (e2 >= total) return;
    const float4 v = *reinterpret_cast<const float4*>(state + e2);
    float2 o;
    o.x = prob32(make_float2(v.x, v.y));
    o.y = prob32(make_float2(v.z, v.w));
    *reinterpret_cast<float2*>(out + e2) = o;
}

// Block (row, blk) reduces 4096 consecutive amplitudes to 13 doubles: total T and the signed sums
// Z_0..Z_11 for the 12 index bits inside the chunk.  Chunk-local index = i*256 + thread
// (bits 0-5 lane, 6-7 wavefront, 8-11 register).
// direct != NULL (only with nblk = 1: a row is one chunk): the block writes the row's <Z_q> itself,
// float(the sum the finishing kernel would copy), for every qubit (q_only < 0) or for q_only alone.
__global__ __launch_bounds__(256) void k_expz_block(const float2* state, u64 rows, int n, int nblk,
                                                    double* partial, float* direct, int q_only) {
    __shared__ double sm[4][11];
    const u64 row = grid_row();
    if (row >= rows) return;
    const u64 dimn = 1ull << n;
    const u64 base = (u64)blockIdx.x * CHUNK;
    const float2* a = state + row * dimn;
    double T = 0.0, zr[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const u64 k = base + (u64)i * 256 + threadIdx.x;
        double p = 0.0;
        if (k < dimn) p = (double)prob32(a[k]);
        T += p;
#pragma unroll
        for (int j = 0; j < 4; ++j) zr[j] += ((i >> j) & 1) ? -p : p;
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    double zl[6];
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        const double Tp = __shfl_xor(T, 1 << b, 64);
#pragma unroll
        for (int j = 0; j < 4; ++j) zr[j] += __shfl_xor(zr[j], 1 << b, 64);
#pragma unroll
        for (int j = 0; j < 6; ++j)
            if (j < b) zl[j] += __shfl_xor(zl[j], 1 << b, 64);
        zl[b] = ((lane >> b) & 1) ? Tp - T : T - Tp;
        T += Tp;
    }
    if (lane == 0) {
        sm[wv][0] = T;
#pragma unroll
        for (int j = 0; j < 6; ++j) sm[wv][1 + j] = zl[j];
#pragma unroll
        for (int j = 0; j < 4; ++j) sm[wv][7 + j] = zr[j];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double loc[13];
        double* o = direct ? loc : partial + (row * nblk + blockIdx.x) * 13;
        const double t0 = sm[0][0], t1 = sm[1][0], t2 = sm[2][0], t3 = sm[3][0];
        o[0] = (t0 + t1) + (t2 + t3);
        for (int j = 0; j < 6; ++j) o[1 + j] = (sm[0][1 + j] + sm[1][1 + j]) + (sm[2][1 + j] + sm[3][1 + j]);
        o[7] = (t0 - t1) + (t2 - t3);
        o[8] = (t0 + t1) - (t2 + t3);
        for (int j = 0; j < 4; ++j) o[9 + j] = (sm[0][7 + j] + sm[1][7 + j]) + (sm[2][7 + j] + sm[3][7 + j]);
        if (direct) {
            if (q_only >= 0) direct[row] = (float)o[1 + q_only];
            else
                for (int q = 0; q < n; ++q) direct[row * n + q] = (float)o[1 + q];
        }
    }
}

// One wavefront per (row, qubit): combine block partials.  Bits below 12 use the blocks' signed
// sums; higher bits are constant inside a block, so they sign the block totals.
__global__ __launch_bounds__(256) void k_expz_finish(const double* partial, u64 rows, int n, int nblk,
                                                     int q_only, float* out_f, double* out_d,
                                                     Scatter sc) {
    const int lane = threadIdx.x & 63;
    const u64 job = (u64)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nq = q_only >= 0 ? 1 : n;
    if (job >= rows * nq) return;
    const u64 row = job / nq;
    const int q = q_only >= 0 ? q_only : (int)(job % nq);
    const double* p = partial + row * nblk * 13;
    double acc = 0.0;
    if (q < CHUNK_BITS) {
        for (int b = lane; b < nblk; b += 64) acc += p[(u64)b * 13 + 1 + q];
    } else {
        for (int b = lane; b < nblk; b += 64) {
            const double t = p[(u64)b * 13];
            acc += ((b >> (q - CHUNK_BITS)) & 1) ? -t : t;
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) {
        u64 o = job;
        if (sc.per > 0) {  // one qubit per row (q_only >= 0): job = row of the chunk
            const u64 gid = (u64)sc.row0 + job;
            o = (gid / (u64)sc.per) * (u64)sc.stride + (u64)sc.offset + gid % (u64)sc.per;
        }
        if (out_f) out_f[o] = (float)acc;
        if (out_d) out_d[o] = acc;
    }
}

// Sums the per-wavefront <Z> partials the last pass wrote, one thread per row, in index order.
__global__ __launch_bounds__(256) void k_zsum_finish(const double* partial, u64 rows, u64 per_row,
                                                     double* out, Scatter sc) {
    const u64 r = (u64)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    const double* p = partial + r * per_row;
    double acc = 0.0;
    for (u64 i = 0; i < per_row; ++i) acc += p[i];
    const u64 gid = (u64)sc.row0 + r;
    out[(gid / (u64)sc.per) * (u64)sc.stride + (u64)sc.offset + gid % (u64)sc.per] = acc;
}

// Copies each row's starting state from the per-sample source (16 bytes per lane and step).
__global__ __launch_bounds__(256) void k_gather_rows(const float2* src, int n, u64 total, RowMap rm,
                                                     float2* states) {
    const u64 e2 = ((u64)blockIdx.x * 256 + threadIdx.x) * 2;
    if (e2 >= total) return;
    const u64 row = e2 >> n;
    const u64 k = e2 & ((1ull << n) - 1);
    const u64 sample = row_ctx(rm, row).sample;
    *reinterpret_cast<float4*>(states + e2) = *reinterpret_cast<const float4*>(src + ((sample << n) | k));
}

__device__ __forceinline__ u64 deposit(u64 v, u64 mask, int n) {  // spread the bits of v over mask
    u64 o = 0;
    int j = 0;
    for (int q = 0; q < n; ++q)
        if ((mask >> q) & 1) { o |= ((v >> j) & 1ull) << q; ++j; }
    return o;
}

// Block (row, v, blk): sum of p over the indices whose mask bits read v, 4096 of them per block.
__global__ __launch_bounds__(256) void k_marginal_block(const float2* state, int n, u64 mask, u64 n_v,
                                                        u64 nblk, u64 sub, double* partial) {
    __shared__ double sm[4];
    const u64 id = blockIdx.x;
    const u64 blk = id % nblk;
    const u64 v = (id / nblk) % n_v;
    const u64 row = id / (nblk * n_v);
    const u64 fixed = deposit(v, mask, n);
    const u64 free_mask = ((1ull << n) - 1) & ~mask;
    const float2* a = state + (row << n);
    double acc = 0.0;
    if ((free_mask & (CHUNK - 1)) == (u64)(CHUNK - 1)) {
        // no mask bit among the low 12 index bits: a block's elements are contiguous
        const float2* ab = a + (fixed | deposit(blk * CHUNK, free_mask, n));
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const u64 lo = (u64)i * 256 + threadIdx.x;
            if (blk * CHUNK + lo < sub) acc += (double)prob32(ab[lo]);
        }
    } else {
#pragma unroll 4
        for (int i = 0; i < 16; ++i) {
            const u64 j = blk * CHUNK + (u64)i * 256 + threadIdx.x;
            if (j < sub) acc += (double)prob32(a[fixed | deposit(j, free_mask, n)]);
        }
    }
    const double tot = block_sum256(acc, sm);
    if (threadIdx.x == 0) partial[id] = tot;
}

// One wavefront per (row, v).  renorm_mode: 0 plain marginal; 1 also scale = 1; 2 also
// scale = 1/sqrt(P) (0 when P = 0).
__global__ __launch_bounds__(256) void k_marginal_finish(const double* partial, u64 jobs, u64 nblk,
                                                         float* out, int renorm_mode, double* scale) {
    const int lane = threadIdx.x & 63;
    const u64 job = (u64)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (job >= jobs) return;
    double acc = 0.0;
    for (u64 b = lane; b < nblk; b += 64) acc += partial[job * nblk + b];
    acc = wave_sum(acc);
    if (lane == 0) {
        out[job] = (float)acc;
        if (renorm_mode == 1) scale[job] = 1.0;
        if (renorm_mode == 2) scale[job] = acc > 0.0 ? 1.0 / sqrt(acc) : 0.0;
    }
}

__global__ __launch_bounds__(256) void k_project(float2* state, u64 total, int n, u64 mask,
                                                 const double* scale) {
    const u64 e = (u64)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    float2 v = state[e];
    if (e & mask) {  // mask has no bits at or above n
        v.x = 0.f; v.y = 0.f;
    } else {
        const double sc = scale[e >> n];
        v.x = (float)((double)v.x * sc);
        v.y = (float)((double)v.y * sc);
    }
    state[e] = v;
}

// Pauli string: T = sum_k conj(a[k ^ f]) (-1)^popcount(k & s) a[k], f = X and Y bits, s = Y and Z
// bits; <P> = Re(i^nY T).  The terms of k and k ^ f are conjugates of each other up to the sign
// (-1)^nY, so for f != 0 only the k whose highest flip bit is clear are visited, each amplitude is
// read once, and a pair adds 2 Re t (nY even) or 2 i Im t (nY odd) with t = conj(a[k ^ f]) sign(k) a[k].
// One block per 4096 visited indices and row; partial: [row][blk][2].
__global__ __launch_bounds__(256) void k_pauli_block(const float2* state, u64 rows, int n, u64 f, u64 s, int ny,
                                                     int nblk, double* partial) {
    __shared__ double sm[4];
    const u64 row = grid_row();
    if (row >= rows) return;
    const float2* a = state + (row << n);
    float tr = 0.f, ti = 0.f;
    if (f == 0) {
        const u64 N = 1ull << n;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const u64 k = (u64)blockIdx.x * CHUNK + (u64)i * 256 + threadIdx.x;
            if (k < N) {
                const float2 v = a[k];
                const float p = v.x * v.x + v.y * v.y;
                tr += (__popcll(k & s) & 1) ? -p : p;
            }
        }
    } else {
        const int hb = 63 - __clzll(f);               // pairs differ in this bit (and the lower bits of f)
        const u64 half = 1ull << (n - 1), low = (1ull << hb) - 1ull;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const u64 j = (u64)blockIdx.x * CHUNK + (u64)i * 256 + threadIdx.x;
            if (j < half) {
                const u64 k = ((j & ~low) << 1) | (j & low);        // bit hb clear
                const float2 v = a[k], u = a[k ^ f];
                float cr = u.x * v.x + u.y * v.y, ci = u.x * v.y - u.y * v.x;   // conj(u) v
                if (__popcll(k & s) & 1) { cr = -cr; ci = -ci; }
                if (ny & 1) ti += 2.f * ci; else tr += 2.f * cr;
            }
        }
    }
    const double t0 = block_sum256((double)tr, sm);
    const double t1 = block_sum256((double)ti, sm);
    if (threadIdx.x == 0) { double* o = partial + (row * nblk + blockIdx.x) * 2; o[0] = t0; o[1] = t1; }
}

__global__ __launch_bounds__(256) void k_pauli_finish(const double* partial, int nblk, int ny, float* out) {
    __shared__ double sm[4];
    const u64 row = blockIdx.x;
    double tr = 0.0, ti = 0.0;
    for (int i = threadIdx.x; i < nblk; i += 256) {
        const double* p = partial + (row * nblk + i) * 2;
        tr += p[0]; ti += p[1];
    }
    const double t0 = block_sum256(tr, sm);
    const double t1 = block_sum256(ti, sm);
    // Re(i^ny (t0 + i t1)): ny mod 4 = 0: t0; 1: -t1; 2: -t0; 3: t1
    if (threadIdx.x == 0) out[row] = (float)((ny & 3) == 0 ? t0 : (ny & 3) == 1 ? -t1 : (ny & 3) == 2 ? -t0 : t1);
}

__global__ __launch_bounds__(256) void k_fidelity_block(const float2* state, u64 rows, int n, const float* x,
                                                        u64 dim, int nblk, RowMap rm, double* partial) {
    __shared__ double sm[4];
    const u64 row = grid_row();
    if (row >= rows) return;
    const float2* a = state + (row << n);
    const float* xb = x + row_ctx(rm, row).sample * dim;
    double sxx = 0.0, sr = 0.0, si = 0.0;
    for (u64 base = (u64)blockIdx.x * CHUNK; base < dim; base += (u64)nblk * CHUNK) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const u64 k = base + (u64)i * 256 + threadIdx.x;
            if (k < dim) {
                const double xv = (double)xb[k];
                const float2 av = a[k];
                sxx += xv * xv;
                sr += xv * (double)av.x;
                si += xv * (double)av.y;
            }
        }
    }
    const double t0 = block_sum256(sxx, sm);
    const double t1 = block_sum256(sr, sm);
    const double t2 = block_sum256(si, sm);
    if (threadIdx.x == 0) {
        double* o = partial + (row * nblk + blockIdx.x) * 3;
        o[0] = t0; o[1] = t1; o[2] = t2;
    }
}

__global__ __launch_bounds__(256) void k_fidelity_finish(const double* partial, int nblk, float* out,
                                                         double* out_d) {
    __shared__ double sm[4];
    const u64 row = blockIdx.x;
    double sxx = 0.0, sr = 0.0, si = 0.0;
    for (int i = threadIdx.x; i < nblk; i += 256) {
        const double* p = partial + (row * nblk + i) * 3;
        sxx += p[0]; sr += p[1]; si += p[2];
    }
    const double t0 = block_sum256(sxx, sm);
    const double t1 = block_sum256(sr, sm);
    const double t2 = block_sum256(si, sm);
    if (threadIdx.x == 0) {
        const double F = t0 > 0.0 ? (t1 * t1 + t2 * t2) / t0 : 0.0;
        if (out) out[row] = (float)F;
        if (out_d) out_d[row] = F;
    }
}

// Trash reset: row gid = row0 + r stands for (sample, outcome t) = (gid / per, gid % per), per = 2^m.
// work[r][k] = state[sample][k | bits of t spread over mask] where k has no mask bit, else 0.
__global__ __launch_bounds__(256) void k_reset_rows(const float2* state, int n, u64 mask, u64 total,
                                                    RowMap rm, float2* work) {
    const u64 e2 = ((u64)blockIdx.x * 256 + threadIdx.x) * 2;
    if (e2 >= total) return;
    const u64 r = e2 >> n, k = e2 & ((1ull << n) - 1);
    const u64 gid = (u64)rm.row0 + r;
    const u64 sample = gid / (u64)rm.per, t = gid % (u64)rm.per;
    const u64 tb = deposit(t, mask, n);
    const float2* src = state + (sample << n);
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if ((k & mask) == 0) { const float2 v = src[k | tb]; o.x = v.x; o.y = v.y; }
    if (((k + 1) & mask) == 0) { const float2 v = src[(k + 1) | tb]; o.z = v.x; o.w = v.y; }
    *reinterpret_cast<float4*>(work + e2) = o;
}

// out[b] = sum over the per outcomes of Frow[b * per + t], in order.
__global__ __launch_bounds__(256) void k_reset_sum(const double* Frow, u64 per, u64 B, float* out) {
    const u64 b = (u64)blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    double acc = 0.0;
    for (u64 t = 0; t < per; ++t) acc += Frow[b * per + t];
    out[b] = (float)acc;
}

// Finite-shot estimate of <Z_q>: one wavefront per (row, qubit); samples < 0 (no valid outcome) are skipped.
__global__ __launch_bounds__(256) void k_shot_expz(const long long* samples, u64 shots, u64 rows, int n,
                                                   float* out) {
    const u64 job = (u64)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (job >= rows * n) return;
    const int lane = threadIdx.x & 63;
    const u64 row = job / n;
    const int q = (int)(job % n);
    const long long* s = samples + row * shots;
    double acc = 0.0, cnt = 0.0;
    for (u64 i = lane; i < shots; i += 64) {
        const long long v = s[i];
        if (v >= 0) { acc += ((v >> q) & 1) ? -1.0 : 1.0; cnt += 1.0; }
    }
    acc = wave_sum(acc);
    cnt = wave_sum(cnt);
    if (lane == 0) out[job] = cnt > 0.0 ? (float)(acc / cnt) : 0.f;
}

// ------------------------------------------------------------------------------------------
// Sampling: integer inverse CDF (see qsv.h).  All sums are uint64, hence order-independent.
__device__ __forceinline__ u64 weight60(float2 a) {
    const double p = (double)prob32(a);
    return p > 0.0 ? (u64)(p * 1152921504606846976.0) : 0ull;  // 2^60, truncation = floor
}

__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(256) void k_sample_blocksum(const float2* state, u64 rows, int n, int nblk, u64* bsum) {
    __shared__ u64 sm[4];
    const u64 row = grid_row();
    if (row >= rows) return;
    const u64 dimn = 1ull << n;
    const float2* a = state + (row << n);
    u64 acc = 0;
    if (dimn >= 2) {
        // two amplitudes per 16-byte load; integer sums do not care about the order
        const float4* a2 = reinterpret_cast<const float4*>(a);
        float4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const u64 k2 = (u64)blockIdx.x * (CHUNK / 2) + (u64)i * 256 + threadIdx.x;
            v[i] = k2 * 2 < dimn ? a2[k2] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc += weight60(make_float2(v[i].x, v[i].y)) + weight60(make_float2(v[i].z, v[i].w));
    } else if (blockIdx.x == 0 && threadIdx.x == 0) {
        acc = weight60(a[0]);
    }
    acc = wave_sum_u64(acc);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) bsum[row * nblk + blockIdx.x] = sm[0] + sm[1] + sm[2] + sm[3];
}

// In-place inclusive prefix sum of each row's block sums (one 1024-thread block per row).
__global__ __launch_bounds__(1024) void k_sample_scan(u64* cum, int nblk) {
    __shared__ u64 sm[1024];
    u64* c = cum + (u64)blockIdx.x * nblk;
    const int per = (nblk + 1023) / 1024;
    const int lo = threadIdx.x * per;
    const int hi = min(lo + per, nblk);
    u64 loc = 0;
    for (int i = lo; i < hi; ++i) loc += c[i];
    sm[threadIdx.x] = loc;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        u64 add = 0;
        if ((int)threadIdx.x >= o) add = sm[threadIdx.x - o];
        __syncthreads();
        sm[threadIdx.x] += add;
        __syncthreads();
    }
    u64 run = sm[threadIdx.x] - loc;  // exclusive prefix of this thread's span
    for (int i = lo; i < hi; ++i) { run += c[i]; c[i] = run; }
}

// One wavefront per shot.
__global__ __launch_bounds__(256) void k_sample_draw(const float2* state, int n, int nblk, const u64* cum,
                                                     const double* uniforms, u64 shots, u64 jobs,
                                                     long long* out) {
    const int lane = threadIdx.x & 63;
    const u64 job = (u64)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (job >= jobs) return;
    const u64 row = job / shots;
    const u64* c = cum + row * nblk;
    const u64 W = c[nblk - 1];
    if (W == 0) { if (lane == 0) out[job] = -1; return; }
    const u64 r = (u64)(uniforms[job] * 9007199254740992.0);  // floor(u * 2^53)
    const u64 t = (__umul64hi(r, W) << 11) | ((r * W) >> 53);   // floor(r * W / 2^53)
    int lo = 0, hi = nblk - 1;                                  // smallest block with cum > t
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (c[mid] > t) hi = mid; else lo = mid + 1;
    }
    u64 base = lo > 0 ? c[lo - 1] : 0;
    const u64 dimn = 1ull << n;
    const float2* a = state + (row << n);
    const u64 k0 = (u64)lo * CHUNK;
    long long found = -1;
    for (int it = 0; it < CHUNK / 64; ++it) {
        const u64 k = k0 + (u64)it * 64 + lane;
        u64 incl = k < dimn ? weight60(a[k]) : 0ull;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u64 up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        const u64 hit = __ballot(base + incl > t);
        if (hit) { found = (long long)(k0 + (u64)it * 64 + (u64)(__ffsll((long long)hit) - 1)); break; }
        base += __shfl(incl, 63, 64);
    }
    if (lane == 0) out[job] = found;
}

// ------------------------------------------------------------------------------------------
// Gradient assembly.
__global__ __launch_bounds__(256) void k_grad_finish(const double* f, u64 B, u64 P, CircDev c,
                                                     const float* feats, float* loss, float* grad) {
    const u64 idx = (u64)blockIdx.x * 256 + threadIdx.x;
    if (idx >= B * (P + 1)) return;
    const u64 b = idx / (P + 1), p = idx % (P + 1);
    const double* fb = f + b * (2 * P + 1);
    if (p == P) { if (loss) loss[b] = (float)fb[2 * P]; return; }
    double g = 0.5 * (fb[2 * p] - fb[2 * p + 1]);
    const int slots = c.reupload + c.n_rot;
    if (c.reupload && ((p / c.n) % slots) == 0) g *= (double)feats[b * c.n + (p % c.n)];
    grad[b * P + p] = (float)g;
}

// Batch means in a fixed order: one block per parameter (block P does the loss); thread t adds the
// samples t, t + 256, ... and the block adds its threads.
__global__ __launch_bounds__(256) void k_grad_mean(const double* f, u64 B, u64 P, CircDev c,
                                                   const float* feats, float* mean_loss,
                                                   float* mean_grad) {
    __shared__ double sm[4];
    const u64 p = blockIdx.x;
    const int slots = c.reupload + c.n_rot;
    double acc = 0.0;
    if (p == P) {
        if (!mean_loss) return;
        for (u64 b = threadIdx.x; b < B; b += 256) acc += f[b * (2 * P + 1) + 2 * P];
        const double tot = block_sum256(acc, sm);
        if (threadIdx.x == 0) mean_loss[0] = (float)(tot / (double)B);
        return;
    }
    if (!mean_grad) return;
    const bool isw = c.reupload && ((p / c.n) % slots) == 0;
    for (u64 b = threadIdx.x; b < B; b += 256) {
        const double* fb = f + b * (2 * P + 1);
        double g = 0.5 * (fb[2 * p] - fb[2 * p + 1]);
        if (isw) g *= (double)feats[b * c.n + (p % c.n)];
        acc += g;
    }
    const double tot = block_sum256(acc, sm);
    if (threadIdx.x == 0) mean_grad[p] = (float)(tot / (double)B);
}

// ------------------------------------------------------------------------------------------
// Reverse-mode (adjoint) gradient of <Z_obs>.  Rows come in pairs: 2r holds psi, 2r+1 holds lambda.

// S[2r] = A[r], S[2r+1] = O A[r] for a diagonal observable O given by its weight w(k):
//   kind 0: Z_q,             w = +1 / -1 by bit q
//   kind 1: -P0(mask),       w = -1 where no bit of mask is set, else 0  (loss 1 - P0)
//   kind 2: sum_q c[r][q] Z_q, w = sum_q c[r][q] (1 - 2 bit_q(k))        (chain rule of the squared error)
struct AdjObs { int kind; int q; u64 mask; const double* coef; };

__device__ __forceinline__ float adj_weight(const AdjObs& o, u64 r, u64 k, int n) {
    if (o.kind == 0) return ((k >> o.q) & 1ull) ? -1.f : 1.f;
    if (o.kind == 1) return (k & o.mask) ? 0.f : -1.f;
    double w = 0.0;
    const double* c = o.coef + r * n;
    for (int q = 0; q < n; ++q) w += ((k >> q) & 1ull) ? -c[q] : c[q];
    return (float)w;
}

__global__ __launch_bounds__(256) void k_adj_init(const float2* A, int n, AdjObs o, u64 total, float2* S,
                                                  int paired) {
    const u64 e2 = ((u64)blockIdx.x * 256 + threadIdx.x) * 2;
    if (e2 >= total) return;
    const u64 r = e2 >> n, k = e2 & ((1ull << n) - 1);
    const float4 v = *reinterpret_cast<const float4*>(A + e2);
    const float w0 = adj_weight(o, r, k, n), w1 = adj_weight(o, r, k + 1, n);
    float4 z;
    z.x = w0 * v.x; z.y = w0 * v.y; z.z = w1 * v.z; z.w = w1 * v.w;
    if (paired) {
        *reinterpret_cast<float4*>(S + (((2 * r) << n) | k)) = v;
        *reinterpret_cast<float4*>(S + (((2 * r + 1) << n) | k)) = z;
    } else {
        *reinterpret_cast<float4*>(S + e2) = z;
    }
}

// P0(mask) of every row: block partials, then one thread per row; f[sample][2P] = 1 - P0.
__global__ __launch_bounds__(256) void k_p0_block(const float2* A, u64 rows, int n, u64 mask, int nblk, double* partial) {
    __shared__ double sm[4];
    const u64 r = grid_row(), N = 1ull << n;
    if (r >= rows) return;
    const float2* a = A + (r << n);
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const u64 k = (u64)blockIdx.x * 4096 + (u64)i * 256 + threadIdx.x;
        if (k < N && (k & mask) == 0) { const float2 v = a[k]; acc += v.x * v.x + v.y * v.y; }
    }
    const double t = block_sum256((double)acc, sm);
    if (threadIdx.x == 0) partial[r * nblk + blockIdx.x] = t;
}

__global__ __launch_bounds__(256) void k_trash_loss(const double* partial, int nblk, u64 rows, u64 sample0,
                                                    u64 P, double* f) {
    const u64 r = (u64)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    double acc = 0.0;
    for (int b = 0; b < nblk; ++b) acc += partial[r * nblk + b];
    f[(sample0 + r) * (2 * P + 1) + 2 * P] = 1.0 - acc;
}

// Squared-error loss on <Z_q>: z [rows][n] (double), y [samples][n] (float):
// f[sample][2P] = 1/n sum (z - y)^2 and coef[r][q] = 2/n (z - y), the weights of the Z_q in lambda.
__global__ __launch_bounds__(256) void k_mse_coef(const double* z, const float* y, int n, u64 rows,
                                                  u64 sample0, u64 P, double* coef, double* f) {
    const u64 r = (u64)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    double acc = 0.0;
    for (int q = 0; q < n; ++q) {
        const double d = z[r * n + q] - (double)y[(sample0 + r) * n + q];
        acc += d * d;
        coef[r * n + q] = 2.0 * d / n;
    }
    f[(sample0 + r) * (2 * P + 1) + 2 * P] = acc / n;
}

// M_q[a][b] = sum over the other qubits of conj(lambda[a, rest]) psi[b, rest], for one row pair
// (blockIdx.z) and one qubit (blockIdx.y); a block covers 4096 index pairs and writes 8 doubles in
// the layout (re, im of M00, M01, M10, M11).  The derivative is 2 Re sum_ab Bt[a][b] M[a][b] with an
// anti-Hermitian Bt (Bt00, Bt11 imaginary, Bt10 = -conj(Bt01)), which equals
// -2 (Im Bt00 Im M00 + Im Bt11 Im M11) + 2 Re(Bt01 K) with K = M01 - conj(M10).  So only Im M00,
// Im M11 and K are summed; K is stored in the place of M01 and the other entries are zero, which lets
// k_adj_layer use the plain formula.  Pair r is (psi0 + rstride r 2^n, lam0 + rstride r 2^n): the two
// states interleaved in one buffer (lam0 = psi0 + 2^n, rstride 2) or in buffers of their own (rstride 1).
__global__ __launch_bounds__(256) void k_trans_block(const float2* psi0, const float2* lam0, int rstride, int n,
                                                     u64 pairs, int nblk, double* partial) {
    __shared__ double sm[4];
    const int q = blockIdx.y;
    const u64 r = blockIdx.z;
    const float2* psi = psi0 + ((rstride * r) << n);
    const float2* lam = lam0 + ((rstride * r) << n);
    const u64 bit = 1ull << q;
    float acc[4];   // Im M00, Re K, Im K, Im M11
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const u64 p = (u64)blockIdx.x * 4096 + (u64)i * 256 + threadIdx.x;
        if (p < pairs) {
            const u64 k0 = ((p >> q) << (q + 1)) | (p & (bit - 1));
            const u64 k1 = k0 | bit;
            const float2 l0 = lam[k0], l1 = lam[k1], s0 = psi[k0], s1 = psi[k1];
            acc[0] += l0.x * s0.y - l0.y * s0.x;
            acc[3] += l1.x * s1.y - l1.y * s1.x;
            acc[1] += (l0.x * s1.x + l0.y * s1.y) - (l1.x * s0.x + l1.y * s0.y);
            acc[2] += (l0.x * s1.y - l0.y * s1.x) + (l1.x * s0.y - l1.y * s0.x);
        }
    }
    double* out = partial + ((r * n + q) * (u64)nblk + blockIdx.x) * 8;
    const double m00 = block_sum256((double)acc[0], sm), kre = block_sum256((double)acc[1], sm);
    const double kim = block_sum256((double)acc[2], sm), m11 = block_sum256((double)acc[3], sm);
    if (threadIdx.x == 0) {
        out[0] = 0.0; out[1] = m00; out[2] = kre; out[3] = kim;
        out[4] = 0.0; out[5] = 0.0; out[6] = 0.0; out[7] = m11;
    }
}

// The same sums for n >= 12, several qubits per read of the two states: a workgroup takes a tile of
// 2^12 amplitudes of psi and of lambda (tile = the c lowest index bits plus 12 - c bits from bit w,
// as in the pass kernel) and forms the index pairs of a qubit in registers: a lane holds, of each
// state, a run of amplitudes that differ in a few tile bits.
// Arithmetic per amplitude and qubit (only Im M00, Im M11 and K = M01 - conj(M10) are needed, see
// k_trans_block): d = Im conj(lambda[k]) psi[k] does not depend on the qubit, Im M00 sums it over the
// indices with the bit clear, and Im (M00 + M11) = sum of all d is the same for every qubit, so it is
// kept once (tsum) and Im M11 comes out as a difference at the end; K takes 8 FMAs per index pair.
// A workgroup covers `per_group` consecutive tiles of one row pair before it reduces its
// accumulators, so the reduction is amortised.
// partial: [(pair * n + qubit) * nblk + group * 4 + wavefront][8] (nblk = 4 * groups), the layout
// k_trans_finish and k_adj_layer read.

// A pointer to global memory that is the same in every lane, moved to scalar registers so that loads
// through it take the scalar-base + 32-bit lane offset form (no 64-bit address per lane).
typedef const __attribute__((address_space(1))) char* global_bytes;
__device__ __forceinline__ global_bytes uniform_ptr(const void* p) {
    const u64 v = (u64)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (global_bytes)(((u64)hi << 32) | lo);
}
__device__ __forceinline__ float2 load_f2(global_bytes base, unsigned byte_offset) {
    const f32x2 v = *(const __attribute__((address_space(1))) f32x2*)(base + byte_offset);
    return make_float2(v.x, v.y);
}

template <int N>
__device__ __forceinline__ void trans_diag(const float2 (&s)[N], const float2 (&l)[N], float (&d)[N],
                                           float& tsum) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
        d[i] = fmaf(-l[i].y, s[i].x, l[i].x * s[i].y);      // Im conj(lambda) psi
        tsum += d[i];
    }
}

// acc: Im M00, Re K, Im K of the qubit behind run bit BIT (K = M01 - conj(M10))
template <int N, int BIT>
__device__ __forceinline__ void trans_acc(const float2 (&s)[N], const float2 (&l)[N], const float (&d)[N],
                                          float (&acc)[3]) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
        if (i & (1 << BIT)) continue;
        constexpr int B = 1 << BIT;
        acc[0] += d[i];
        acc[1] = fmaf(-l[i | B].y, s[i].y, fmaf(-l[i | B].x, s[i].x,
                 fmaf(l[i].y, s[i | B].y, fmaf(l[i].x, s[i | B].x, acc[1]))));
        acc[2] = fmaf(-l[i | B].y, s[i].x, fmaf(l[i | B].x, s[i].y,
                 fmaf(-l[i].y, s[i | B].x, fmaf(l[i].x, s[i | B].y, acc[2]))));
    }
}

// What a wavefront writes for one qubit: the 8-double layout of k_trans_block.
__device__ __forceinline__ void trans_store(double* out, double m00, double kre, double kim, double tsum) {
    out[0] = 0.0; out[1] = m00; out[2] = kre; out[3] = kim;
    out[4] = 0.0; out[5] = 0.0; out[6] = 0.0; out[7] = tsum - m00;
}

// Tile bits J0..11, J0 >= 8 (a window of which only the top bits are still wanted): they are the run
// of the 16 amplitudes a lane loads from memory (tau = i * 256 + lane index, coalesced), so nothing
// goes through LDS.
template <int J0>
__global__ __launch_bounds__(256) void k_trans_tile(const float2* psi0, const float2* lam0, int rstride, int n,
                                                    int c, int w, int per_group, int nblk, double* partial) {
    static_assert(J0 >= 8 && J0 < 12, "lower tile bits are served by k_trans_wave");
    constexpr int NJ = 12 - J0;                      // acc[a] belongs to tile bit J0 + a
    const u64 r = blockIdx.y;
    const float2* psi = psi0 + ((rstride * r) << n);
    const float2* lam = lam0 + ((rstride * r) << n);
    const unsigned t = threadIdx.x;
    const unsigned cmask = (1u << c) - 1u;
    const int wc = w - c;
    float acc[NJ][3];
    float tsum = 0.f;
#pragma unroll
    for (int a = 0; a < NJ; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) acc[a][b] = 0.f;
    // tau = i * 256 + t sits at index base | (tau & cmask) | (tau >> c) << w = base + i * stride + kt, both
    // for contiguous tiles (c = 12) and for c = 4 (tau >> 4 = i * 16 + (t >> 4)); base + i * stride is the
    // same for all lanes (scalar registers), kt a 32-bit lane offset
    const u64 stride = c == 12 ? 256ull : (16ull << w);
    const unsigned kt8 = ((t & cmask) | ((t >> c) << w)) * 8u;   // in bytes: below 2^(n-1)
    for (int g = 0; g < per_group; ++g) {
        const u64 tb = (u64)blockIdx.x * per_group + g;      // tile of the row
        const u64 base = ((tb & ((1ull << wc) - 1ull)) << c) | ((tb >> wc) << (w + 12 - c));
        float2 s[16], l[16];
        float d[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            s[i] = load_f2(uniform_ptr(psi + (base + (u64)i * stride)), kt8);
            l[i] = load_f2(uniform_ptr(lam + (base + (u64)i * stride)), kt8);
        }
        trans_diag<16>(s, l, d, tsum);
        if constexpr (J0 <= 8) trans_acc<16, 0>(s, l, d, acc[J0 <= 8 ? 8 - J0 : 0]);
        if constexpr (J0 <= 9) trans_acc<16, 1>(s, l, d, acc[J0 <= 9 ? 9 - J0 : 0]);
        if constexpr (J0 <= 10) trans_acc<16, 2>(s, l, d, acc[J0 <= 10 ? 10 - J0 : 0]);
        trans_acc<16, 3>(s, l, d, acc[11 - J0]);
    }
    // every wavefront writes its own partial: index (group, wavefront)
    const double t1 = wave_sum((double)tsum);
#pragma unroll
    for (int a = 0; a < NJ; ++a) {
        const int j = J0 + a;
        const int q = j < c ? j : j - c + w;                 // the qubit behind tile bit j
        double* out = partial + ((r * n + q) * (u64)nblk + (u64)blockIdx.x * 4 + (t >> 6)) * 8;
        double tot[3];
#pragma unroll
        for (int b = 0; b < 3; ++b) tot[b] = wave_sum((double)acc[a][b]);
        if ((t & 63u) == 0) trans_store(out, tot[0], tot[1], tot[2], t1);
    }
}

// Where the 12 bits of a tile index come from when a wavefront reads the tile from LDS in runs of RB
// bits starting at tile bit R0: pos[0..RB) = the run, pos[RB..RB+6) = the lane bits, the rest = the
// step counter h.  The four low lane bits are placed so that, after the swizzle tau ^ ((tau >> 4) & 15),
// 16 consecutive lanes fall on 16 different 8-byte slots of a 128-byte row: into the free bits of the
// low nibble, and, for every low-nibble bit p the run occupies, into bit p + 4 (which the swizzle
// folds onto p).
template <int RB, int R0>
struct TransMap {
    int pos[12];
    constexpr TransMap() : pos{} {
        bool used[12] = {};
        int k = 0;
        for (int j = 0; j < RB; ++j) { pos[k++] = R0 + j; used[R0 + j] = true; }
        for (int p = 0; p < 4; ++p)
            if (!used[p]) { pos[k++] = p; used[p] = true; }
        for (int j = 0; j < RB; ++j)
            if (R0 + j < 4) { pos[k++] = R0 + j + 4; used[R0 + j + 4] = true; }
        for (int p = 0; p < 12; ++p)
            if (!used[p]) { pos[k++] = p; used[p] = true; }
    }
    // bits [first, first + count) of the source list take the low bits of v
    constexpr unsigned deposit(int first, int count, unsigned v) const {
        unsigned a = 0;
        for (int j = 0; j < count; ++j) a |= ((v >> j) & 1u) << pos[first + j];
        return a;
    }
};
__device__ constexpr unsigned trans_swz(unsigned tau) { return tau ^ ((tau >> 4) & 15u); }

// One wavefront, the whole tile in LDS, the qubits behind tile bits R0..R0+RB-1: 2^(6-RB) steps of one
// run per lane; the reads of a step are issued before the sums of the step before it.
template <int RB, int R0>
__device__ __forceinline__ void trans_wave(const float2* ps, const float2* lm, unsigned lane,
                                           float (&acc)[RB][3], float& tsum) {
    constexpr TransMap<RB, R0> map{};
    constexpr int NR = 1 << RB, HB = 6 - RB, NH = 1 << HB;
    unsigned lp = 0;
#pragma unroll
    for (int j = 0; j < 6; ++j) lp |= ((lane >> j) & 1u) << map.pos[RB + j];
    lp = trans_swz(lp);                              // the swizzle is linear over XOR
    float2 rs[2][NR], rl[2][NR];
    auto read_step = [&](int h, float2 (&a)[NR], float2 (&b)[NR]) __attribute__((always_inline)) {
        unsigned hp = 0;
#pragma unroll
        for (int j = 0; j < HB; ++j) hp |= (((unsigned)h >> j) & 1u) << map.pos[RB + 6 + j];
        const unsigned base = lp ^ trans_swz(hp);
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const unsigned ip = trans_swz(map.deposit(0, RB, (unsigned)i));
            a[i] = ps[base ^ ip];
            b[i] = lm[base ^ ip];
        }
    };
    auto sums = [&](const float2 (&a)[NR], const float2 (&b)[NR]) __attribute__((always_inline)) {
        float d[NR];
        trans_diag<NR>(a, b, d, tsum);
        trans_acc<NR, 0>(a, b, d, acc[0]);
        trans_acc<NR, 1>(a, b, d, acc[1]);
        if constexpr (RB > 2) trans_acc<NR, 2>(a, b, d, acc[RB > 2 ? 2 : 0]);
    };
    read_step(0, rs[0], rl[0]);
#pragma unroll 1
    for (int h = 0; h < NH; h += 2) {
        read_step(h + 1, rs[1], rl[1]);
        sums(rs[0], rl[0]);
        if (h + 2 < NH) read_step(h + 2, rs[0], rl[0]);
        sums(rs[1], rl[1]);
    }
}

// The sums for tile bits JB..11 (JB = 0 with RB = 3: contiguous tiles; JB = 4 with RB = 2: tiles with
// a window), of which bits >= j0 are wanted.  The tile of psi and of lambda goes from memory through
// registers into LDS (64 KiB); then every wavefront reads the whole tile in runs of its own RB bits
// (wavefront v: tile bits JB + RB v ...), so a lane carries accumulators for RB qubits only and the
// loads of the workgroup's next tile stay in flight meanwhile (the loop is rotated for that: load
// tile g, sums of tile g - 1, tile g into LDS).  Every wavefront sums d over the whole tile, so
// Im M11 = tsum - Im M00 holds per wavefront.  Output layout as k_trans_tile; the wavefronts that do not own
// a qubit write zeros for it.
template <int RB>
__global__ __launch_bounds__(256, 2) void k_trans_wave(const float2* psi0, const float2* lam0, int rstride,
                                                       int n, int c, int w, int j0, int per_group, int nblk,
                                                       double* partial) {
    __shared__ float2 ps[4096];
    __shared__ float2 lm[4096];                      // 64 KiB in all
    constexpr int JB = RB == 3 ? 0 : 4;
    const u64 r = blockIdx.y;
    const float2* psi = psi0 + ((rstride * r) << n);
    const float2* lam = lam0 + ((rstride * r) << n);
    const unsigned t = threadIdx.x, lane = t & 63u;
    const int wv = (int)(t >> 6);
    const unsigned cmask = (1u << c) - 1u;
    const int wc = w - c;
    float acc[RB][3];
    float tsum = 0.f;
#pragma unroll
    for (int a = 0; a < RB; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) acc[a][b] = 0.f;
    const unsigned tc = t ^ ((t >> 4) & 15u);        // swizzled lane part of the layout loaded from memory
    float2 s[16], l[16];                             // tau = i * 256 + t
    const u64 stride = c == 12 ? 256ull : (16ull << w);          // addressing as in k_trans_tile
    const unsigned kt8 = ((t & cmask) | ((t >> c) << w)) * 8u;
    const bool active = JB + RB * wv + RB - 1 >= j0;             // the wavefront owns a wanted bit
    for (int g = 0; g <= per_group; ++g) {
        if (g < per_group) {
            const u64 tb = (u64)blockIdx.x * per_group + g;      // tile of the row
            const u64 base = ((tb & ((1ull << wc) - 1ull)) << c) | ((tb >> wc) << (w + 12 - c));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s[i] = load_f2(uniform_ptr(psi + (base + (u64)i * stride)), kt8);
                l[i] = load_f2(uniform_ptr(lam + (base + (u64)i * stride)), kt8);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (g > 0 && active) {
            switch (wv) {
                case 0: trans_wave<RB, JB>(ps, lm, lane, acc, tsum); break;
                case 1: trans_wave<RB, JB + RB>(ps, lm, lane, acc, tsum); break;
                case 2: trans_wave<RB, JB + 2 * RB>(ps, lm, lane, acc, tsum); break;
                default: trans_wave<RB, JB + 3 * RB>(ps, lm, lane, acc, tsum); break;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (g < per_group) {
            if (g) __syncthreads();                  // the previous tile has been read by everyone
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                ps[(unsigned)i * 256u + tc] = s[i];
                lm[(unsigned)i * 256u + tc] = l[i];
            }
            __syncthreads();
        }
    }
    const double t1 = wave_sum((double)tsum);
    double tot[RB][3];
#pragma unroll
    for (int a = 0; a < RB; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) tot[a][b] = wave_sum((double)acc[a][b]);
    if (lane != 0) return;
    for (int j = j0 > JB ? j0 : JB; j < 12; ++j) {
        const int q = j < c ? j : j - c + w;                 // the qubit behind tile bit j
        double* out = partial + ((r * n + q) * (u64)nblk + (u64)blockIdx.x * 4 + wv) * 8;
        if ((j - JB) / RB != wv) {
            for (int b = 0; b < 8; ++b) out[b] = 0.0;
            continue;
        }
#pragma unroll
        for (int a = 0; a < RB; ++a)
            if ((j - JB) % RB == a) trans_store(out, tot[a][0], tot[a][1], tot[a][2], t1);
    }
}

// Adds the nblk partials of every (row pair, qubit): one wavefront per job, lanes stride over the
// partials, fixed order.  out: [jobs][8].
__global__ __launch_bounds__(256) void k_trans_finish(const double* partial, int nblk, u64 jobs, double* out) {
    const u64 job = (u64)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (job >= jobs) return;
    const int lane = threadIdx.x & 63;
    double acc[8];
    for (int j = 0; j < 8; ++j) acc[j] = 0.0;
    const double* p = partial + job * (u64)nblk * 8;
    for (int b = lane; b < nblk; b += 64)
        for (int j = 0; j < 8; ++j) acc[j] += p[(u64)b * 8 + j];
    for (int j = 0; j < 8; ++j) {
        const double t = wave_sum(acc[j]);
        if (lane == 0) out[job * 8 + j] = t;
    }
}

// Gradients of one layer from the transition matrices: thread = (row pair, slot, qubit).  With
// W = R_{s-1} ... R_0 (the slots before s on that qubit) the derivative with respect to the angle of
// slot s is 2 Re sum_ab Bt[a][b] M[a][b], Bt = W^dagger (-i/2 P_s) W.  Written as f+ = g, f- = -g so
// that the same finishing kernels as for the shift rule apply (they halve the difference and
// multiply re-upload weights by the feature).
__global__ __launch_bounds__(256) void k_adj_layer(const double* partial, int nblk, CircDev c, int layer,
                                                   const float* params, const float* feats, u64 sample0,
                                                   u64 pairs_rows, u64 P, double* f) {
    const u64 idx = (u64)blockIdx.x * 256 + threadIdx.x;
    const int slots = c.reupload + c.n_rot;
    const u64 per = (u64)slots * c.n;
    if (idx >= pairs_rows * per) return;
    const u64 r = idx / per;
    const int s = (int)((idx % per) / c.n), q = (int)(idx % c.n);
    const u64 sample = sample0 + r;
    double M[8];
    for (int j = 0; j < 8; ++j) M[j] = 0.0;
    const double* pp = partial + ((r * c.n + q) * (u64)nblk) * 8;
    for (int b = 0; b < nblk; ++b)
        for (int j = 0; j < 8; ++j) M[j] += pp[(u64)b * 8 + j];
    M2 w;
    for (int k = 0; k < 4; ++k) { w.r[k] = (k == 0 || k == 3) ? 1.0 : 0.0; w.i[k] = 0.0; }
    int axis = QSV_RX;
    for (int sl = 0; sl <= s; ++sl) {
        double t = (double)params[((u64)layer * slots + sl) * c.n + q];
        if (c.reupload && sl == 0) { t *= (double)feats[sample * c.n + q]; axis = QSV_RX; }
        else axis = c.rot[sl - c.reupload];
        if (sl < s) w = mul_m(rot_m(axis, t), w);
    }
    // G = -i/2 P for the axis of slot s
    M2 g;
    for (int k = 0; k < 4; ++k) { g.r[k] = 0.0; g.i[k] = 0.0; }
    if (axis == QSV_RX) { g.i[1] = -0.5; g.i[2] = -0.5; }
    else if (axis == QSV_RY) { g.r[1] = -0.5; g.r[2] = 0.5; }
    else { g.i[0] = -0.5; g.i[3] = 0.5; }
    M2 wd;   // W^dagger
    wd.r[0] = w.r[0]; wd.i[0] = -w.i[0]; wd.r[1] = w.r[2]; wd.i[1] = -w.i[2];
    wd.r[2] = w.r[1]; wd.i[2] = -w.i[1]; wd.r[3] = w.r[3]; wd.i[3] = -w.i[3];
    const M2 bt = mul_m(wd, mul_m(g, w));
    double acc = 0.0;
    for (int k = 0; k < 4; ++k) acc += bt.r[k] * M[2 * k] - bt.i[k] * M[2 * k + 1];
    const u64 p = ((u64)layer * slots + s) * c.n + q;
    double* fb = f + sample * (2 * P + 1);
    fb[2 * p] = 2.0 * acc;
    fb[2 * p + 1] = -2.0 * acc;
}

// ------------------------------------------------------------------------------------------
// Optimiser steps on the parameter vector, in double, stored as float.
__global__ __launch_bounds__(256) void k_sgd(float* p, const float* g, u64 count, double lr) {
    const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = (float)((double)p[i] - lr * (double)g[i]);
}

__global__ __launch_bounds__(256) void k_adam(float* p, const float* g, float* m, float* v, u64 count,
                                              double lr, double b1, double b2, double eps, double c1,
                                              double c2) {
    const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const double gi = (double)g[i];
    const double mi = b1 * (double)m[i] + (1.0 - b1) * gi;
    const double vi = b2 * (double)v[i] + (1.0 - b2) * gi * gi;
    p[i] = (float)((double)p[i] - lr * (mi / c1) / (sqrt(vi / c2) + eps));
    m[i] = (float)mi;
    v[i] = (float)vi;
}

// ------------------------------------------------------------------------------------------
// A whole small workload in one launch (at most 10 qubits): amplitude encoding, the circuit (and,
// as decoder, its exact inverse), the final state and one measurement.  A thread keeps 2^R
// amplitudes in registers (index bits 0..R-1), the index bits above are bits of the thread number:
// up to six inside the wavefront, the rest across the wavefronts of the workgroup; with fewer than
// six the spare lane bits number the samples that share the wavefront.  A gate on a register bit
// pairs registers; on a lane bit it exchanges with the partner lane (DPP, the LDS crossbar);
// on a bit across wavefronts it exchanges through LDS.  Nothing goes to device memory between the
// gates.  R = 2, 3 or 4 is chosen so that the batch gives the chip enough wavefronts (a lone
// wavefront on a SIMD issues one vector instruction in about eight cycles, four of them one every
// three).  The matrices are built once per workgroup, one per thread at a time, and kept in LDS.
template <int R> struct Amps { float re[1 << R], im[1 << R]; };  // every index is a compile-time constant after unrolling

__device__ __forceinline__ float lane_xchg(int addr, float v) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(v)));
}

// The value that the lane whose number differs in bit B holds.  Bits 0..3: DPP moves (inside a row
// of 16 lanes; XOR 4 = reversal of 8 then of 4, XOR 8 = reversal of 16 then of 8); bit 4: the
// swizzle of the LDS crossbar; bit 5: ds_bpermute (addr = 4 * partner lane).
template <int B>
__device__ __forceinline__ float lane_flip(float v, int addr) {
    const int x = __float_as_int(v);
    if constexpr (B == 0) return __int_as_float(__builtin_amdgcn_mov_dpp(x, 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
    else if constexpr (B == 1) return __int_as_float(__builtin_amdgcn_mov_dpp(x, 0x4E, 0xf, 0xf, true));   // [2,3,0,1]
    else if constexpr (B == 2)
        return __int_as_float(__builtin_amdgcn_mov_dpp(__builtin_amdgcn_mov_dpp(x, 0x141, 0xf, 0xf, true), 0x1B, 0xf, 0xf, true));
    else if constexpr (B == 3)
        return __int_as_float(__builtin_amdgcn_mov_dpp(__builtin_amdgcn_mov_dpp(x, 0x140, 0xf, 0xf, true), 0x141, 0xf, 0xf, true));
    else if constexpr (B == 4) return __int_as_float(__builtin_amdgcn_ds_swizzle(x, 0x401F));           // xor 16 within 32 lanes
    else return lane_xchg(addr, v);
}

// Exchange between the wavefronts of a workgroup: every thread puts its registers into the current
// one of two buffers [2 * 2^R][threads], and after the barrier reads another thread's.  The
// buffers alternate, so one barrier per exchange is enough (whoever writes a buffer again has
// passed the barrier of the exchange in between, which every reader of the old contents reaches
// only after reading).
struct Xchg { float* buf; int threads, cur; };

template <int R>
__device__ __forceinline__ void xchg_through_lds(const Amps<R>& a, float* pr, float* pi, Xchg& x, int tid, int src) {
    float* b = x.buf + (size_t)x.cur * (2 << R) * x.threads;
#pragma unroll
    for (int k = 0; k < (1 << R); ++k) {
        b[(2 * k) * x.threads + tid] = a.re[k];
        b[(2 * k + 1) * x.threads + tid] = a.im[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < (1 << R); ++k) {
        pr[k] = b[(2 * k) * x.threads + src];
        pi[k] = b[(2 * k + 1) * x.threads + src];
    }
    x.cur ^= 1;
}

// m = (m00r, m00i, m01r, m01i, m10r, m10i, m11r, m11i)
template <int R, int J>
__device__ __forceinline__ void small_u_reg(Amps<R>& a, const float* m) {
#pragma unroll
    for (int k = 0; k < (1 << R); ++k) {
        if (k & (1 << J)) continue;
        const int k1 = k | (1 << J);
        const float ar = a.re[k], ai = a.im[k], br = a.re[k1], bi = a.im[k1];
        a.re[k] = m[0] * ar - m[1] * ai + m[2] * br - m[3] * bi;
        a.im[k] = m[0] * ai + m[1] * ar + m[2] * bi + m[3] * br;
        a.re[k1] = m[4] * ar - m[5] * ai + m[6] * br - m[7] * bi;
        a.im[k1] = m[4] * ai + m[5] * ar + m[6] * bi + m[7] * br;
    }
}

// The qubit is bit B of the thread number: this thread holds the amplitudes with the bit equal to
// its own, the partner thread the ones with the other value.
template <int R, int B>
__device__ __forceinline__ void small_u_thr(Amps<R>& a, const float* m, int tid, Xchg& x) {
    constexpr int NR = 1 << R;
    const bool bit = (tid >> B) & 1;
    const float sr = bit ? m[6] : m[0], si = bit ? m[7] : m[1];   // row `bit`, own column
    const float qr = bit ? m[4] : m[2], qi = bit ? m[5] : m[3];   // row `bit`, the partner's column
    float pr[NR], pi[NR];                    // all exchanges first: their latencies overlap
    if constexpr (B < 6) {
        const int addr = ((tid & 63) ^ (1 << B)) << 2;
#pragma unroll
        for (int k = 0; k < NR; ++k) { pr[k] = lane_flip<B>(a.re[k], addr); pi[k] = lane_flip<B>(a.im[k], addr); }
    } else {
        xchg_through_lds<R>(a, pr, pi, x, tid, tid ^ (1 << B));
    }
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const float ar = a.re[k], ai = a.im[k];
        a.re[k] = sr * ar - si * ai + qr * pr[k] - qi * pi[k];
        a.im[k] = sr * ai + si * ar + qr * pi[k] + qi * pr[k];
    }
}

template <int R, int C, int T>
__device__ __forceinline__ void small_cx_rr(Amps<R>& a) {
    if constexpr (C < R && T < R) {
#pragma unroll
        for (int k = 0; k < (1 << R); ++k) {
            if (!(k & (1 << C)) || (k & (1 << T))) continue;
            const int k1 = k | (1 << T);
            const float r = a.re[k], i = a.im[k];
            a.re[k] = a.re[k1]; a.im[k] = a.im[k1];
            a.re[k1] = r; a.im[k1] = i;
        }
    }
}

template <int R>
__device__ __forceinline__ void small_cx_to_reg0(Amps<R>& a, bool ctrl) {  // control on a thread bit, target register bit 0
#pragma unroll
    for (int k = 0; k < (1 << R); k += 2) {
        const float r0 = a.re[k], i0 = a.im[k], r1 = a.re[k + 1], i1 = a.im[k + 1];
        a.re[k] = ctrl ? r1 : r0; a.im[k] = ctrl ? i1 : i0;
        a.re[k + 1] = ctrl ? r0 : r1; a.im[k + 1] = ctrl ? i0 : i1;
    }
}

// The CNOT ring on n qubits, control q, target q + 1 (the last one's target is qubit 0), in order,
// or with reverse = true in the opposite order (the ring's inverse).  The CNOTs between register
// bits rename registers; the one from the top register bit to thread bit 0 exchanges half of the
// registers with the neighbouring lane; the CNOTs between thread bits are together one
// permutation of the threads (src_f / src_r: the thread each one reads from), done by
// ds_bpermute inside a wavefront and through LDS across wavefronts; the closing one swaps register
// pairs in the threads whose top index bit is set.
template <int R>
__device__ __forceinline__ void small_ring(Amps<R>& a, int n, int tid, int tb, bool reverse, int src_f, int src_r,
                                           Xchg& x) {
    constexpr int NR = 1 << R;
    auto wrap = [&]() {
        if (n > R) small_cx_to_reg0<R>(a, (tid >> (tb - 1)) & 1);
        else if (n == 2) small_cx_rr<R, 1, 0>(a);
        else if (n == 3) small_cx_rr<R, 2, 0>(a);
        else if (n == 4) small_cx_rr<R, 3, 0>(a);
    };
    auto bridge = [&]() {                          // control register bit R - 1, target thread bit 0
        if (n > R) {
#pragma unroll
            for (int k = NR / 2; k < NR; ++k) { a.re[k] = lane_flip<0>(a.re[k], 0); a.im[k] = lane_flip<0>(a.im[k], 0); }
        }
    };
    auto chain = [&](int src) {
        if (tb < 2) return;
        float pr[NR], pi[NR];
        if (tb <= 6) {
            const int addr = src << 2;             // src differs from tid in lane bits only
#pragma unroll
            for (int k = 0; k < NR; ++k) { pr[k] = lane_xchg(addr, a.re[k]); pi[k] = lane_xchg(addr, a.im[k]); }
        } else {
            xchg_through_lds<R>(a, pr, pi, x, tid, src);
        }
#pragma unroll
        for (int k = 0; k < NR; ++k) { a.re[k] = pr[k]; a.im[k] = pi[k]; }
    };
    if (!reverse) {
        if (n >= 2) small_cx_rr<R, 0, 1>(a);
        if (n >= 3) small_cx_rr<R, 1, 2>(a);
        if (n >= 4) small_cx_rr<R, 2, 3>(a);
        bridge();
        chain(src_f);
        wrap();
    } else {
        wrap();
        chain(src_r);
        bridge();
        if (n >= 4) small_cx_rr<R, 2, 3>(a);
        if (n >= 3) small_cx_rr<R, 1, 2>(a);
        if (n >= 2) small_cx_rr<R, 0, 1>(a);
    }
}

// CZ on qubits q and q + 1 for q = 0..n-2 (the gates commute, so the order does not matter): the
// sign of an amplitude changes once for every pair of neighbouring set bits of its index.
template <int R>
__device__ __forceinline__ void small_cz_ladder(Amps<R>& a, int n, int ti) {
    const int mask = (1 << (n - 1)) - 1;           // pairs (q, q + 1) for q = 0..n-2
#pragma unroll
    for (int k = 0; k < (1 << R); ++k) {
        const int idx = (ti << R) | k;
        const bool f = __builtin_popcount(idx & (idx >> 1) & mask) & 1;
        a.re[k] = f ? -a.re[k] : a.re[k];
        a.im[k] = f ? -a.im[k] : a.im[k];
    }
}

struct SmallArgs {
    const float* x;        // [batch][dim]
    int64_t dim, batch;
    CircDev c;
    int entangler;         // qsv_ent
    const float* params;
    const float* feats;
    int pass_first, pass_last;  // 0 = the circuit, 1 = its inverse: (0,0) circuit, (0,1) circuit then inverse, (1,1) inverse
    int from_state;        // 1: start from the amplitudes in `state` instead of encoding x
    int kind;              // QSV_M_PROBS, QSV_M_EXPZ_ALL, or 0: no measurement
    float2* state;         // [batch][2^n], receives the final state
    float* out;            // probabilities [batch][2^n] or expectations [batch][n]
    float* norm_out;       // [batch] or NULL
    int mat_floats;        // LDS floats set aside for the workgroup's matrices (a multiple of 8)
};

// dynamic LDS: [64] doubles for sums across wavefronts, the workgroup's matrices, then the exchange buffers
template <int R>
__global__ __launch_bounds__(256) void k_forward_small(SmallArgs a) {
    constexpr int NR = 1 << R;
    extern __shared__ __align__(16) unsigned char small_lds[];
    double* red = reinterpret_cast<double*>(small_lds);
    float* mats = reinterpret_cast<float*>(small_lds + 64 * sizeof(double));
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = a.c.n, L = a.c.n_layers;
    const int tb = n > R ? n - R : 0;            // index bits held by the thread number
    const int lb = tb < 6 ? tb : 6;              // of which inside the wavefront
    const int n_waves = (int)blockDim.x >> 6;    // 2^(tb - 6) when tb > 6, else 1
    const int rows_g = 64 >> lb;                 // samples per workgroup (1 when tb >= 6)
    const int r_in = tb < 6 ? lane >> tb : 0;
    const int ti = tid & ((1 << tb) - 1);
    Xchg xc;
    xc.buf = mats + a.mat_floats;
    xc.threads = (int)blockDim.x;
    xc.cur = 0;
    const int64_t first = (int64_t)blockIdx.x * rows_g;
    const int64_t sample = first + r_in;
    const bool live = sample < a.batch;
    const int per = L * n;
    const bool has_u = a.c.reupload + a.c.n_rot > 0;
    if (has_u) {
        const int rows_m = a.c.reupload ? rows_g : 1;
        for (int i = tid; i < rows_m * per; i += (int)blockDim.x) {
            const int r = i / per, lq = i % per;
            const int64_t s = first + r < a.batch ? first + r : a.batch - 1;
            const M2 u = fused_raw(a.c, a.params, a.feats, (u64)s, lq / n, lq % n, -1, 0.0, 0);
            float* o = mats + (size_t)i * 8;
#pragma unroll
            for (int k = 0; k < 4; ++k) { o[2 * k] = (float)u.r[k]; o[2 * k + 1] = (float)u.i[k]; }
        }
    }
    // amplitude encoding: x / ||x||, the norm in double (or the amplitudes the state already holds)
    Amps<R> A;
    if (a.from_state) {
        const float2* srow = a.state + ((live ? sample : 0) << n) + ((int64_t)ti << R);
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int64_t idx = ((int64_t)ti << R) | k;
            const float2 v = (live && idx < ((int64_t)1 << n)) ? srow[k] : make_float2(0.f, 0.f);
            A.re[k] = v.x; A.im[k] = v.y;
        }
    } else {
        const float* xb = a.x + (live ? sample : 0) * a.dim;
        float xv[NR];
        double ss = 0.0;
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int64_t idx = ((int64_t)ti << R) | k;
            const float v = (live && idx < a.dim) ? xb[idx] : 0.f;
            xv[k] = v;
            ss += (double)v * (double)v;
        }
#pragma unroll
        for (int b = 0; b < 6; ++b)
            if (b < lb) ss += __shfl_xor(ss, 1 << b, 64);
        if (n_waves > 1) {
            if (lane == 0) red[wave] = ss;
            __syncthreads();
            ss = 0.0;
            for (int w = 0; w < n_waves; ++w) ss += red[w];
        }
        const double nrm = sqrt(ss);
        const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
#pragma unroll
        for (int k = 0; k < NR; ++k) { A.re[k] = (float)((double)xv[k] * inv); A.im[k] = 0.f; }
        if (a.norm_out && live && ti == 0) a.norm_out[sample] = (float)nrm;
    }
    __syncthreads();                             // the matrices are in LDS; red[] may be written again
    const float* mrow = mats + (size_t)(a.c.reupload ? r_in * per : 0) * 8;
    // Thread permutations of the ring's CNOTs between thread bits (qubits R..n-1): an amplitude in
    // thread j moves to C(j), so afterwards thread j holds what thread C_first(...C_last(j)) held.
    int src_f = tid, src_r = tid;
    for (int b = tb - 2; b >= 0; --b) src_f ^= ((src_f >> b) & 1) << (b + 1);
    for (int b = 0; b + 1 < tb; ++b) src_r ^= ((src_r >> b) & 1) << (b + 1);
    // the gates: per layer the unitaries then the entangler; in the decoder layers last to first,
    // the entangler's gates in reverse order first, then the conjugate-transposed unitaries
    for (int pass = a.pass_first; pass <= a.pass_last; ++pass) {
        for (int ll = 0; ll < L; ++ll) {
            const int l = pass ? L - 1 - ll : ll;
            for (int stage = 0; stage < 2; ++stage) {
                if ((stage == 0) == (pass == 1)) {
                    if (a.entangler == QSV_ENT_CNOT_RING) small_ring<R>(A, n, tid, tb, pass != 0, src_f, src_r, xc);
                    else if (a.entangler == QSV_ENT_CZ_LADDER) small_cz_ladder<R>(A, n, ti);
                } else if (has_u) {
                    const float* ml = mrow + (size_t)l * n * 8;
                    auto load_m = [&](int q, float* m) {
                        const float4 lo = *reinterpret_cast<const float4*>(ml + q * 8);
                        const float4 hi = *reinterpret_cast<const float4*>(ml + q * 8 + 4);
                        if (!pass) {
                            m[0] = lo.x; m[1] = lo.y; m[2] = lo.z; m[3] = lo.w;
                            m[4] = hi.x; m[5] = hi.y; m[6] = hi.z; m[7] = hi.w;
                        } else {                 // conjugate transpose
                            m[0] = lo.x; m[1] = -lo.y; m[2] = hi.x; m[3] = -hi.y;
                            m[4] = lo.z; m[5] = -lo.w; m[6] = hi.z; m[7] = -hi.w;
                        }
                    };
                    float m[8];
#define QSV_SMALL_U(Q)                                                      \
    if (n > Q) {                                                            \
        load_m(Q, m);                                                       \
        if constexpr (Q < R) small_u_reg<R, Q>(A, m);                       \
        else if constexpr (Q - R < 8) small_u_thr<R, Q - R>(A, m, tid, xc); \
    }
                    QSV_SMALL_U(0) QSV_SMALL_U(1) QSV_SMALL_U(2) QSV_SMALL_U(3) QSV_SMALL_U(4)
                    QSV_SMALL_U(5) QSV_SMALL_U(6) QSV_SMALL_U(7) QSV_SMALL_U(8) QSV_SMALL_U(9)
#undef QSV_SMALL_U
                }
            }
        }
    }
    // final state and the measurement
    const int dimn = 1 << n;
    if (live) {
        float2* srow = a.state + (sample << n) + ((int64_t)ti << R);
        if (n >= R) {
#pragma unroll
            for (int k = 0; k < NR; k += 2)
                *reinterpret_cast<float4*>(srow + k) = make_float4(A.re[k], A.im[k], A.re[k + 1], A.im[k + 1]);
        } else {
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (k < dimn) srow[k] = make_float2(A.re[k], A.im[k]);
        }
    }
    if (a.kind == 0) return;
    float p[NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) p[k] = prob32(make_float2(A.re[k], A.im[k]));
    if (a.kind == QSV_M_PROBS) {
        if (live) {
            float* prow = a.out + (sample << n) + ((int64_t)ti << R);
            if (n >= R) {
#pragma unroll
                for (int k = 0; k < NR; k += 4)
                    *reinterpret_cast<float4*>(prow + k) = make_float4(p[k], p[k + 1], p[k + 2], p[k + 3]);
            } else {
#pragma unroll
                for (int k = 0; k < NR; ++k)
                    if (k < dimn) prow[k] = p[k];
            }
        }
        return;
    }
    // <Z_q> for every qubit: signed sums in double, combined over the threads of the sample
    double T = 0.0, zr[R], zl[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int j = 0; j < R; ++j) zr[j] = 0.0;
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const double pk = (double)p[k];
        T += pk;
#pragma unroll
        for (int j = 0; j < R; ++j) zr[j] += ((k >> j) & 1) ? -pk : pk;
    }
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        if (b < lb) {
            const double Tp = __shfl_xor(T, 1 << b, 64);
#pragma unroll
            for (int j = 0; j < R; ++j) zr[j] += __shfl_xor(zr[j], 1 << b, 64);
#pragma unroll
            for (int j = 0; j < 6; ++j)
                if (j < b) zl[j] += __shfl_xor(zl[j], 1 << b, 64);
            zl[b] = ((lane >> b) & 1) ? Tp - T : T - Tp;
            T += Tp;
        }
    }
    if (n_waves == 1) {
        if (live && ti == 0) {
            float* orow = a.out + sample * n;
#pragma unroll
            for (int q = 0; q < R; ++q)            // qubits behind register bits
                if (q < n) orow[q] = (float)zr[q];
#pragma unroll
            for (int b = 0; b < 6; ++b)            // qubits behind lane bits
                if (R + b < n) orow[R + b] = (float)zl[b];
        }
        return;
    }
    // several wavefronts hold the sample: totals per wavefront through LDS, thread q adds up qubit q
    // (qubits beyond the lane bits take the wavefront totals signed by the wavefront's number)
    if (lane == 0) {
        double* o = red + wave * 16;
        o[0] = T;
#pragma unroll
        for (int j = 0; j < R; ++j) o[1 + j] = zr[j];
#pragma unroll
        for (int j = 0; j < 6; ++j) o[1 + R + j] = zl[j];
    }
    __syncthreads();
    if (tid < n && live) {
        const int q = tid;
        double acc = 0.0;
        for (int w = 0; w < n_waves; ++w) {
            const double* o = red + w * 16;
            if (q < R + 6) acc += o[1 + q];
            else acc += ((w >> (q - R - 6)) & 1) ? -o[0] : o[0];
        }
        a.out[sample * n + q] = (float)acc;
    }
}

inline unsigned blocks_for(u64 items, unsigned per) { return (unsigned)((items + per - 1) / per); }

// grid of the reduction kernels: chunks in x, rows over y and z (see grid_row)
inline dim3 rows_grid(unsigned nblk, u64 rows) {
    const unsigned gy = (unsigned)(rows < 32768 ? rows : 32768);
    return dim3(nblk, gy, (unsigned)((rows + gy - 1) / gy));
}

}  // namespace

// ============================================================================================
// Launchers.
template <int T, int PLANES>
static hipError_t set_attr_for() {
    const int bytes = PLANES * (1 << T) * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_pass<T, false, PLANES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_pass<T, true, PLANES>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// the two variants that use 64 KiB of dynamic LDS
hipError_t set_pass_attributes() {
    const hipError_t e = set_attr_for<13, 2>();
    return e != hipSuccess ? e : set_attr_for<14, 1>();
}

template <int T, int PLANES>
static void launch_pass_t(const PassArgs& a, dim3 grid, hipStream_t st) {
    const size_t lds = (size_t)PLANES * ((size_t)1 << T) * sizeof(float);
    if (a.n >= T) hipLaunchKernelGGL((k_pass<T, false, PLANES>), grid, dim3(1 << (T - R)), lds, st, a);
    else hipLaunchKernelGGL((k_pass<T, true, PLANES>), grid, dim3(1 << (T - R)), lds, st, a);
}

hipError_t launch_pass(int tile, int planes, const PassArgs& a, uint64_t n_tiles, hipStream_t st) {
    if (n_tiles == 0 || n_tiles > 0x7fffffffull) return hipErrorInvalidValue;
    if (planes != 1 && planes != 2) return hipErrorInvalidValue;
    if (tile == 14) planes = 1;   // the largest tile exists with one plane only
    const dim3 grid((unsigned)n_tiles);
    switch (tile * 2 + planes - 1) {
        case 20: launch_pass_t<10, 1>(a, grid, st); break;
        case 21: launch_pass_t<10, 2>(a, grid, st); break;
        case 22: launch_pass_t<11, 1>(a, grid, st); break;
        case 23: launch_pass_t<11, 2>(a, grid, st); break;
        case 24: launch_pass_t<12, 1>(a, grid, st); break;
        case 25: launch_pass_t<12, 2>(a, grid, st); break;
        case 26: launch_pass_t<13, 1>(a, grid, st); break;
        case 27: launch_pass_t<13, 2>(a, grid, st); break;
        case 28: launch_pass_t<14, 1>(a, grid, st); break;   // two planes of 2^14 floats do not fit the offset fields
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_naive_u(float2* state, int64_t rows, int n, int q, const float* mats,
                          const float* ovr, int mat_id, int n_mats, int rowdep, const RowMap& rm,
                          hipStream_t st) {
    const u64 pairs = ((u64)rows << n) >> 1;
    hipLaunchKernelGGL(k_naive_u, dim3(blocks_for(pairs, 256)), dim3(256), 0, st, state, pairs, n, q,
                       mats, ovr, mat_id, n_mats, rowdep, rm);
    return hipGetLastError();
}

hipError_t launch_naive_cnot(float2* state, int64_t rows, int n, int ctrl, int tgt, hipStream_t st) {
    const u64 total = (u64)rows << n;
    hipLaunchKernelGGL(k_naive_cnot, dim3(blocks_for(total, 256)), dim3(256), 0, st, state, total, ctrl,
                       tgt);
    return hipGetLastError();
}

hipError_t launch_naive_cz_ladder(float2* state, int64_t rows, int n, hipStream_t st) {
    const u64 total = (u64)rows << n;
    hipLaunchKernelGGL(k_naive_cz_ladder, dim3(blocks_for(total, 256)), dim3(256), 0, st, state, total,
                       n);
    return hipGetLastError();
}

hipError_t launch_build_mats(const CircDev& c, const float* params, const float* feats,
                             int64_t samples, int inverse, const int* order, const int* exec_of, float* out,
                             double* side, hipStream_t st, int period) {
    if (period < 0 || (period > 0 && period != c.n)) return hipErrorInvalidValue;
    const u64 tables = (u64)(c.reupload ? samples : 1);
    const u64 count = tables * c.n_layers * c.n;
    if (count == 0) return hipSuccess;
    if ((order == nullptr) != (exec_of == nullptr)) return hipErrorInvalidValue;
    if (!c.reupload && c.n <= 8) {   // few qubits: the serial factor loop is shorter than a second launch
        hipLaunchKernelGGL(k_build_mats_shared, dim3(blocks_for(count, 256)), dim3(256), 0, st, c, params,
                           count, inverse, order, period, out);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_build_mats, dim3(blocks_for(count, 256)), dim3(256), 0, st, c, params, feats,
                       count, inverse, order, period, out, side);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_build_mats_last, dim3(blocks_for(tables * c.n_layers, 256)), dim3(256), 0, st, c,
                       tables, exec_of, period, out, side);
    return hipGetLastError();
}

hipError_t launch_build_shifted(const CircDev& c, const float* params, const float* feats,
                                int64_t samples, float* out, hipStream_t st) {
    const u64 two_p = 2ull * c.n_layers * c.slots() * c.n;
    const u64 count = (u64)(c.reupload ? samples : 1) * two_p;
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(k_build_shifted, dim3(blocks_for(count, 256)), dim3(256), 0, st, c, params,
                       feats, count, out);
    return hipGetLastError();
}

// ||x_b|| of every sample: inv_norm [samples] (0 for a zero vector), norm_out optional.  One launch
// when a sample fits one block, else block partials and a finishing launch.
hipError_t launch_norms(const float* x, int64_t samples, int64_t dim, double* partial, int nblk,
                        double* inv_norm, float* norm_out, hipStream_t st) {
    const bool one = nblk == 1;
    hipLaunchKernelGGL(k_sumsq, rows_grid(nblk, (u64)samples), dim3(256), 0, st, x, (u64)samples, (u64)dim, partial, nblk,
                       one ? inv_norm : (double*)nullptr, one ? norm_out : (float*)nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || one) return e;
    hipLaunchKernelGGL(k_norm_finish, dim3((unsigned)samples), dim3(256), 0, st, partial, nblk,
                       inv_norm, norm_out);
    return hipGetLastError();
}

hipError_t launch_encode_small(const float* x, int64_t samples, int64_t dim, int n, double* inv_norm, float* norm_out,
                               float2* state, hipStream_t st) {
    if (dim > 4096 || n > 12) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_encode_small, rows_grid(1, (u64)samples), dim3(256), 0, st, x, (u64)samples, (u64)dim, n,
                       inv_norm, norm_out, state);
    return hipGetLastError();
}

hipError_t launch_forward_small(int regs, const float* x, int64_t dim, int64_t batch, const CircDev& c, int entangler,
                                const float* params, const float* feats, int pass_first, int pass_last, int kind,
                                float2* state, float* out, float* norm_out, hipStream_t st) {
    if (c.n < 1 || c.n > kSmallMaxQubits || batch < 1) return hipErrorInvalidValue;
    if (x && (dim < 1 || dim > ((int64_t)1 << c.n))) return hipErrorInvalidValue;
    if (pass_first < 0 || pass_last > 1 || pass_first > pass_last || (kind != 0 && !out)) return hipErrorInvalidValue;
    if (regs < 2 || regs > 4 || c.n - regs > 8) return hipErrorInvalidValue;
    if (small_mats_per_group(c, regs) > kSmallMats) return hipErrorInvalidValue;
    const int rows_g = small_rows_per_group(c.n, regs);
    const int tb = c.n > regs ? c.n - regs : 0;
    const unsigned threads = tb > 6 ? 64u << (tb - 6) : 64u;
    SmallArgs a;
    a.x = x; a.dim = dim; a.batch = batch; a.c = c; a.entangler = entangler; a.params = params; a.feats = feats;
    a.pass_first = pass_first; a.pass_last = pass_last; a.from_state = x ? 0 : 1; a.kind = kind;
    a.state = state; a.out = out; a.norm_out = norm_out;
    const int64_t blocks = (batch + rows_g - 1) / rows_g;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    // sums across wavefronts, the matrices (only as many as this circuit has: LDS per workgroup decides how
    // many workgroups a CU holds), and (several wavefronts per sample only) two exchange buffers
    a.mat_floats = (int)small_mats_per_group(c, regs) * 8;
    size_t lds = 64 * sizeof(double) + (size_t)a.mat_floats * sizeof(float);
    if (threads > 64) lds += 2 * (size_t)(2 << regs) * threads * sizeof(float);
    const dim3 grid((unsigned)blocks), block(threads);
    switch (regs) {
        case 2: hipLaunchKernelGGL(k_forward_small<2>, grid, block, lds, st, a); break;
        case 3: hipLaunchKernelGGL(k_forward_small<3>, grid, block, lds, st, a); break;
        default: hipLaunchKernelGGL(k_forward_small<4>, grid, block, lds, st, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_encode_write(const float* x, int64_t dim, int n, int64_t rows, const double* inv_norm,
                               const RowMap& rm, float2* state, hipStream_t st) {
    const u64 total = (u64)rows << n;
    hipLaunchKernelGGL(k_encode_write, dim3(blocks_for(total / 2, 256)), dim3(256), 0, st, x, (u64)dim,
                       n, total, inv_norm, rm, state);
    return hipGetLastError();
}

hipError_t launch_probs(const float2* state, uint64_t total, float* out, hipStream_t st) {
    hipLaunchKernelGGL(k_probs, dim3(blocks_for(total / 2, 256)), dim3(256), 0, st, state, (u64)total,
                       out);
    return hipGetLastError();
}

static inline int chunk_blocks(int bits) { return bits > CHUNK_BITS ? 1 << (bits - CHUNK_BITS) : 1; }

hipError_t launch_expz_block(const float2* state, int64_t rows, int n, double* partial, hipStream_t st) {
    const int nblk = chunk_blocks(n);
    hipLaunchKernelGGL(k_expz_block, rows_grid(nblk, (u64)rows), dim3(256), 0, st, state, (u64)rows, n, nblk,
                       partial, (float*)nullptr, -1);
    return hipGetLastError();
}

hipError_t launch_expz_small(const float2* state, int64_t rows, int n, int q_only, float* out_f, hipStream_t st) {
    if (chunk_blocks(n) != 1 || !out_f || q_only >= n) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_expz_block, rows_grid(1, (u64)rows), dim3(256), 0, st, state, (u64)rows, n, 1,
                       (double*)nullptr, out_f, q_only);
    return hipGetLastError();
}

hipError_t launch_expz_finish(const double* partial, int64_t rows, int n, int q_only, float* out_f,
                              double* out_d, hipStream_t st) {
    const u64 jobs = (u64)rows * (q_only >= 0 ? 1 : n);
    hipLaunchKernelGGL(k_expz_finish, dim3(blocks_for(jobs, 4)), dim3(256), 0, st, partial, (u64)rows, n,
                       chunk_blocks(n), q_only, out_f, out_d, Scatter{0, 0, 0, 0});
    return hipGetLastError();
}

hipError_t launch_expz_finish_scatter(const double* partial, int64_t rows, int n, int q, double* out,
                                      const Scatter& sc, hipStream_t st) {
    if (q < 0 || sc.per < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_expz_finish, dim3(blocks_for((u64)rows, 4)), dim3(256), 0, st, partial, (u64)rows,
                       n, chunk_blocks(n), q, (float*)nullptr, out, sc);
    return hipGetLastError();
}

hipError_t launch_zsum_finish(const double* partial, int64_t rows, int64_t per_row, double* out,
                              const Scatter& sc, hipStream_t st) {
    if (rows < 1 || per_row < 1 || sc.per < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_zsum_finish, dim3(blocks_for((u64)rows, 256)), dim3(256), 0, st, partial, (u64)rows,
                       (u64)per_row, out, sc);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const float2* src, int n, int64_t rows, const RowMap& rm, float2* states,
                              hipStream_t st) {
    if (n < 1) return hipErrorInvalidValue;   // rows of one amplitude cannot be copied in pairs
    const u64 total = (u64)rows << n;
    hipLaunchKernelGGL(k_gather_rows, dim3(blocks_for(total / 2, 256)), dim3(256), 0, st, src, n, total, rm,
                       states);
    return hipGetLastError();
}

hipError_t launch_marginal_block(const float2* state, int64_t rows, int n, uint64_t mask, int64_t n_v,
                                 double* partial, hipStream_t st) {
    const int m = __builtin_popcountll(mask);
    const u64 sub = 1ull << (n - m);
    const u64 nblk = (u64)chunk_blocks(n - m);
    const u64 blocks = (u64)rows * (u64)n_v * nblk;
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_marginal_block, dim3((unsigned)blocks), dim3(256), 0, st, state, n, (u64)mask,
                       (u64)n_v, nblk, sub, partial);
    return hipGetLastError();
}

hipError_t launch_marginal_finish(const double* partial, int64_t jobs, int64_t nblk, float* out,
                                  int renorm_mode, double* scale, hipStream_t st) {
    hipLaunchKernelGGL(k_marginal_finish, dim3(blocks_for((u64)jobs, 4)), dim3(256), 0, st, partial,
                       (u64)jobs, (u64)nblk, out, renorm_mode, scale);
    return hipGetLastError();
}

hipError_t launch_project(float2* state, int64_t rows, int n, uint64_t mask, const double* scale,
                          hipStream_t st) {
    const u64 total = (u64)rows << n;
    hipLaunchKernelGGL(k_project, dim3(blocks_for(total, 256)), dim3(256), 0, st, state, total, n,
                       (u64)mask, scale);
    return hipGetLastError();
}

hipError_t launch_fidelity_block(const float2* state, int64_t rows, int n, const float* x, int64_t dim,
                                 double* partial, int nblk, const RowMap& rm, hipStream_t st) {
    hipLaunchKernelGGL(k_fidelity_block, rows_grid(nblk, (u64)rows), dim3(256), 0, st, state, (u64)rows, n, x,
                       (u64)dim, nblk, rm, partial);
    return hipGetLastError();
}

hipError_t launch_fidelity_finish(const double* partial, int nblk, int64_t rows, float* out, double* out_d,
                                  hipStream_t st) {
    hipLaunchKernelGGL(k_fidelity_finish, dim3((unsigned)rows), dim3(256), 0, st, partial, nblk, out, out_d);
    return hipGetLastError();
}

hipError_t launch_reset_rows(const float2* state, int n, uint64_t mask, int64_t rows, const RowMap& rm,
                             float2* work, hipStream_t st) {
    const u64 total = (u64)rows << n;
    hipLaunchKernelGGL(k_reset_rows, dim3(blocks_for(total / 2, 256)), dim3(256), 0, st, state, n, (u64)mask,
                       total, rm, work);
    return hipGetLastError();
}

hipError_t launch_reset_sum(const double* Frow, int64_t per, int64_t B, float* out, hipStream_t st) {
    hipLaunchKernelGGL(k_reset_sum, dim3(blocks_for((u64)B, 256)), dim3(256), 0, st, Frow, (u64)per, (u64)B, out);
    return hipGetLastError();
}

hipError_t launch_shot_expz(const long long* samples, int64_t shots, int64_t rows, int n, float* out,
                            hipStream_t st) {
    hipLaunchKernelGGL(k_shot_expz, dim3(blocks_for((u64)rows * n, 4)), dim3(256), 0, st, samples, (u64)shots,
                       (u64)rows, n, out);
    return hipGetLastError();
}

hipError_t launch_pauli(const float2* state, int64_t rows, int n, uint64_t xmask, uint64_t ymask,
                        uint64_t zmask, double* partial, float* out, hipStream_t st) {
    const u64 f = (u64)(xmask | ymask);
    const int nblk = chunk_blocks(f ? n - 1 : n);    // with flips, half the indices are visited
    hipLaunchKernelGGL(k_pauli_block, rows_grid(nblk, (u64)rows), dim3(256), 0, st, state, (u64)rows, n,
                       f, (u64)(ymask | zmask), __builtin_popcountll(ymask), nblk, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_pauli_finish, dim3((unsigned)rows), dim3(256), 0, st, partial, nblk,
                       __builtin_popcountll(ymask), out);
    return hipGetLastError();
}

hipError_t launch_sample(const float2* state, int64_t rows, int n, const double* uniforms, int64_t shots,
                         unsigned long long* cum, long long* out, hipStream_t st) {
    const int nblk = chunk_blocks(n);
    hipLaunchKernelGGL(k_sample_blocksum, rows_grid(nblk, (u64)rows), dim3(256), 0, st, state, (u64)rows, n, nblk,
                       cum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_sample_scan, dim3((unsigned)rows), dim3(1024), 0, st, cum, nblk);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const u64 jobs = (u64)rows * (u64)shots;
    if (jobs == 0) return hipSuccess;
    hipLaunchKernelGGL(k_sample_draw, dim3(blocks_for(jobs, 4)), dim3(256), 0, st, state, n, nblk, cum,
                       uniforms, (u64)shots, jobs, out);
    return hipGetLastError();
}

hipError_t launch_adj_init(const float2* A, int n, int kind, int q, uint64_t mask, const double* coef,
                           int64_t rows, float2* S, int paired, hipStream_t st) {
    if (n < 1 || rows < 1 || kind < 0 || kind > 2 || (kind == 2 && !coef)) return hipErrorInvalidValue;
    const u64 total = (u64)rows << n;
    const AdjObs o{kind, q, (u64)mask, coef};
    hipLaunchKernelGGL(k_adj_init, dim3(blocks_for(total / 2, 256)), dim3(256), 0, st, A, n, o, total, S, paired);
    return hipGetLastError();
}

hipError_t launch_trash_loss(const float2* A, int n, uint64_t mask, int64_t rows, int64_t sample0, int64_t P,
                             double* partial, double* f, hipStream_t st) {
    if (rows < 1) return hipErrorInvalidValue;
    const int nblk = chunk_blocks(n);
    hipLaunchKernelGGL(k_p0_block, rows_grid(nblk, (u64)rows), dim3(256), 0, st, A, (u64)rows, n, (u64)mask, nblk, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_trash_loss, dim3(blocks_for((u64)rows, 256)), dim3(256), 0, st, partial, nblk,
                       (u64)rows, (u64)sample0, (u64)P, f);
    return hipGetLastError();
}

hipError_t launch_mse_coef(const double* z, const float* y, int n, int64_t rows, int64_t sample0, int64_t P,
                           double* coef, double* f, hipStream_t st) {
    hipLaunchKernelGGL(k_mse_coef, dim3(blocks_for((u64)rows, 256)), dim3(256), 0, st, z, y, n, (u64)rows,
                       (u64)sample0, (u64)P, coef, f);
    return hipGetLastError();
}

hipError_t launch_sgd(float* p, const float* g, int64_t count, double lr, hipStream_t st) {
    if (count < 1) return hipSuccess;
    hipLaunchKernelGGL(k_sgd, dim3(blocks_for((u64)count, 256)), dim3(256), 0, st, p, g, (u64)count, lr);
    return hipGetLastError();
}

hipError_t launch_adam(float* p, const float* g, float* m, float* v, int64_t count, int64_t t, double lr,
                       double b1, double b2, double eps, hipStream_t st) {
    if (count < 1) return hipSuccess;
    const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
    hipLaunchKernelGGL(k_adam, dim3(blocks_for((u64)count, 256)), dim3(256), 0, st, p, g, m, v, (u64)count,
                       lr, b1, b2, eps, c1, c2);
    return hipGetLastError();
}



// The fewest tiles of a row one workgroup of the tile kernels takes, and the resulting (largest
// number of) groups per row.
static inline int trans_tiles_per_group(int n) { const int tiles = 1 << (n - 12); return tiles < 4 ? tiles : 4; }
static inline int trans_groups(int n) { return (1 << (n - 12)) / trans_tiles_per_group(n); }

// upper bound of the partial entries per (row pair, qubit) of the transition sums
int adj_trans_blocks(int n) { return n < 12 ? 1 : 4 * trans_groups(n); }

hipError_t launch_adj_layer(const float2* psi0, const float2* lam0, int rstride, int n, int64_t row_pairs,
                            double* partial, const CircDev& c,
                            int layer, const float* params, const float* feats, int64_t sample0, int64_t P,
                            double* f, hipStream_t st) {
    if (row_pairs < 1 || row_pairs > 65535) return hipErrorInvalidValue;
    int nblk;
    if (n < 12) {
        nblk = adj_trans_blocks(n);
        hipLaunchKernelGGL(k_trans_block, dim3(nblk, n, (unsigned)row_pairs), dim3(256), 0, st, psi0, lam0, rstride,
                           n, (u64)1 << (n - 1), nblk, partial);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else {
        // qubits 0..11 from contiguous tiles, then 8 more per read from tiles whose window sits higher
        // (the last window ends at bit n and only its not yet covered qubits are taken)
        // A workgroup's first load and last sums overlap with nothing, so it takes as many tiles as
        // still leaves two workgroups per compute unit (never fewer than the buffer was sized for).
        const int tiles = 1 << (n - 12);
        int per_group = trans_tiles_per_group(n);
        while (per_group * 2 <= tiles && per_group < 32 && (int64_t)(tiles / (per_group * 2)) * row_pairs >= 512)
            per_group *= 2;
        const int groups = tiles / per_group;
        nblk = 4 * groups;                               // one partial per wavefront of a group
        const dim3 grid(groups, (unsigned)row_pairs);
        hipLaunchKernelGGL((k_trans_wave<3>), grid, dim3(256), 0, st, psi0, lam0, rstride, n, 12, 12, 0, per_group,
                           nblk, partial);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        for (int done = 12; done < n;) {
            int w = done, j0 = 4;
            if (w + 8 > n) { w = n - 8; j0 = 4 + (done - w); }
            switch (j0) {
#define QSV_TRANS_CASE(J) case J: hipLaunchKernelGGL((k_trans_tile<J>), grid, dim3(256), 0, st, psi0, lam0, rstride, n, 4, w, per_group, nblk, partial); break;
                case 4: case 5: case 6: case 7:
                    hipLaunchKernelGGL((k_trans_wave<2>), grid, dim3(256), 0, st, psi0, lam0, rstride, n, 4, w, j0, per_group,
                                       nblk, partial);
                    break;
                QSV_TRANS_CASE(8) QSV_TRANS_CASE(9) QSV_TRANS_CASE(10) QSV_TRANS_CASE(11)
#undef QSV_TRANS_CASE
                default: return hipErrorInvalidValue;
            }
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            done = w + 8;
        }
    }
    const u64 jobs = (u64)row_pairs * c.slots() * c.n;
    if (jobs == 0) return hipSuccess;
    const double* sums = partial;
    if (nblk > 1) {   // the summed matrices go behind the partials
        double* M = partial + (u64)row_pairs * n * nblk * 8;
        hipLaunchKernelGGL(k_trans_finish, dim3(blocks_for((u64)row_pairs * n, 4)), dim3(256), 0, st, partial,
                           nblk, (u64)row_pairs * n, M);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        sums = M;
        nblk = 1;
    }
    hipLaunchKernelGGL(k_adj_layer, dim3(blocks_for(jobs, 256)), dim3(256), 0, st, sums, nblk, c, layer,
                       params, feats, (u64)sample0, (u64)row_pairs, (u64)P, f);
    return hipGetLastError();
}

hipError_t launch_grad_finish(const double* f, int64_t B, int64_t P, const CircDev& c, const float* feats,
                              float* loss, float* grad, float* mean_loss, float* mean_grad,
                              hipStream_t st) {
    hipLaunchKernelGGL(k_grad_finish, dim3(blocks_for((u64)B * (P + 1), 256)), dim3(256), 0, st, f,
                       (u64)B, (u64)P, c, feats, loss, grad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (mean_loss || mean_grad) {
        hipLaunchKernelGGL(k_grad_mean, dim3((unsigned)(P + 1)), dim3(256), 0, st, f, (u64)B,
                           (u64)P, c, feats, mean_loss, mean_grad);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace qsv

// ============================================================================================
// Scratch memory for callers that cannot allocate (code under HIP graph capture, serving loops,
// harnesses that forbid hipMalloc): a fixed array in the code object, one copy per GPU that loads
// the library, held until the process ends.  Its name is a host-side stand-in, not a device
// address: host code asks the runtime for the address once per device and uses that pointer.
static __device__ __align__(256) unsigned char scratch[qsv::kStaticScratchBytes];

namespace qsv {

hipError_t static_scratch(int device, void** ptr) {
    constexpr int kMaxDevices = 64;
    static void* ptrs[kMaxDevices] = {};
    static std::mutex mu;
    if (device < 0 || device >= kMaxDevices || !ptr) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[device]) {
        // the caller has made `device` current: the address is that device's copy of the array
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptrs[device] = p;
    }
    *ptr = ptrs[device];
    return hipSuccess;
}

}  // namespace qsv
