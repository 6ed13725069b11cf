// Per-row solve: one 256-thread workgroup per decode position, everything after the streaming
// selection lives in LDS.
//
//   merge the slices' candidates -> top-k support V_0       (App. "Top-k Sampling ...")
//   order by decreasing q/p, prefix psi, H*, alpha*         (Sec. 5.1, Thm 3.1)
//   suffix minima -> outer targets p_i and block boundaries (Thm 6.2, Lemma 6.3)
//   truncation sets T                                       (Alg. 1, Sec. 6.3)
//   softmax weights of Theta_T / Phi_T by iterative scaling (Thm 6.5 / Thm 6.4)
//
// A second kernel (full_programs_kernel) runs the same programs for rows whose steps 1-2 were done in
// HBM because the support is the whole vocabulary.
//
// The gradient of Theta_T / Phi_T is (mass routed to token j) - target_j.  The routed mass is a sum
// over draft tuples; here it is evaluated in polynomial time from
//     1/x = int_0^inf e^{-xt} dt,
//     E[ prod_{i in set(tuple)} x_i ] = n! [z^n] e^{z ctx} prod_i (1 + x_i (e^{z q_i} - 1)),  x_i = e^{-t w_i},
// with truncated power series in z (degree n) and the trapezoid rule in log t: lanes are quadrature
// nodes, waves split the tokens, the series live in registers.
#include "gr_internal.h"

namespace gr {

namespace {

// Optional cycle accounting (builds with -DGR_PHASE_CLOCKS only): thread 0 adds the shader-clock cycles since
// its previous mark to one of 16 slots; the totals per row are written to RowInfo::clk.
#ifdef GR_PHASE_CLOCKS
#define GR_CLK(L, slot) do { if (threadIdx.x == 0) { const long long now_ = clock64(); (L).clk[slot] += now_ - (L).clk_last; (L).clk_last = now_; } } while (0)
#else
#define GR_CLK(L, slot) do {} while (0)
#endif

constexpr int KS = kMaxSupport;
constexpr int kST = 256;             // threads of the solve workgroup (one wave per SIMD: each may use all 512 registers)
constexpr int kSW = kST / 64;
constexpr double kQuadStep = 0.45;   // trapezoid step in log t (discretisation error ~1e-9 relative)
constexpr double kQuadLo = 1e-4;     // t_lo * (slack + sum w): the part below t_lo is added in closed form
constexpr double kQuadHi = 25.0;     // t_hi * (slowest decay rate)
constexpr double kStretch = 4.0;      // first cap on the per-coordinate stretch of the fixed-point step
constexpr int kStall = 3;            // iterations without a better point before the cap is halved
constexpr int kMixBudget = 60;       // the mixed fixed-point iteration gets kMixBudget + m evaluations before Newton takes over
constexpr int kCols = kHist - 1;                       // Anderson columns
constexpr int kGram = kCols * (kCols + 1) / 2 + kCols; // upper triangle of the Gram matrix + right-hand side

// Operands of the light-token arithmetic, packed so that one token (phase 1) or one quadrature node
// (phase 3) is three 16-byte LDS reads at constant offsets.
struct alignas(16) NodeRec { double t, qw, T[4]; };          // abscissa, weight, total series at degrees n-1 .. n-4
struct alignas(16) TokRec { double aw, e[4], pad; };         // weight, q^k / k! for k = 1..4

// D: the series degree of the kernel (>= n): the per-token and per-node series hold D + 1 terms, so the
// kernels of small D leave LDS for a streaming workgroup of the next batch beside a live row.
template <int D>
struct Lds {
    static constexpr int kS = D + 1;  // stride of a series
    // support, in ratio order
    int tok[KS]; int blk[KS]; int inT[KS]; int ordq[KS]; int apos[kMaxT];
    int flag[KS + 2]; int blo[KS + 2];
    double qn[KS]; double pn[KS]; double rho[KS]; double tgt[KS]; double wgt[KS];
    double Q[KS + 1]; double F[KS + 2];
    // one convex program
    double aq[kMaxT]; double at[kMaxT]; double aal[kMaxT]; double aw[kMaxT]; double aR[kMaxT]; double af[kMaxT];
    double apd[kMaxT];              // Pr[token drawn within the program] = atot^n - (atot - q)^n
    double etab[kMaxT * kS];        // q^a / a!, a = 0..D
    int adeg[kMaxT];                // degree at which the token's exponential series may be cut
    // Newton fallback (its Jacobian lives in a per-row HBM scratch)
    double nR[kMaxT]; double nstep[kMaxT]; double nsave[kMaxT]; int nused[kMaxT]; int ncolof[kMaxT];
    double Ha[kHist][kMaxT]; double Hf[kHist][kMaxT]; double aBest[kMaxT]; double fBest[kMaxT]; double rBest[kMaxT];
    double gram[kGram]; double gamma[kCols];
    // evaluator: node abscissae and weights, total series per node, per-wave partial routed mass
    double tnode[64]; double qwnode[64]; double Tl[64 * kS];
    double aS[kMaxT];               // routed mass weighted by the node abscissa t; aS_i = R_i - dR_i/d(log w_i)
    // scans and counters of the prologue (dead once the first program starts) share their bytes with the
    // evaluator's per-wave partial sums
    union {
        struct {
            int cnt0[KS + 2]; int cnt1[KS + 2];
            double qd[KS]; double accb[KS];
            double P[KS + 1]; double S[KS + 1]; double G0[KS + 2]; double G1[KS + 2];
        };
        struct {
            double rpart[kSW][kMaxT];
            double spart[kSW][kMaxT];   // the same sums weighted by t
            double cum[kSW * 4 * 64];   // per-wave cumulant sums of the light tokens, per node
        };
    };
    NodeRec nrec[64 + 16];          // nodes of the current chunk; the 16 beyond are zero (weight 0)
    TokRec trec[kMaxT + 16];        // active tokens; the 16 beyond the last have aw = 1e300 (x = 0)
    double e2tab[32];               // 2^(-j/32)
    int nbig;                       // number of heavy tokens of the current program
    double work;                    // sum over evaluator calls of nodes x active tokens (thread 0 only)
#ifdef GR_PHASE_CLOCKS
    long long clk[16]; long long clk_last;
#endif
    double red[kSW]; double R0acc; int ok; int pick[4]; int count; int hist[256];
    // unsorted candidates (select merge), later the per-wave partial products of the evaluator
    union {
        unsigned long long keys[kSelCap];
        double part[kSW * kS * 64];
    } u;
};


// e^{-y} for y >= 0: Cody-Waite reduction by ln 2 and a degree-12 Taylor polynomial on
// |r| <= ln(2)/2 (relative error below 1e-15; underflows to 0 beyond y = 708).
__device__ __forceinline__ double exp_neg(double y) {
    if (y > 708.0) return 0.0;
    const double k = rint(y * 1.4426950408889634);
    double r = fma(k, -6.93147180369123816490e-01, y);
    r = fma(k, -1.90821492927058770002e-10, r);
    r = -r;
    double p = 2.08767569878680989792e-09;              // 1/12!
    p = fma(p, r, 2.50521083854417187751e-08);           // 1/11!
    p = fma(p, r, 2.75573192239858906526e-07);           // 1/10!
    p = fma(p, r, 2.75573192239858906526e-06);           // 1/9!
    p = fma(p, r, 2.48015873015873015873e-05);           // 1/8!
    p = fma(p, r, 1.98412698412698412698e-04);           // 1/7!
    p = fma(p, r, 1.38888888888888888889e-03);           // 1/6!
    p = fma(p, r, 8.33333333333333333333e-03);           // 1/5!
    p = fma(p, r, 4.16666666666666666667e-02);           // 1/4!
    p = fma(p, r, 1.66666666666666666667e-01);           // 1/3!
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, -static_cast<int>(k));
}

// A(z) <- A(z) * (1 + x (e^{zq} - 1)), the exponential series cut at degree C <= D.
// e[a] = q^a / a!.
template <int D, int C>
__device__ __forceinline__ void mul_factor(double (&A)[D + 1], double x, const double* e) {
    double ee[C + 1];
#pragma unroll
    for (int a = 1; a <= C; ++a) ee[a] = e[a];
#pragma unroll
    for (int d = D; d >= 1; --d) {
        double acc = 0.0;
#pragma unroll
        for (int a = 1; a <= (d < C ? d : C); ++a) acc = fma(ee[a], A[d - a], acc);
        A[d] = fma(x, acc, A[d]);
    }
}

// A(z) <- A(z) * B(z), truncated at degree D.
template <int D>
__device__ __forceinline__ void mul_series(double (&A)[D + 1], const double (&B)[D + 1]) {
#pragma unroll
    for (int d = D; d >= 0; --d) {
        double acc = 0.0;
#pragma unroll
        for (int a = 0; a <= d; ++a) acc = fma(A[a], B[d - a], acc);
        A[d] = acc;
    }
}

// [z^n] of  (e^{zq} - 1) * T(z) / (1 + x (e^{zq} - 1)): the leave-one-out coefficient of a token,
// by series division (the quotient is only needed below degree n).
template <int D, int C>
__device__ __forceinline__ double loo_coeff(const double (&T)[D + 1], double x, const double* e, int n) {
    double ee[C + 1];
#pragma unroll
    for (int a = 1; a <= C; ++a) ee[a] = e[a];
    double Bq[D + 1];
    Bq[0] = T[0];
    double cn = 0.0;
#pragma unroll
    for (int d = 1; d <= D; ++d) {
        double conv = 0.0;
#pragma unroll
        for (int a = 1; a <= (d < C ? d : C); ++a) conv = fma(ee[a], Bq[d - a], conv);
        Bq[d] = fma(-x, conv, T[d]);
        if (d == n) cn = conv;
    }
    return cn;
}

// Four independent copies of the primitives, interleaved instruction by instruction so that the
// dependent fp64 chains of one copy fill the latency of the others.
//
// e^{-y} for y >= 0 with a 32-entry table: y = k ln2/32 + r, |r| <= ln2/64, e^{-y} =
// 2^-(k>>5) * tab[k&31] * e^{-r} with tab[j] = 2^(-j/32) and a degree-5 polynomial (error < 3e-15).
__device__ __forceinline__ void exp_neg4(const double (&y)[4], double (&out)[4], const double* tab) {
    double kf[4], r[4], p[4], tv[4];
    int ki[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kf[j] = rint(fmin(y[j], 1000.0) * 46.166241308446828);
#pragma unroll
    for (int j = 0; j < 4; ++j) { ki[j] = static_cast<int>(kf[j]); tv[j] = tab[ki[j] & 31]; }
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = fma(kf[j], -(6.93147180369123816490e-01 / 32.0), fmin(y[j], 1000.0));
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = -fma(kf[j], -(1.90821492927058770002e-10 / 32.0), r[j]);
    const double c[5] = {4.16666666666666666667e-02, 1.66666666666666666667e-01, 0.5, 1.0, 1.0};
#pragma unroll
    for (int j = 0; j < 4; ++j) p[j] = 8.33333333333333333333e-03;
#pragma unroll
    for (int i = 0; i < 5; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) p[j] = fma(p[j], r[j], c[i]);
#pragma unroll
    for (int j = 0; j < 4; ++j) out[j] = ldexp(p[j] * tv[j], -(ki[j] >> 5));      // 2^-1442 flushes to 0
}

template <int D, int C>
__device__ __forceinline__ void mul_factor4(double (&A)[4][D + 1], const double (&x)[4], const double (&e)[4][C + 1]) {
#pragma unroll
    for (int d = D; d >= 1; --d) {
        double acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = e[j][1] * A[j][d - 1];
#pragma unroll
        for (int a = 2; a <= (d < C ? d : C); ++a)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = fma(e[j][a], A[j][d - a], acc[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) A[j][d] = fma(x[j], acc[j], A[j][d]);
    }
}

// four quotients T_j / (1 + x_j (e^{zq} - 1)) of the same token (series e) at four nodes
template <int D, int C>
__device__ __forceinline__ void loo_coeff4(const double (&T)[4][D + 1], const double (&x)[4], const double (&e)[D + 1],
                                           int n, double (&cn)[4]) {
    double Bq[4][D + 1];
#pragma unroll
    for (int j = 0; j < 4; ++j) { Bq[j][0] = T[j][0]; cn[j] = 0.0; }
#pragma unroll
    for (int d = 1; d <= D; ++d) {
        double conv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) conv[j] = e[1] * Bq[j][d - 1];
#pragma unroll
        for (int a = 2; a <= (d < C ? d : C); ++a)
#pragma unroll
            for (int j = 0; j < 4; ++j) conv[j] = fma(e[a], Bq[j][d - a], conv[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) { Bq[j][d] = fma(-x[j], conv[j], T[j][d]); if (d == n) cn[j] = conv[j]; }
    }
}

// Phase 1, tokens that keep their full factor: tokens i0, i0+4, i0+8, i0+12 (below `bound`) into the
// four running products.
template <int D>
__device__ __forceinline__ void phase1_big(double (&A)[4][D + 1], const Lds<D>& L, int i0, int bound, double t) {
    double y[4], x[4], e[4][D + 1];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * kSW;
        const int ii = i < bound ? i : i0;
        y[j] = i < bound ? t * L.aw[ii] : 1000.0;             // a missing token gets x = 0: its factor is 1
#pragma unroll
        for (int a = 1; a <= D; ++a) e[j][a] = L.etab[ii * (D + 1) + a];
    }
    exp_neg4(y, x, L.e2tab);
    mul_factor4<D, D>(A, x, e);
}

// Phase 1, light tokens: log(1 + x (e^u - 1)) = sum_k kappa_k(x) u^k / k!  with the cumulants of a
// Bernoulli(x) variable, so the product of their factors is the exponential of four sums.
// Tokens first, first + kSW, ... below m, four at a time (records beyond m contribute nothing); two
// register sets alternate so that the LDS operands of the next four are requested before the
// arithmetic of the current four.
template <class LdsT>
__device__ __forceinline__ void phase1_small_load(const LdsT& L, int i0, TokRec (&r)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = L.trec[i0 + j * kSW];
}
__device__ __forceinline__ void phase1_small_quad(double (&K)[4][4], const TokRec (&r)[4], double t, const double* tab) {
    double y[4], x[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) y[j] = t * r[j].aw;
    exp_neg4(y, x, tab);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double v = x[j] * (1.0 - x[j]);                  // kappa_2
        const double k3 = v * fma(-2.0, x[j], 1.0);            // kappa_3 = v (1 - 2x)
        const double k4 = v * fma(-6.0, v, 1.0);               // kappa_4 = v (1 - 6 v)
        K[j][0] = fma(x[j], r[j].e[0], K[j][0]);
        K[j][1] = fma(v, r[j].e[1], K[j][1]);
        K[j][2] = fma(k3, r[j].e[2], K[j][2]);
        K[j][3] = fma(k4, r[j].e[3], K[j][3]);
    }
}
template <class LdsT>
__device__ __forceinline__ void phase1_small(double (&K)[4][4], const LdsT& L, int first, int m, double t) {
    if (first >= m) return;
    TokRec a[4], b[4];
    phase1_small_load(L, first, a);
    for (int i0 = first; i0 < m; i0 += 8 * kSW) {
        const bool more = i0 + 4 * kSW < m;
        if (more) phase1_small_load(L, i0 + 4 * kSW, b);
        phase1_small_quad(K, a, t, L.e2tab);
        if (!more) break;
        if (i0 + 8 * kSW < m) phase1_small_load(L, i0 + 8 * kSW, a);
        phase1_small_quad(K, b, t, L.e2tab);
    }
}

// Phase 3, a token with its full factor at the four nodes nu0 + j*stride (j = 0..3).
template <int D>
__device__ __forceinline__ double phase3_big(const Lds<D>& L, const double (&e)[D + 1], double wt, int n, int nu0,
                                             int stride, int nn, double& acc_t) {
    double T[4][D + 1], y[4], x[4], qq[4], cn[4], tt[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int nu = nu0 + j * stride;
        const int nv = nu < nn ? nu : 0;
        tt[j] = L.tnode[nv];
        y[j] = tt[j] * wt;
        qq[j] = nu < nn ? L.qwnode[nv] : 0.0;
#pragma unroll
        for (int d = 0; d <= D; ++d) T[j][d] = L.Tl[nv * (D + 1) + d];
    }
    exp_neg4(y, x, L.e2tab);
    loo_coeff4<D, D>(T, x, e, n, cn);
    double acc = 0.0, at = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double term = qq[j] * x[j] * cn[j];
        acc += term;
        at = fma(term, tt[j], at);
    }
    acc_t = at;
    return acc;
}

// Phase 3, a light token: (e^u - 1) / (1 + x (e^u - 1)) = u + (1/2 - x) u^2 + (1/6 - x + x^2) u^3 +
// (1/24 - 7x/12 + 3x^2/2 - x^3) u^4 + ..., so the leave-one-out coefficient is a four-term sum over
// T[n-1..n-4].  e[k] = q^k / k! (zero for k > n), so the brackets are multiplied by k!.
// This wave's nodes wv, wv + kSW, ..., four at a time from the node records (uniform over the wave;
// records at or beyond nn carry weight 0); two register sets alternate as in phase 1.
template <class LdsT>
__device__ __forceinline__ void phase3_small_load(const LdsT& L, int nu0, NodeRec (&r)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = L.nrec[nu0 + j * kSW];
}
__device__ __forceinline__ void phase3_small_quad(const NodeRec (&c)[4], const double (&e)[5], double wt, const double* tab,
                                                  double& acc, double& at) {
    double y[4], x[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) y[j] = c[j].t * wt;
    exp_neg4(y, x, tab);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double xx = x[j];
        const double g2 = fma(-2.0, xx, 1.0);
        const double g3 = fma(6.0 * xx, xx - 1.0, 1.0);
        const double g4 = fma(xx, fma(xx, fma(-24.0, xx, 36.0), -14.0), 1.0);
        double cn = e[1] * c[j].T[0];
        cn = fma(e[2] * g2, c[j].T[1], cn);
        cn = fma(e[3] * g3, c[j].T[2], cn);
        cn = fma(e[4] * g4, c[j].T[3], cn);
        const double term = c[j].qw * xx * cn;
        acc += term;
        at = fma(term, c[j].t, at);
    }
}
template <class LdsT>
__device__ __forceinline__ double phase3_small(const LdsT& L, const double (&e)[5], double wt, int wv, int nn, double& acc_t) {
    double acc = 0.0, at = 0.0;
    acc_t = 0.0;
    if (wv >= nn) return acc;
    NodeRec a[4], b[4];
    phase3_small_load(L, wv, a);
    for (int nu0 = wv; nu0 < nn; nu0 += 8 * kSW) {
        const bool more = nu0 + 4 * kSW < nn;
        if (more) phase3_small_load(L, nu0 + 4 * kSW, b);
        phase3_small_quad(a, e, wt, L.e2tab, acc, at);
        if (!more) break;
        if (nu0 + 8 * kSW < nn) phase3_small_load(L, nu0 + 8 * kSW, a);
        phase3_small_quad(b, e, wt, L.e2tab, acc, at);
    }
    acc_t = at;
    return acc;
}

// Routed mass of every active token, and the mass left to the slack term.
//
// Tokens are held in decreasing q.  The first L.nbig of them ("heavy") keep their full factor
// 1 + x (e^{zq} - 1); the others ("light": q so small that terms beyond u^4 cannot change the z^n
// coefficient, or n <= 4 where four terms are exact) enter through four cumulant sums.
// Per chunk of 64 quadrature nodes:
//   phase 1  lanes = nodes; wave w takes tokens w, w+4, ...: heavy ones into four interleaved running
//            products, light ones into the cumulant sums;
//   phase 2  wave 0 forms T(node) = exp(z ctx + cumulant series) * product of the heavy products -> LDS;
//   phase 3  lanes = tokens, wave w walks nodes w, w+4, ...: each lane takes the leave-one-out
//            coefficient of its token (series division for heavy tokens, the four-term expansion for
//            light ones) and accumulates; no cross-lane reduction for the light tokens, two shuffles
//            for the heavy ones (16 tokens x 4 node groups per wave).
// In: L.aq, L.aal, L.etab / L.nbig / L.apd (set up by solve_program), m, n, ctx, slack, qsum = sum aq.
// Out: L.aR[0..m), L.R0acc (slack mass; meaningful when slack = 1).  All threads call it.
template <int D>
__device__ __forceinline__ void routed_eval(Lds<D>& L, int m, int n, double ctx, int slack, double qsum) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nbig = L.nbig;
    GR_CLK(L, 12);
    double w = 0.0;
    if (tid < m) { w = exp(L.aal[tid]); L.aw[tid] = w; L.trec[tid].aw = w; }
    if (tid < 16) { NodeRec z; z.t = 0.0; z.qw = 0.0; z.T[0] = z.T[1] = z.T[2] = z.T[3] = 0.0; L.nrec[64 + tid] = z; }
    const double wsum = block_sum<kSW>(tid < m ? w : 0.0, L.red);
    const double wmin = block_min<kSW>(tid < m ? w : 1e300, L.red);
    const double t_lo = kQuadLo / (slack + wsum);
    const double t_hi = kQuadHi / (slack + ((slack == 0 || ctx == 0.0) ? wmin : 0.0));
    const double range = log(t_hi / t_lo);
    double step = kQuadStep;
    int N = static_cast<int>(ceil(range / step)) + 1;
    if (N > 64 && range <= 0.5 * 63.0) { step = range / 63.0; N = 64; }
    if (N < 1) N = 1;
    if (N > 4096) N = 4096;
    const double atot = ctx + qsum;
    const double estep = exp(step);
    const double tail = step * t_lo / (estep - 1.0);       // trapezoid sum of the nodes below t_lo, x = 1 there
    const double tail2 = step * t_lo * t_lo / (estep * estep - 1.0);   // the same for the integrand times t
    double fact = 1.0;
    for (int i = 2; i <= n; ++i) fact *= i;
    double r0 = 0.0;                                       // slack mass, accumulated by lane 0 of wave 0
    double racc[2] = {0.0, 0.0};                           // phase 3 accumulators of light tokens lane, lane + 64
    double sacc[2] = {0.0, 0.0};                           // the same, weighted by the node abscissa t
    if (tid < m) { for (int w2 = 0; w2 < kSW; ++w2) { L.rpart[w2][tid] = 0.0; L.spart[w2][tid] = 0.0; } }
    const int first_small = nbig + ((wv - nbig) % kSW + kSW) % kSW;   // first light token of this wave
    // this lane's light tokens in phase 3: series terms q^k / k!, k <= min(n, 4)
    double es[2][5]; double ws[2];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tok = pass * 64 + lane;
        const int tk = tok < m ? tok : 0;
        ws[pass] = m > 0 ? L.aw[tk] : 0.0;
#pragma unroll
        for (int a = 1; a <= 4; ++a) es[pass][a] = (a <= n && a <= D && m > 0) ? L.etab[tk * (D + 1) + (a <= D ? a : 0)] : 0.0;
        es[pass][0] = 0.0;
    }
    __syncthreads();
    GR_CLK(L, 6);

    for (int c0 = 0; c0 < N; c0 += 64) {
        const int node = c0 + lane;
        const double t = t_lo * exp(step * node);
        const double qw = node < N ? step * t * exp_neg(slack * t) : 0.0;
        if (wv == 0) { L.tnode[lane] = t; L.qwnode[lane] = qw; }
        // ---- phase 1
        if (nbig > 0) {
            double A[4][D + 1];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int d = 0; d <= D; ++d) A[j][d] = d == 0;
            for (int i0 = wv; i0 < nbig; i0 += 4 * kSW) phase1_big<D>(A, L, i0, nbig, t);
            mul_series<D>(A[0], A[1]); mul_series<D>(A[2], A[3]); mul_series<D>(A[0], A[2]);
#pragma unroll
            for (int d = 0; d <= D; ++d) L.u.part[(wv * (D + 1) + d) * 64 + lane] = A[0][d];
        }
        {
            double K[4][4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k) K[j][k] = 0.0;
            phase1_small(K, L, first_small, m, t);
#pragma unroll
            for (int k = 0; k < 4; ++k) L.cum[(wv * 4 + k) * 64 + lane] = (K[0][k] + K[1][k]) + (K[2][k] + K[3][k]);
        }
        __syncthreads();
        GR_CLK(L, 7);
        // ---- phase 2 (wave 0)
        if (wv == 0) {
            double Kt[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                Kt[k] = 0.0;
                for (int w2 = 0; w2 < kSW; ++w2) Kt[k] += L.cum[(w2 * 4 + k) * 64 + lane];
            }
            Kt[0] += ctx;                                  // e^{z ctx}
            // T = exp(Kt_1 z + ... + Kt_4 z^4):  d T_d = sum_k k Kt_k T_{d-k}
            double T[D + 1];
            T[0] = 1.0;
#pragma unroll
            for (int d = 1; d <= D; ++d) {
                double acc = Kt[0] * T[d - 1];
#pragma unroll
                for (int k = 2; k <= (d < 4 ? d : 4); ++k) acc = fma(static_cast<double>(k) * Kt[k - 1], T[d - k], acc);
                T[d] = acc * (1.0 / d);
            }
            if (nbig > 0) {
                for (int w2 = 0; w2 < kSW; ++w2) {
                    double Bc[D + 1];
#pragma unroll
                    for (int d = 0; d <= D; ++d) Bc[d] = L.u.part[(w2 * (D + 1) + d) * 64 + lane];
                    mul_series<D>(T, Bc);
                }
            }
            double tn = 0.0;
            NodeRec rec; rec.t = t; rec.qw = qw; rec.T[0] = rec.T[1] = rec.T[2] = rec.T[3] = 0.0;
#pragma unroll
            for (int d = 0; d <= D; ++d) {
                L.Tl[lane * (D + 1) + d] = T[d];
                if (d == n) tn = T[d];
                if (d == n - 1) rec.T[0] = T[d];
                if (d == n - 2) rec.T[1] = T[d];
                if (d == n - 3) rec.T[2] = T[d];
                if (d == n - 4) rec.T[3] = T[d];
            }
            L.nrec[lane] = rec;
            r0 += wave_sum(qw * tn);
        }
        __syncthreads();
        GR_CLK(L, 8);
        // ---- phase 3
        const int nn = min(64, N - c0);
        // heavy tokens: 16 per round, lane = (token, node group); this wave's nodes are wv, wv+4, ...,
        // node group g takes every fourth of them
        for (int b0 = 0; b0 < nbig; b0 += 16) {
            const int tok = b0 + (lane & 15);
            const int tk = tok < nbig ? tok : 0;
            double e[D + 1];
#pragma unroll
            for (int a = 0; a <= D; ++a) e[a] = L.etab[tk * (D + 1) + a];
            double acct;
            double acc = phase3_big<D>(L, e, L.aw[tk], n, wv + kSW * (lane >> 4), 4 * kSW, nn, acct);
            acc += __shfl_xor(acc, 16); acct += __shfl_xor(acct, 16);
            acc += __shfl_xor(acc, 32); acct += __shfl_xor(acct, 32);
            if (lane < 16 && tok < nbig) { L.rpart[wv][tok] += acc; L.spart[wv][tok] += acct; }
        }
        // light tokens
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            if (pass * 64 < m && (pass + 1) * 64 > nbig) {
                double at;
                racc[pass] += phase3_small(L, es[pass], ws[pass], wv, nn, at);
                sacc[pass] += at;
            }
        }
        __syncthreads();                                   // part / cum / Tl / tnode are rewritten by the next chunk
        GR_CLK(L, 9);
    }
    if (lane < m && lane >= nbig) { L.rpart[wv][lane] = racc[0]; L.spart[wv][lane] = sacc[0]; }
    if (64 + lane < m && 64 + lane >= nbig) { L.rpart[wv][64 + lane] = racc[1]; L.spart[wv][64 + lane] = sacc[1]; }
    if (tid == 0) { L.R0acc = (r0 + ipow(atot, n) * tail / fact) * fact * slack; L.work += static_cast<double>(N) * m; }
    __syncthreads();
    if (tid < m) {
        double r = L.apd[tid] * tail / fact;
        // the nodes below t_lo (x = 1 there) add tail to the integral of 1 and tail2 to that of t
        double sq = L.apd[tid] * tail2 / fact;
        for (int w2 = 0; w2 < kSW; ++w2) { r += L.rpart[w2][tid]; sq += L.spart[w2][tid]; }
        L.aR[tid] = r * L.aw[tid] * fact;
        L.aS[tid] = sq * L.aw[tid] * L.aw[tid] * fact;
    }
    __syncthreads();
    GR_CLK(L, 10);
#ifdef GR_PHASE_CLOCKS
    if (tid == 0) L.clk[15] += 1;
#endif
}

// One evaluation and the stopping measure: max_i | log(target_i / routed_i) - common term |, where the
// common term is log(slack_target / slack mass) with slack, log(sum target / sum routed) without
// (the latter is zero in exact arithmetic and removes the common quadrature error).  f -> L.af;
// L.aR and L.aS stay valid until the next evaluation.
template <int D>
__device__ double defect_eval(Lds<D>& L, int m, int n, double ctx, int slack, double slack_target, double qsum,
                              double tsum, double* rsum_out) {
    const int tid = threadIdx.x;
    routed_eval<D>(L, m, n, ctx, slack, qsum);
    // the sum of the routed masses is needed without slack (common term) and by the Newton iteration
    const double rsum = (!slack || rsum_out) ? block_sum<kSW>(tid < m ? L.aR[tid] : 0.0, L.red) : 0.0;
    double f = 0.0;
    if (tid < m) {
        const double common = slack ? L.R0acc / slack_target : rsum / tsum;
        f = log(L.at[tid] / L.aR[tid] * common);
        L.af[tid] = f;
    }
    if (rsum_out) *rsum_out = rsum;
    const double worst = block_max<kSW>(tid < m ? fabs(f) : 0.0, L.red);
    GR_CLK(L, 11);
    return worst;
}

// Damped Newton iteration on routed(alpha) = target with a finite-difference Jacobian (the Hessian of
// Theta_T / Phi_T in alpha), for programs on which the fixed-point iteration is slow (a target that
// nearly exhausts the tuples containing its token).  One step costs one evaluation per variable, so
// it only takes over when the mixed iteration has used up its budget.  Without slack the last weight
// is pinned (the system is singular along the common shift).  Starts from L.aal.
// J: this row's scratch in HBM, kMaxT rows of kMaxT + 1 doubles (the last column is the right-hand side).
template <int D>
__device__ int newton_program(Lds<D>& L, double* J, int m, int n, double ctx, int slack, double slack_target, double qsum,
                              double tsum, double rel_tol, int max_evals, int* evals) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int nfree = slack ? m : m - 1;
    constexpr int LD = kMaxT + 1;
    constexpr double kFd = 1e-6;
    double rsum;
    double err = defect_eval<D>(L, m, n, ctx, slack, slack_target, qsum, tsum, &rsum);
    *evals += 1;
    while (err > rel_tol && *evals < max_evals && err < 1e300) {
        if (tid < m) L.nR[tid] = L.aR[tid];
        // common ratio routed/target over all vertices, the slack vertex included: Newton aims at
        // routed_j = ratio * target_j, which is what the stopping measure asks for
        const double ratio = slack ? (rsum + L.R0acc) / (tsum + slack_target) : rsum / tsum;
        __syncthreads();
        for (int k = 0; k < nfree; ++k) {
            if (tid == k) L.aal[k] += kFd;
            __syncthreads();
            routed_eval<D>(L, m, n, ctx, slack, qsum);
            if (tid < nfree) J[tid * LD + k] = (L.aR[tid] - L.nR[tid]) / kFd;
            if (tid == k) L.aal[k] -= kFd;
            __syncthreads();
        }
        *evals += nfree;
        if (tid < nfree) { J[tid * LD + kMaxT] = L.at[tid] * ratio - L.nR[tid]; L.nused[tid] = 0; L.ncolof[tid] = -1; L.nstep[tid] = 0.0; }
        __syncthreads();
        // Gauss-Jordan with partial pivoting: thread r owns row r
        for (int c = 0; c < nfree; ++c) {
            const double mag = (tid < nfree && !L.nused[tid]) ? fabs(J[tid * LD + c]) : -1.0;
            const double best = block_max<kSW>(mag, L.red);
            if (!(best > 0.0)) continue;                   // no pivot left in this column: its step stays 0
            const int who = static_cast<int>(block_min<kSW>(mag == best ? static_cast<double>(tid) : 1e9, L.red));
            const double piv = J[who * LD + c];
            if (tid < nfree && tid != who) {
                const double fct = J[tid * LD + c] / piv;
                for (int j = c; j < nfree; ++j) J[tid * LD + j] -= fct * J[who * LD + j];
                J[tid * LD + kMaxT] -= fct * J[who * LD + kMaxT];
            }
            if (tid == who) { L.nused[tid] = 1; L.ncolof[tid] = c; }
            __syncthreads();
        }
        if (tid < nfree && L.ncolof[tid] >= 0) {
            const int my_col = L.ncolof[tid];
            const double dg = J[tid * LD + my_col];
            L.nstep[my_col] = dg != 0.0 ? J[tid * LD + kMaxT] / dg : 0.0;
        }
        __syncthreads();
        const double smax = block_max<kSW>(tid < nfree ? fabs(L.nstep[tid]) : 0.0, L.red);
        if (!(smax < 1e300)) break;
        const double clip = smax > 2.0 ? 2.0 / smax : 1.0;
        // slope of the objective along the step: grad . d with grad_j = routed_j - ratio * target_j
        double slope0 = block_sum<kSW>(tid < nfree ? (L.nR[tid] - L.at[tid] * ratio) * clip * L.nstep[tid] : 0.0, L.red);
        if (!(slope0 < 0.0)) {
            // not a descent direction (noise in the difference quotients): take the plain
            // fixed-point step instead, which always is one
            if (tid < nfree) L.nstep[tid] = L.af[tid] / clip;
            __syncthreads();
            slope0 = block_sum<kSW>(tid < nfree ? (L.nR[tid] - L.at[tid] * ratio) * L.af[tid] : 0.0, L.red);
        }
        if (tid < m) L.nsave[tid] = L.aal[tid];
        __syncthreads();
        // Backtracking on the slope: the objective is convex, so it decreases along the step as long
        // as the slope stays negative; accept the first lam whose slope is below half of |slope0|.
        double lam = 1.0, err2 = err;
        bool ok = false;
        for (int ls = 0; ls < 20 && !ok; ++ls) {
            if (tid < nfree) L.aal[tid] = L.nsave[tid] + lam * clip * L.nstep[tid];
            __syncthreads();
            err2 = defect_eval<D>(L, m, n, ctx, slack, slack_target, qsum, tsum, &rsum);
            *evals += 1;
            const double ratio2 = slack ? (rsum + L.R0acc) / (tsum + slack_target) : rsum / tsum;
            const double slope = block_sum<kSW>(tid < nfree ? (L.aR[tid] - L.at[tid] * ratio2) * clip * L.nstep[tid] : 0.0, L.red);
            ok = (err2 < 1e300) && (slope <= 0.5 * fabs(slope0) || err2 < err);
            if (!ok) lam *= 0.5;
        }
        if (!ok) {                                 // no acceptable point along the direction: stop here
            if (tid < m) L.aal[tid] = L.nsave[tid];
            __syncthreads();
            break;
        }
        err = err2;
    }
    __syncthreads();
    return err <= rel_tol ? 0 : 1;
}

// Solve one program by iterative scaling with Anderson mixing.  Returns 0 when converged.
// In: L.aq, L.at (targets, already scaled to the tuple mass), L.aal (start log weights).
// Out: L.aal.  `evals` counts evaluator calls.
template <int D>
__device__ __forceinline__ int solve_program(Lds<D>& L, double* newton_ws, int m, int n, double ctx, int slack, double slack_target,
                             double rel_tol, int max_iter, int* evals) {
    const int tid = threadIdx.x;
    if (n == 1) {
        // One draft: a tuple is a single token, so the routed mass of token i is q_i w_i / (1 + w_i)
        // with the slack term (the single-draft rule, w_i = t_i / (q_i - t_i) in closed form) and q_i
        // whatever the weights without it.
        // A scaled target at or above its token's draw probability has no finite weight: the program
        // is reported as not converged, like an iteration that ran into its cap.
        int stuck = 0;
        if (slack && tid < m) {
            const double d = L.aq[tid] - L.at[tid];
            stuck = !(d > 0.0);
            L.aal[tid] = stuck ? 690.0 : log(L.at[tid] / d);
        }
        return block_sum_i<kSW>(stuck, L.red) ? 1 : 0;
    }
    const double qsum = block_sum<kSW>(tid < m ? L.aq[tid] : 0.0, L.red);
    const double tsum = block_sum<kSW>(tid < m ? L.at[tid] : 0.0, L.red);
    if (tid < m) {
        // per-token series of e^{zq}, and the degree beyond which its terms change the z^n
        // coefficient by less than 1e-11 relative: C(n-1, c) (q/atot)^c / (c+1) < 1e-11
        const double q = L.aq[tid], atot = ctx + qsum;
        double e = 1.0;
        L.etab[tid * (D + 1)] = 1.0;
        for (int a = 1; a <= (D > 4 ? D : 4); ++a) {
            e = e * q / a;
            if (a <= D) L.etab[tid * (D + 1) + a] = e;
            if (a <= 4) L.trec[tid].e[a - 1] = e;
        }
        // light if the u^5 and later terms of its factor cannot change the z^n coefficient by more
        // than 1e-11 relative: C(n-1, 4) (q/atot)^4 / 5 < 1e-11; exact for n <= 4
        const double r = q / atot;
        double binom = 1.0;
        for (int c = 1; c <= 4; ++c) binom = binom * (n - c) / c;         // C(n-1, 4)
        L.adeg[tid] = (n <= 4 || binom * r * r * r * r / 5.0 < 1e-11) ? 0 : D;
        L.apd[tid] = pow_diff(atot, q, n);
    }
    if (tid < 32) L.e2tab[tid] = exp2(-static_cast<double>(tid) / 32.0);
    if (tid < 16) { TokRec z; z.aw = 1e300; z.e[0] = z.e[1] = z.e[2] = z.e[3] = 0.0; z.pad = 0.0; L.trec[m + tid] = z; }
    const int nheavy = block_sum_i<kSW>((tid < m && L.adeg[tid] != 0) ? 1 : 0, L.red);
    if (tid == 0) L.nbig = nheavy;
    __syncthreads();
    GR_CLK(L, 5);
    int hcount = 0, plain = 0, since = 0;
    double best_err = 1e300, cap = kStretch;
    int result = 1;
    const int mix_iters = (max_iter > kMixBudget + m) ? kMixBudget + m : max_iter;
    for (int it = 1; it <= mix_iters; ++it) {
        if (!slack) {
            const double amax = block_max<kSW>(tid < m ? L.aal[tid] : -1e300, L.red);
            if (tid < m) L.aal[tid] -= amax;
            __syncthreads();
        }
        const double err = defect_eval<D>(L, m, n, ctx, slack, slack_target, qsum, tsum, nullptr);
        *evals += 1;
        // The fixed-point step log(target / routed) treats the routed mass as proportional to the
        // weight; its true logarithmic derivative is (R - S) / R with S = w^2 int t ... (the share a
        // token loses to itself), so the step of each coordinate is stretched by R / (R - S), at most
        // `cap`.  The stretched iteration is no longer monotone: when kStall iterations bring no
        // better point it returns to the best one with half the cap; at cap 1 (the plain step, whose
        // stopping measure need not fall at every step) it is left alone.
        double f = 0.0, ratio = 1.0;
        if (tid < m) {
            f = L.af[tid];
            const double R = L.aR[tid], d = R - L.aS[tid];
            ratio = (d > 0.0) ? fmin(R / d, 1e30) : 1e30;
        }
        if (err <= rel_tol) { result = 0; break; }
        if (!(err < 1e300) || err > 100.0 * best_err) {
            // a mixed step went astray: back to the best point, unmixed steps for a while
            if (!(best_err < 1e300)) break;        // no finite point seen: give up on this program
            if (tid < m) { L.aal[tid] = L.aBest[tid]; f = L.fBest[tid]; ratio = L.rBest[tid]; }
            hcount = 0; plain = 20; since = 0;
        } else if (err < best_err) {
            best_err = err; since = 0;
            if (tid < m) { L.aBest[tid] = L.aal[tid]; L.fBest[tid] = f; L.rBest[tid] = ratio; }
        } else if (cap > 1.0 && ++since >= kStall) {
            if (tid < m) { L.aal[tid] = L.aBest[tid]; f = L.fBest[tid]; ratio = L.rBest[tid]; }
            hcount = 0; since = 0;
            cap = fmax(1.0, 0.5 * cap);
        }
        f *= fmin(ratio, cap);
        const int cur = it % kHist;
        if (tid < m) { L.Ha[cur][tid] = L.aal[tid]; L.Hf[cur][tid] = f; }
        const int ncol = plain > 0 ? 0 : min(hcount, kHist - 1);
        if (plain > 0) --plain;
        double stepv = f;
        if (ncol >= 1) {
            // normal equations of  min || f - dF gamma ||  with dF_c = f - f_c
            double dF[kHist - 1], dA[kHist - 1];
#pragma unroll
            for (int c = 0; c < kHist - 1; ++c) {
                const int slot = (cur - 1 - c + 2 * kHist) % kHist;
                const bool on = c < ncol && tid < m;
                dF[c] = on ? f - L.Hf[slot][tid] : 0.0;
                dA[c] = on ? L.aal[tid] - L.Ha[slot][tid] : 0.0;
            }
            // Gram matrix and right-hand side
            __syncthreads();                               // Hf[cur] is complete
            {
                // entry e of (upper triangle of the Gram matrix, then dF_a . f) goes to wave e mod 4;
                // lanes cover the tokens.  The loop is unrolled, so the columns of an entry are constants.
                const int wv = tid >> 6, lane = tid & 63;
#pragma unroll
                for (int e = 0; e < kGram; ++e) {
                    constexpr int kTri = kCols * (kCols + 1) / 2;
                    int ca = 0, cb = 0, idx = 0;
#pragma unroll
                    for (int a2 = 0; a2 < kCols; ++a2)
#pragma unroll
                        for (int b2 = a2; b2 < kCols; ++b2) { if (idx == e) { ca = a2; cb = b2; } ++idx; }
                    const bool rhs = e >= kTri;
                    if (rhs) { ca = e - kTri; cb = 0; }
                    if ((e % kSW) != wv) continue;
                    double acc = 0.0;
                    if (ca < ncol && (rhs || cb < ncol)) {
                        const int sa = (cur - 1 - ca + 2 * kHist) % kHist, sb = (cur - 1 - cb + 2 * kHist) % kHist;
                        for (int i = lane; i < m; i += 64) {
                            const double fi = L.Hf[cur][i];
                            const double da = fi - L.Hf[sa][i];
                            acc = fma(da, rhs ? fi : fi - L.Hf[sb][i], acc);
                        }
                        acc = wave_sum(acc);
                    }
                    if (lane == 0) L.gram[e] = acc;
                }
            }
            __syncthreads();
            if (tid == 0) {
                // normal equations by Gaussian elimination without pivoting (the matrix is symmetric
                // positive definite after the ridge); fully unrolled so that it stays in registers
                double Gm[kCols][kCols + 1];
                {
                    int idx = 0;
#pragma unroll
                    for (int a = 0; a < kCols; ++a)
#pragma unroll
                        for (int b = a; b < kCols; ++b) {
                            const double g = L.gram[idx];
                            Gm[a][b] = g; Gm[b][a] = g; ++idx;
                        }
#pragma unroll
                    for (int a = 0; a < kCols; ++a) {
                        Gm[a][kCols] = L.gram[idx]; ++idx;
                    }
                }
                bool good = true;
                double pivinv[kCols];
#pragma unroll
                for (int c = 0; c < kCols; ++c) pivinv[c] = 0.0;
#pragma unroll
                for (int c = 0; c < kCols; ++c) {
                    if (c < ncol) {
                        // a ridge relative to the column itself: recent columns are far shorter than old ones
                        Gm[c][c] = Gm[c][c] * (1.0 + 1e-10) + 1e-300;
                        good = good && (Gm[c][c] > 0.0);
                        const double inv = 1.0 / Gm[c][c];
                        pivinv[c] = inv;
#pragma unroll
                        for (int r = c + 1; r < kCols; ++r) {
                            if (r < ncol) {
                                const double fct = Gm[r][c] * inv;
#pragma unroll
                                for (int j = c + 1; j <= kCols; ++j) Gm[r][j] = fma(-fct, Gm[c][j], Gm[r][j]);
                            }
                        }
                    }
                }
                double gam[kCols];
#pragma unroll
                for (int c = kCols - 1; c >= 0; --c) {
                    double sacc = Gm[c][kCols];
#pragma unroll
                    for (int j = c + 1; j < kCols; ++j) if (j < ncol) sacc = fma(-Gm[c][j], gam[j], sacc);
                    gam[c] = (c < ncol) ? sacc * pivinv[c] : 0.0;
                }
                double gnorm = 0.0;
#pragma unroll
                for (int c = 0; c < kCols; ++c) { L.gamma[c] = gam[c]; gnorm += fabs(gam[c]); }
                L.ok = (good && gnorm < 1e300) ? 1 : 0;
            }
            __syncthreads();
            double cand = f;
#pragma unroll
            for (int c = 0; c < kCols; ++c) cand -= (dA[c] + dF[c]) * L.gamma[c];
            const int solved = L.ok;
            const double cmax = block_max<kSW>(tid < m ? fabs(cand) : 0.0, L.red);
            // a mixed step longer than 3 in log weight is cut to that length (the same cap as the
            // Newton fallback); a failed solve drops the history
            if (solved && cmax < 1e300) stepv = cmax > 3.0 ? cand * (3.0 / cmax) : cand;
            else hcount = 0;
        }
        if (ncol < 1) {                                    // a plain step: the same cap on its length
            const double fmx = block_max<kSW>(tid < m ? fabs(f) : 0.0, L.red);
            if (fmx > 3.0) stepv = f * (3.0 / fmx);
        }
        if (tid < m) L.aal[tid] += stepv;
        ++hcount;
        __syncthreads();
    }
    __syncthreads();
    GR_CLK(L, 12);
    if (result != 0 && mix_iters < max_iter && best_err < 1e300) {
        if (tid < m) L.aal[tid] = L.aBest[tid];
        __syncthreads();
        result = newton_program<D>(L, newton_ws, m, n, ctx, slack, slack_target, qsum, tsum, rel_tol, max_iter, evals);
        GR_CLK(L, 13);
    }
    return result;
}

// Build the active list of one program: the support positions in [lo, hi) that belong to T and have
// a positive target, in decreasing q (L.ordq lists the positions of H* and of the rest in that
// order).  Returns m (possibly > kMaxT, in which case nothing was written beyond kMaxT).
template <class LdsT>
__device__ int compact_active(LdsT& L, int lo, int hi, int kk) {
    const int tid = threadIdx.x;
    const int j = tid < kk ? L.ordq[tid] : -1;           // kk <= KS <= kST
    const int on = (j >= lo && j < hi && L.inT[j] && L.tgt[j] > 0.0) ? 1 : 0;
    // inclusive scan of `on` over the workgroup
    int incl = on;
    for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl, o); if ((tid & 63) >= o) incl += up; }
    int* wtot = reinterpret_cast<int*>(L.red);
    if ((tid & 63) == 63) wtot[tid >> 6] = incl;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < kSW; ++w) { if (w < (tid >> 6)) base += wtot[w]; total += wtot[w]; }
    const int slot = base + incl - 1;
    if (on && slot < kMaxT) L.apos[slot] = j;
    __syncthreads();
    return total;
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kST) void solve_kernel(SolveParams sp) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    Lds<D>& L = *reinterpret_cast<Lds<D>*>(lds_raw);
    const int tid = threadIdx.x;
    const int row = blockIdx.x;
    const int n = sp.n, V = sp.V;
    RowInfo info;
    info.support = 0; info.h = 0; info.status = GR_ROW_OK; info.iterations = 0;
    info.alpha_star = 0.0; info.res_total = 0.0; info.p_total = 0.0; info.q_total = 0.0; info.node_tokens = 0.0;

    // ---- merge the slices
    int total = 0, bad = 0;
    double ptot = 0.0, qtot = 0.0;
    for (int s = 0; s < sp.splits; ++s) {
        total += sp.cand_count[row * sp.splits + s];
        bad |= sp.part_bad[row * sp.splits + s];
        ptot += sp.part_psum[row * sp.splits + s];
        qtot += sp.part_qsum[row * sp.splits + s];
    }
    info.p_total = ptot; info.q_total = qtot;
    if (bad || !(fabs(ptot - 1.0) <= 1e-3) || !(fabs(qtot - 1.0) <= 1e-3) || total <= 0 || total > kSelCap) {
        if (tid == 0) {
            info.status = GR_ROW_BAD;
            info.alpha_star = __longlong_as_double(0x7ff8000000000000ll);
            sp.info[row] = info;
            sp.accept_prob[row] = __uint_as_float(0x7fc00000u);
            sp.status[row] = GR_ROW_BAD;
        }
        return;
    }
    {
        int off = 0;
        for (int s = 0; s < sp.splits; ++s) {
            const int c = sp.cand_count[row * sp.splits + s];
            const unsigned long long* src = sp.cand + (static_cast<size_t>(row) * sp.splits + s) * kMaxSupport;
            for (int i = tid; i < c; i += kST) L.u.keys[off + i] = src[i];
            off += c;
        }
    }
    if (tid == 0) { L.count = 0; L.work = 0.0; }
#ifdef GR_PHASE_CLOCKS
    if (tid == 0) { for (int i = 0; i < 16; ++i) L.clk[i] = 0; L.clk_last = clock64(); }
#endif
    __syncthreads();
    unsigned long long theta = 0ull;
    if (total > sp.k) theta = block_kth_largest<kST>(L.u.keys, total, sp.k, L.hist, L.pick);
    const int kk = min(total, sp.k);
    for (int i = tid; i < total; i += kST) {
        const unsigned long long key = L.u.keys[i];
        if (key >= theta) {
            const int slot = atomicAdd(&L.count, 1);
            if (slot < KS) { L.ordq[slot] = key_id(key); L.accb[slot] = static_cast<double>(key_q(key)); }
        }
    }
    __syncthreads();
    // unsorted: token ids in ordq, q in accb (exact float values), p gathered into G0
    if (tid < kk) L.G0[tid] = static_cast<double>(sp.p[static_cast<size_t>(row) * V + L.ordq[tid]]);
    __syncthreads();
    GR_CLK(L, 0);
    // ---- order by decreasing q/p: exact cross products (float x float fits a double), ties by id.
    // Rank counting; `parts` threads share a token (each counts over a stretch of the others).
    {
        const int parts = kk <= kST / 4 ? 4 : (kk <= kST / 2 ? 2 : 1);
        const int per = kST / parts;                       // tokens a part can hold
        const int me = tid % per, part = tid / per;
        if (tid < kk) L.cnt0[tid] = 0;
        __syncthreads();
        if (me < kk) {
            const double qa = L.accb[me], pa = L.G0[me];
            const int ta = L.ordq[me];
            const int j0 = (kk * part) / parts, j1 = (kk * (part + 1)) / parts;
            int rank = 0;
#pragma unroll 8
            for (int j = j0; j < j1; ++j) {
                const double lhs = L.accb[j] * pa, rhs = qa * L.G0[j];   // j before me?
                rank += static_cast<int>(lhs > rhs) | (static_cast<int>(lhs == rhs) & static_cast<int>(L.ordq[j] < ta));
            }
            if (parts > 1) atomicAdd(&L.cnt0[me], rank); else L.cnt0[me] = rank;
        }
        __syncthreads();
        if (tid < kk) {
            const int rank = L.cnt0[tid];
            const double pa = L.G0[tid];
            L.tok[rank] = L.ordq[tid]; L.qd[rank] = L.accb[tid]; L.pn[rank] = pa / ptot;
        }
        __syncthreads();
    }
    GR_CLK(L, 1);
    // ---- prefix sums in the order, sequentially (bit-reproducible), then F(m) = P_m - Q_m^n
    {
#pragma clang fp contract(off)
        if ((tid >> 6) == 0) wave_sequential_scan(L.pn, L.P, kk, 0.0);
        if ((tid >> 6) == 1) wave_sequential_scan(L.qd, L.S, kk, 0.0);
        __syncthreads();
        const double stot = L.S[kk];
        for (int m = tid; m <= kk; m += kST) {
            const double Qm = L.S[m] / stot;
            L.Q[m] = Qm;
            L.F[m] = (m == 0) ? 0.0 : L.P[m] - ipow(Qm, n);
            if (m < kk) L.qn[m] = L.qd[m] / stot;
        }
        __syncthreads();
    }
    // ---- H*: the smallest minimising prefix
    double fmin_local = 1e300;
    for (int m = tid; m <= kk; m += kST) fmin_local = fmin(fmin_local, L.F[m]);
    const double Fmin = block_min<kSW>(fmin_local, L.red);
    double hcand = 1e9;
    for (int m = tid; m <= kk; m += kST) if (L.F[m] == Fmin) hcand = fmin(hcand, static_cast<double>(m));
    const int h = static_cast<int>(block_min<kSW>(hcand, L.red));
    // ---- G = suffix minima of F (Hillis-Steele over kk+1 entries)
    for (int m = tid; m <= kk; m += kST) L.G0[m] = L.F[m];
    __syncthreads();
    {
        double* src = L.G0; double* dst = L.G1;
        for (int o = 1; o <= kk; o <<= 1) {
            for (int m = tid; m <= kk; m += kST) dst[m] = (m + o <= kk) ? fmin(src[m], src[m + o]) : src[m];
            __syncthreads();
            double* t = src; src = dst; dst = t;
        }
        if (src != L.G0) { for (int m = tid; m <= kk; m += kST) L.G0[m] = src[m]; }
        __syncthreads();
    }
    // residuals, targets, records (F(m) <= G(m+1) for m >= h; m = kk always)
    for (int m = tid; m <= kk; m += kST) {
        L.flag[m] = (m >= h && (m == kk || L.F[m] <= L.G0[m + 1])) ? 1 : 0;
        if (m < kk) {
            const double r = (m >= h) ? L.G0[m + 1] - L.G0[m] : 0.0;
            L.rho[m] = r; L.tgt[m] = L.pn[m] - r;
        }
    }
    __syncthreads();
    // inclusive count of records -> block id of each token outside H*, and block bounds
    for (int m = tid; m <= kk; m += kST) L.cnt0[m] = L.flag[m];
    __syncthreads();
    {
        int* src = L.cnt0; int* dst = L.cnt1;
        for (int o = 1; o <= kk; o <<= 1) {
            for (int m = tid; m <= kk; m += kST) dst[m] = (m >= o) ? src[m] + src[m - o] : src[m];
            __syncthreads();
            int* t = src; src = dst; dst = t;
        }
        if (src != L.cnt0) { for (int m = tid; m <= kk; m += kST) L.cnt0[m] = src[m]; }
        __syncthreads();
    }
    const int nrec = L.cnt0[kk];
    const int nblk = nrec - 1;
    for (int m = tid; m <= kk; m += kST) {
        if (L.flag[m]) L.blo[L.cnt0[m]] = m;             // record number c (1-based) sits at rank m
        if (m < kk) L.blk[m] = (m >= h) ? L.cnt0[m] : 0; // token m (rank m+1) lies after record cnt0[m]
    }
    __syncthreads();
    GR_CLK(L, 2);
    // ---- truncation sets: fewest tokens by decreasing q with gamma_T <= tau / epsilon_T <= tau
    {
        const int parts = kk <= kST / 4 ? 4 : (kk <= kST / 2 ? 2 : 1);
        const int per = kST / parts;
        const int me = tid % per, part = tid / per;
        if (tid < kk) L.cnt1[tid] = 0;
        __syncthreads();
        if (me < kk) {
            const int mine_in = me < h;
            const float qa = static_cast<float>(L.qd[me]);
            const int ta = L.tok[me];
            const int j0 = (kk * part) / parts, j1 = (kk * (part + 1)) / parts;
            int rank = 0;
#pragma unroll 8
            for (int j = j0; j < j1; ++j) {
                const int same = (j < h) == mine_in;
                const float qj = static_cast<float>(L.qd[j]);
                rank += same & (static_cast<int>(qj > qa) | (static_cast<int>(qj == qa) & static_cast<int>(L.tok[j] < ta)));
            }
            if (parts > 1) atomicAdd(&L.cnt1[me], rank); else L.cnt1[me] = rank;
        }
        __syncthreads();
        if (tid < kk) L.ordq[(tid < h ? 0 : h) + L.cnt1[tid]] = tid;
    }
    __syncthreads();
    const double Qh = L.Q[h];
    {
#pragma clang fp contract(off)
        // running q mass in decreasing-q order: G0 <- q in that order, G1 <- its sequential prefix sums
        if (tid < kk) L.G0[tid] = L.qn[L.ordq[tid]];
        __syncthreads();
        if ((tid >> 6) == 0) wave_sequential_scan(L.G0, L.G1, h, 0.0);
        if ((tid >> 6) == 1) wave_sequential_scan(L.G0 + h, L.G1 + h + 1, kk - h, Qh);
        __syncthreads();
        if (tid < kk) L.accb[L.ordq[tid]] = L.G1[tid < h ? tid : tid + 1];
        __syncthreads();
        if (tid < kk) {
            const double a = L.accb[tid];
            const double an = (a > 0.0) ? ipow(a, n) : 0.0;
            L.inT[tid] = (tid < h) ? ((ipow(Qh, n) - an) > sp.tau) : ((1.0 - an) > sp.tau);
        }
    }
    // ---- start weights: target / Pr[token drawn within its system], inner ones in the slack's gauge
    if (tid < kk) {
        const int hi = (tid < h) ? h : L.blo[L.blk[tid] + 1];
        const double top = L.Q[hi];
        const double gauge = (tid < h) ? ipow(top, n) / (-L.F[h]) : 1.0;
        const double t = L.tgt[tid];
        L.wgt[tid] = (t > 0.0) ? gauge * t / pow_diff(top, L.qn[tid], n) : 0.0;
    }
    __syncthreads();

    GR_CLK(L, 3);
    // ---- the convex programs: program 0 = inner system, then every outer block of two or more tokens
    int status = GR_ROW_OK, evals = 0;
    for (int b = (h > 0 ? 0 : 1); b <= nblk && status != GR_ROW_TRUNC_CAP; ++b) {
        const int lo = (b == 0) ? 0 : L.blo[b];
        const int hi = (b == 0) ? h : L.blo[b + 1];
        if (b > 0 && hi - lo < 2) continue;
        const int m = compact_active(L, lo, hi, kk);
        if (m > sp.max_T) { status = GR_ROW_TRUNC_CAP; break; }
        if (m == 0 || (b > 0 && m < 2)) continue;
        if (tid < m) {
            const int j = L.apos[tid];
            L.aq[tid] = L.qn[j]; L.at[tid] = L.tgt[j]; L.aal[tid] = log(L.wgt[j]);
        }
        __syncthreads();
        const double qa = block_sum<kSW>(tid < m ? L.aq[tid] : 0.0, L.red);
        const double ta = block_sum<kSW>(tid < m ? L.at[tid] : 0.0, L.red);
        double ctx, scale, slack_target = 0.0;
        if (b == 0) {
            // context = tokens of T with target 0 (weight 0): they fill tuples but take no mass
            const int j = tid;
            ctx = block_sum<kSW>((j < h && L.inT[j] && !(L.tgt[j] > 0.0)) ? L.qn[j] : 0.0, L.red);
            const double mass = ipow(ctx + qa, n);
            scale = mass / (ta - L.F[h]);
            slack_target = -L.F[h] * scale;
        } else {
            ctx = L.Q[lo];
            scale = pow_diff(ctx + qa, qa, n) / ta;
        }
        const double w0sum = block_sum<kSW>(tid < m ? L.wgt[L.apos[tid]] : 0.0, L.red);
        if (tid < m) L.at[tid] *= scale;
        __syncthreads();
        GR_CLK(L, 4);
        const int rc = solve_program<D>(L, sp.newton_ws + static_cast<size_t>(row) * kMaxT * (kMaxT + 1), m, n, ctx, b == 0, slack_target, sp.rel_tol, sp.max_iter, &evals);
        if (rc != 0 && status == GR_ROW_OK) status = GR_ROW_ITER_CAP;
        const double wv = (tid < m) ? exp(L.aal[tid]) : 0.0;
        const double wsum = block_sum<kSW>(wv, L.red);
        if (tid < m) L.wgt[L.apos[tid]] = (b == 0) ? wv : wv * (w0sum / wsum);
        __syncthreads();
    }

    // ---- policy object
    int* o_order = sp.order + static_cast<size_t>(row) * KS;
    int* o_block = sp.block + static_cast<size_t>(row) * KS;
    double* o_w = sp.weight + static_cast<size_t>(row) * KS;
    double* o_rho = sp.rho + static_cast<size_t>(row) * KS;
    double* o_pn = sp.pnorm + static_cast<size_t>(row) * KS;
    if (tid < kk) {
        o_order[tid] = L.tok[tid]; o_block[tid] = L.blk[tid]; o_w[tid] = L.wgt[tid];
        o_rho[tid] = L.rho[tid]; o_pn[tid] = L.pn[tid];
    }
    if (tid == 0) {
        info.support = kk; info.h = h; info.status = status; info.iterations = evals;
        info.alpha_star = 1.0 + L.F[h];
        info.res_total = -L.F[h];
        info.node_tokens = L.work;
#ifdef GR_PHASE_CLOCKS
        { const long long now_ = clock64(); L.clk[14] += now_ - L.clk_last; for (int i = 0; i < 16; ++i) info.clk[i] = L.clk[i]; }
#endif
        sp.info[row] = info;
        sp.accept_prob[row] = static_cast<float>(1.0 + L.F[h]);
        sp.status[row] = status;
    }
}

// ---- full-vocabulary policies: the convex programs of a row whose steps 1-2 were done in HBM.
// Start weights of every support token, the dense per-token arrays the verify kernel reads, then the
// inner program over T inside H* and one outer program per block that holds two or more active
// tokens of T -- the same programs, in the same arithmetic, as the LDS-resident path.
template <int D>
__global__ __launch_bounds__(kST) void full_programs_kernel(FullParams fp) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    Lds<D>& L = *reinterpret_cast<Lds<D>*>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, row = blockIdx.x;
    const int n = fp.n, V = fp.V;
    const size_t vs = static_cast<size_t>(V) + 2;
    RowInfo info = fp.info[row];
    if (info.status == GR_ROW_BAD) return;
    const int kk = info.support, h = info.h;
    const float* pr = fp.p + static_cast<size_t>(row) * V;
    const int* order = fp.order + row * vs; const int* byq = fp.byq + row * vs;
    const double* qn = fp.qn + row * vs; const double* Q = fp.Q + row * vs; const double* F = fp.F + row * vs;
    const double* rho = fp.rho + row * vs; const double* tgt = fp.tgt + row * vs;
    const int* blk = fp.blk + row * vs; const int* blo = fp.blo + row * vs; const int* inT = fp.inT + row * vs;
    const int* bcount = fp.bcount + row * vs;
    double* weight = fp.weight + row * vs; double* rho_id = fp.rho_id + row * vs; int* rank_of = fp.rank_of + row * vs;
    const double Fh = F[h];

    // tokens outside the support keep all of p as residual; then the support by rank
    for (int i = tid; i < V; i += kST) { rank_of[i] = -1; rho_id[i] = static_cast<double>(pr[i]) / info.p_total; }
    __syncthreads();
    for (int r0 = tid; r0 < kk; r0 += 4 * kST) {             // four independent chains of gathers per thread in flight
        int bl[4], hi[4], id[4]; double top[4], t[4], qv[4], rv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = r0 + j * kST;
            const bool ok = r < kk;
            bl[j] = (ok && r >= h) ? blk[r] : 0;
            t[j] = ok ? tgt[r] : 0.0; qv[j] = ok ? qn[r] : 0.0; rv[j] = ok ? rho[r] : 0.0; id[j] = ok ? order[r] : 0;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) { const int r = r0 + j * kST; hi[j] = (r < h || r >= kk) ? h : blo[bl[j] + 1]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) top[j] = Q[hi[j]];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = r0 + j * kST;
            if (r < kk) {
                const double gauge = (r < h) ? ipow(top[j], n) / (-Fh) : 1.0;
                weight[r] = (t[j] > 0.0) ? gauge * t[j] / pow_diff(top[j], qv[j], n) : 0.0;
                rank_of[id[j]] = r; rho_id[id[j]] = rv[j];
            }
        }
    }
    if (info.status != GR_ROW_OK) return;
    if (tid == 0) L.work = 0.0;
    __syncthreads();

    int status = GR_ROW_OK, evals = 0;
    // ---- inner program: T inside H* is the first tcount[0] entries of byq, already by decreasing q
    if (h > 0) {
        const int c_in = fp.tcount[2 * row];
        int m = 0;
        double ctx_part = 0.0;
        for (int base = 0; base < c_in; base += kST) {
            const int i = base + tid;
            const int r = i < c_in ? byq[i] : -1;
            const double t = r >= 0 ? tgt[r] : 0.0;
            const bool on = r >= 0 && t > 0.0;
            if (r >= 0 && !on) ctx_part += qn[r];
            const unsigned long long mask = __ballot(on);
            if (lane == 0) L.hist[wv] = __popcll(mask);
            __syncthreads();
            int slot = m + __popcll(mask & ((1ull << lane) - 1ull));
            int tile_total = 0;
            for (int w = 0; w < kSW; ++w) { if (w < wv) slot += L.hist[w]; tile_total += L.hist[w]; }
            if (on && slot < kMaxT) { L.apos[slot] = r; L.aq[slot] = qn[r]; L.at[slot] = t; L.aal[slot] = log(weight[r]); }
            m += tile_total;
            __syncthreads();
        }
        const double ctx = block_sum<kSW>(ctx_part, L.red);
        if (m > 0 && m <= kMaxT) {
            const double qa = block_sum<kSW>(tid < m ? L.aq[tid] : 0.0, L.red);
            const double ta = block_sum<kSW>(tid < m ? L.at[tid] : 0.0, L.red);
            const double mass = ipow(ctx + qa, n);
            const double scale = mass / (ta - Fh);
            const double slack_target = -Fh * scale;
            if (tid < m) L.at[tid] *= scale;
            __syncthreads();
            const int rc = solve_program<D>(L, fp.newton_ws + static_cast<size_t>(row) * kMaxT * (kMaxT + 1), m, n, ctx, 1, slack_target, fp.rel_tol, fp.max_iter, &evals);
            if (rc != 0) status = GR_ROW_ITER_CAP;
            if (tid < m) weight[L.apos[tid]] = exp(L.aal[tid]);
            __syncthreads();
        }
    }
    // ---- outer programs: windows of kST blocks, those with two or more active tokens of T
    const int nblk = fp.nblk[row];
    for (int b0 = 1; b0 <= nblk; b0 += kST) {
        const int bme = b0 + tid;
        const bool need = bme <= nblk && bcount[bme] >= 2;
        const unsigned long long nmask = __ballot(need);
        if (lane == 0) L.hist[wv] = __popcll(nmask);
        __syncthreads();
        int pslot = __popcll(nmask & ((1ull << lane) - 1ull));
        int nprog = 0;
        for (int w = 0; w < kSW; ++w) { if (w < wv) pslot += L.hist[w]; nprog += L.hist[w]; }
        if (need) L.flag[pslot] = bme;                      // nprog <= kST <= KS + 2
        __syncthreads();
        for (int pi = 0; pi < nprog; ++pi) {
            const int b = L.flag[pi];
            const int lo = blo[b], hi = blo[b + 1];
            // active tokens of the block, by rank
            int m = 0;
            for (int base = lo; base < hi; base += kST) {
                const int r = base + tid;
                const bool on = r < hi && inT[r] && tgt[r] > 0.0;
                const unsigned long long mask = __ballot(on);
                if (lane == 0) L.hist[wv] = __popcll(mask);
                __syncthreads();
                int slot = m + __popcll(mask & ((1ull << lane) - 1ull));
                int tile_total = 0;
                for (int w = 0; w < kSW; ++w) { if (w < wv) slot += L.hist[w]; tile_total += L.hist[w]; }
                if (on && slot < kMaxT) { L.adeg[slot] = r; L.af[slot] = qn[r]; L.aR[slot] = tgt[r]; L.aw[slot] = log(weight[r]); }
                m += tile_total;
                __syncthreads();
            }
            if (m < 2 || m > kMaxT) continue;               // cannot happen for a row with status OK
            // by decreasing q (the evaluator takes its heavy tokens first), ties by rank
            if (tid < m) {
                const double qa = L.af[tid];
                int pos = 0;
                for (int j = 0; j < m; ++j) pos += (L.af[j] > qa) || (L.af[j] == qa && j < tid);
                L.apos[pos] = L.adeg[tid]; L.aq[pos] = qa; L.at[pos] = L.aR[tid]; L.aal[pos] = L.aw[tid];
            }
            __syncthreads();
            const double qa = block_sum<kSW>(tid < m ? L.aq[tid] : 0.0, L.red);
            const double ta = block_sum<kSW>(tid < m ? L.at[tid] : 0.0, L.red);
            const double ctx = Q[lo];
            const double scale = pow_diff(ctx + qa, qa, n) / ta;
            const double w0sum = block_sum<kSW>(tid < m ? exp(L.aal[tid]) : 0.0, L.red);
            if (tid < m) L.at[tid] *= scale;
            __syncthreads();
            const int rc = solve_program<D>(L, fp.newton_ws + static_cast<size_t>(row) * kMaxT * (kMaxT + 1), m, n, ctx, 0, 0.0, fp.rel_tol, fp.max_iter, &evals);
            if (rc != 0 && status == GR_ROW_OK) status = GR_ROW_ITER_CAP;
            const double wvv = (tid < m) ? exp(L.aal[tid]) : 0.0;
            const double wsum = block_sum<kSW>(wvv, L.red);
            if (tid < m) weight[L.apos[tid]] = wvv * (w0sum / wsum);
            __syncthreads();
        }
        __syncthreads();
    }
    if (tid == 0) {
        info.status = status; info.iterations = evals; info.node_tokens = L.work;
        fp.info[row] = info;
        fp.status[row] = status;
    }
}

hipError_t launch_full_programs(const FullParams& fp, hipStream_t stream) {
    const dim3 grid(fp.B), block(kST);
    if (fp.n <= 2) hipLaunchKernelGGL(full_programs_kernel<2>, grid, block, sizeof(Lds<2>), stream, fp);
    else if (fp.n <= 4) hipLaunchKernelGGL(full_programs_kernel<4>, grid, block, sizeof(Lds<4>), stream, fp);
    else if (fp.n <= 8) hipLaunchKernelGGL(full_programs_kernel<8>, grid, block, sizeof(Lds<8>), stream, fp);
    else hipLaunchKernelGGL(full_programs_kernel<16>, grid, block, sizeof(Lds<16>), stream, fp);
    return hipGetLastError();
}

static_assert(sizeof(Lds<16>) + 20 * 1024 <= 160 * 1024,
              "the solve workgroup's state and one streaming workgroup of the next batch must fit the CU's LDS together");

hipError_t solve_kernel_setup() {
    const void* kernels[8] = {reinterpret_cast<const void*>(solve_kernel<2>), reinterpret_cast<const void*>(solve_kernel<4>),
                              reinterpret_cast<const void*>(solve_kernel<8>), reinterpret_cast<const void*>(solve_kernel<16>),
                              reinterpret_cast<const void*>(full_programs_kernel<2>), reinterpret_cast<const void*>(full_programs_kernel<4>),
                              reinterpret_cast<const void*>(full_programs_kernel<8>), reinterpret_cast<const void*>(full_programs_kernel<16>)};
    const size_t sizes[8] = {sizeof(Lds<2>), sizeof(Lds<4>), sizeof(Lds<8>), sizeof(Lds<16>),
                             sizeof(Lds<2>), sizeof(Lds<4>), sizeof(Lds<8>), sizeof(Lds<16>)};
    for (int i = 0; i < 8; ++i) {
        const hipError_t e = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizes[i]));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// One kernel per series degree D >= n (2, 4, 8, 16), so that each keeps its series in registers.
hipError_t launch_solve(const SolveParams& sp, hipStream_t stream) {
    const dim3 grid(sp.B), block(kST);
    if (sp.n <= 2) hipLaunchKernelGGL(solve_kernel<2>, grid, block, sizeof(Lds<2>), stream, sp);
    else if (sp.n <= 4) hipLaunchKernelGGL(solve_kernel<4>, grid, block, sizeof(Lds<4>), stream, sp);
    else if (sp.n <= 8) hipLaunchKernelGGL(solve_kernel<8>, grid, block, sizeof(Lds<8>), stream, sp);
    else hipLaunchKernelGGL(solve_kernel<16>, grid, block, sizeof(Lds<16>), stream, sp);
    return hipGetLastError();
}

}  // namespace gr
